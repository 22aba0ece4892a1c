/*
 * CPU oracle of the batch-decode MoE layer with and without SERE re-routing.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the layer computes, written from the paper; the tests compare the HIP
 * library against it.  It shares no code with the HIP library, and nothing in
 * the product path may call it.
 *
 * Arithmetic: every floating-point step is IEEE double on the exact stored
 * input bits (fp32, or bf16 carried as uint16); sums run in ascending index
 * order.  Indices are 0-based.  The OpenMP pragmas only spread *independent*
 * outer iterations (tokens, experts) over threads; no sum is split.
 *
 * What each function follows:
 *   router logits, top-k, gate      appendix "Preliminaries on MoEs" (router
 *                                   logits R(x), top-k gating equation) and
 *                                   the ordered list R(t) of Sec. 3.2.2
 *   expert FFN, layer output        appendix "Preliminaries on MoEs", the
 *                                   layer-output and expert equations
 *   primary mask                    Sec. 3.2.2 Step 1 (primary-set equation)
 *   re-route, per assignment        the appendix algorithm "CUDA-accelerated
 *                                   SERE", followed step by step
 *   re-route, per expert (sets)     Sec. 3.2.2 Steps 2-3 (arg-max, re-routing
 *                                   condition and final-set equations)
 *   compaction                      Sec. 3.2.2 Step 3: the updated
 *                                   token-to-expert mapping, listed per expert
 *   Frobenius similarity matrix     Sec. 3.1.1 accumulation equation, the
 *                                   appendix "Frobenius Similarity" and the
 *                                   appendix algorithm "Expert Similarity
 *                                   Estimation"
 *   cosine similarity matrix        the same, with the appendix "Cosine
 *                                   Similarity"
 *
 * Readings taken where the paper leaves a choice (all listed in the design
 * notes of this repository):
 *   - the gate is a softmax over the K selected logits;
 *   - equal logits / equal similarities: the lower expert index wins;
 *   - rho <= 0 disables the threshold test (the algorithm's rule), and
 *     sim* == rho re-routes (kept only when strictly below);
 *   - sim[u][v]: row u is the secondary expert, column v the candidate;
 *   - re-routing never changes gate weights, never merges or drops a slot;
 *   - the activation is SiLU;
 *   - shared experts see every token with weight 1 and are outside routing;
 *   - the Frobenius maximum is taken per calibration batch over all pairs;
 *     the diagonal accumulates Sim(A_p, A_p) = 1 once per batch (the
 *     accumulation equation), not twice.
 *
 * Parity unpinned: the numerical value of a layer output on random data has
 * no printed reference in the paper; it is pinned by closed forms, by an
 * fp64 library matmul formulation and by a brute-force second implementation
 * in the tests, not by published numbers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

/* exact widening of element i of a stored tensor */
static inline double load_elem(const void *p, int dtype, size_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[i];
    uint32_t w = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static inline const void *elem_ptr(const void *p, int dtype, size_t i)
{
    return (const char *)p + i * (dtype == ORACLE_F32 ? 4 : 2);
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* logit[t][e] = <x_t, Wr_e>  (router logits R(x)) */
void oracle_router_logits(const void *hidden, const void *router_w, int dtype,
                          int T, int M, int dh, double *logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < M; ++e) {
            double acc = 0.0;
            for (int i = 0; i < dh; ++i)
                acc += load_elem(hidden, dtype, (size_t)t * dh + i) *
                       load_elem(router_w, dtype, (size_t)e * dh + i);
            logits[(size_t)t * M + e] = acc;
        }
}

/*
 * Ordered list r_1..r_K of each token by descending logit (equal logits:
 * lower index first) and the gate P = softmax over the K selected logits.
 * min_gap (may be NULL) receives the smallest difference between adjacent
 * ranks 1..K+1 over all tokens: how far the ordering is from ambiguous.
 */
void oracle_topk_gate(const double *logits, int T, int M, int K,
                      int32_t *ids, double *weights, double *min_gap)
{
    double gap = INFINITY;
    char *taken = (char *)malloc((size_t)M);
    for (int t = 0; t < T; ++t) {
        const double *l = logits + (size_t)t * M;
        memset(taken, 0, (size_t)M);
        double prev = 0.0;
        for (int k = 0; k <= K && k < M; ++k) {
            int best = -1;
            for (int e = 0; e < M; ++e)
                if (!taken[e] && (best < 0 || l[e] > l[best]))
                    best = e;              /* strict '>' keeps the lower index */
            if (k > 0 && prev - l[best] < gap)
                gap = prev - l[best];
            prev = l[best];
            if (k < K) {
                taken[best] = 1;
                ids[(size_t)t * K + k] = best;
            }
        }
        double top = l[ids[(size_t)t * K]];
        double denom = 0.0;
        for (int k = 0; k < K; ++k)
            denom += exp(l[ids[(size_t)t * K + k]] - top);
        for (int k = 0; k < K; ++k)
            weights[(size_t)t * K + k] = exp(l[ids[(size_t)t * K + k]] - top) / denom;
    }
    free(taken);
    if (min_gap)
        *min_gap = gap;
}

/* H[e] = 1 iff e is among the first S experts of some token (primary set) */
void oracle_primary_mask(const int32_t *ids, int T, int K, int S, int M, int32_t *H)
{
    for (int e = 0; e < M; ++e)
        H[e] = 0;
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < S; ++s)
            H[ids[(size_t)t * K + s]] = 1;
}

/*
 * Row `row` = similarities of one expert to all M experts.  Visits the experts
 * marked in `primary` in ascending index; a later one displaces the current
 * choice only when it is strictly more similar (so equal similarities go to
 * the lower index).  With no marked expert, or none whose similarity exceeds
 * the value passed in, *choice and *value stay as the caller set them.
 */
static void most_similar_primary(const float *row, const int32_t *primary, int M,
                                 int *choice, float *value)
{
    for (int v = 0; v < M; ++v) {
        if (!primary[v])
            continue;
        if (row[v] > *value) {
            *value = row[v];
            *choice = v;
        }
    }
}

/*
 * Re-routing seen from the slots (Sec. 3.2.2 Steps 1-2 and the appendix
 * algorithm's contract: top-K indices in, indices out).  Every slot of rank
 * >= S whose expert is in nobody's top-S gets the most similar primary in its
 * place, unless the threshold test is on (rho > 0) and that similarity is
 * below rho.  The search starts from (-inf, expert 0), which is also its
 * result when no similarity is above -inf.
 */
void oracle_reroute_per_slot(const int32_t *ids, const float *sim, int T, int K,
                             int M, int S, float rho, int32_t *ids_out)
{
    int32_t *primary = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
    oracle_primary_mask(ids, T, K, S, M, primary);
    const int threshold_on = rho > 0.0f;
    for (size_t slot = 0; slot < (size_t)T * K; ++slot) {
        const int rank = (int)(slot % (size_t)K);
        const int u = ids[slot];
        ids_out[slot] = u;
        if (rank < S || primary[u])
            continue;                    /* top-S slot, or retained by some token */
        int v = 0;
        float closeness = -INFINITY;
        most_similar_primary(sim + (size_t)u * M, primary, M, &v, &closeness);
        const int critical = threshold_on && closeness < rho;
        if (!critical)
            ids_out[slot] = v;
    }
    free(primary);
}

/*
 * Re-routing from the set equations: U = activated experts outside the
 * primary set; for each u in U the most similar primary v*_u and sim*_u;
 * every occurrence of u in a secondary slot becomes v*_u when the re-routing
 * condition holds; final set = primary set plus the preserved (critical) u.
 * target[u] = v*_u for u in U, else -1; sim_star[u] likewise (else 0);
 * final_set[e] in {0,1}.
 */
void oracle_reroute_sets(const int32_t *ids, const float *sim, int T, int K,
                         int M, int S, float rho, int32_t *ids_out,
                         int32_t *final_set, int32_t *target, float *sim_star)
{
    int32_t *H = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
    char *activated = (char *)calloc((size_t)M, 1);
    oracle_primary_mask(ids, T, K, S, M, H);
    for (size_t a = 0; a < (size_t)T * K; ++a)
        activated[ids[a]] = 1;
    for (int u = 0; u < M; ++u) {
        target[u] = -1;
        sim_star[u] = 0.0f;
        final_set[u] = H[u];
        if (!activated[u] || H[u])
            continue;
        int v_star = -1;
        for (int v = 0; v < M; ++v)
            if (H[v] && (v_star < 0 || sim[(size_t)u * M + v] > sim[(size_t)u * M + v_star]))
                v_star = v;
        target[u] = v_star;
        sim_star[u] = sim[(size_t)u * M + v_star];
        if (rho > 0.0f && sim_star[u] < rho)
            final_set[u] = 1;           /* critical expert: preserved */
    }
    for (int t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            int u = ids[(size_t)t * K + k];
            int out = u;
            if (k >= S && target[u] >= 0 && !final_set[u])
                out = target[u];
            ids_out[(size_t)t * K + k] = out;
        }
    free(H);
    free(activated);
}

/*
 * The token-to-expert mapping listed per expert: count[e] slots, exclusive
 * prefix offsets[M+1], and the (token, slot) pairs of expert e at
 * [offsets[e], offsets[e+1]) in ascending (token, slot).  n_active = number
 * of experts with a non-zero count.
 */
void oracle_compact(const int32_t *ids, int T, int K, int M, int32_t *count,
                    int32_t *offsets, int32_t *sorted_token,
                    int32_t *sorted_slot, int32_t *n_active)
{
    for (int e = 0; e < M; ++e)
        count[e] = 0;
    for (size_t a = 0; a < (size_t)T * K; ++a)
        count[ids[a]]++;
    offsets[0] = 0;
    int active = 0;
    for (int e = 0; e < M; ++e) {
        offsets[e + 1] = offsets[e] + count[e];
        active += count[e] > 0;
    }
    for (int e = 0; e < M; ++e) {
        int pos = offsets[e];
        for (int t = 0; t < T; ++t)
            for (int k = 0; k < K; ++k)
                if (ids[(size_t)t * K + k] == e) {
                    sorted_token[pos] = t;
                    sorted_slot[pos] = k;
                    ++pos;
                }
    }
    *n_active = active;
}

static double silu(double z)
{
    return z / (1.0 + exp(-z));
}

/*
 * One expert on one token: y = W_down (silu(W_gate x) * (W_up x)).
 * w_gate_up is [2*dm][dh] (rows 0..dm-1 gate, dm..2dm-1 up), w_down [dh][dm].
 * scratch holds dm doubles.
 */
static void expert_ffn(const void *x, const void *w_gate_up, const void *w_down,
                       int dtype, int dh, int dm, double *scratch, double *y)
{
    for (int j = 0; j < dm; ++j) {
        double g = 0.0, u = 0.0;
        for (int i = 0; i < dh; ++i) {
            double xi = load_elem(x, dtype, (size_t)i);
            g += load_elem(w_gate_up, dtype, (size_t)j * dh + i) * xi;
            u += load_elem(w_gate_up, dtype, (size_t)(dm + j) * dh + i) * xi;
        }
        scratch[j] = silu(g) * u;
    }
    for (int r = 0; r < dh; ++r) {
        double acc = 0.0;
        for (int j = 0; j < dm; ++j)
            acc += load_elem(w_down, dtype, (size_t)r * dm + j) * scratch[j];
        y[r] = acc;
    }
}

void oracle_expert_ffn(const void *x, const void *w_gate_up, const void *w_down,
                       int dtype, int dh, int dm, double *y)
{
    double *scratch = (double *)malloc(sizeof(double) * (size_t)dm);
    expert_ffn(x, w_gate_up, w_down, dtype, dh, dm, scratch, y);
    free(scratch);
}

/*
 * Layer output for a given token-to-expert map:
 *   out[t] = sum_k weights[t][k] * E_{ids[t][k]}(x_t) + sum_s Eshared_s(x_t)
 * (slot order k ascending, then shared experts).  With ids = the router's
 * top-k this is the standard top-k MoE layer; with ids = the re-routed map it
 * is the SERE layer (same weights).
 */
void oracle_moe_layer(const void *hidden, const void *w_gate_up, const void *w_down,
                      const void *shared_gate_up, const void *shared_down,
                      int dtype, int T, int dh, int M, int K, int dm, int n_sh,
                      const int32_t *ids, const double *weights, double *out)
{
    (void)M;
    size_t gu = (size_t)2 * dm * dh, dn = (size_t)dh * dm;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)dm);
        double *y = (double *)malloc(sizeof(double) * (size_t)dh);
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < T; ++t) {
            const void *x = elem_ptr(hidden, dtype, (size_t)t * dh);
            double *o = out + (size_t)t * dh;
            for (int r = 0; r < dh; ++r)
                o[r] = 0.0;
            for (int k = 0; k < K; ++k) {
                int e = ids[(size_t)t * K + k];
                expert_ffn(x, elem_ptr(w_gate_up, dtype, (size_t)e * gu),
                           elem_ptr(w_down, dtype, (size_t)e * dn), dtype, dh, dm,
                           scratch, y);
                double w = weights[(size_t)t * K + k];
                for (int r = 0; r < dh; ++r)
                    o[r] += w * y[r];
            }
            for (int s = 0; s < n_sh; ++s) {
                expert_ffn(x, elem_ptr(shared_gate_up, dtype, (size_t)s * gu),
                           elem_ptr(shared_down, dtype, (size_t)s * dn), dtype, dh, dm,
                           scratch, y);
                for (int r = 0; r < dh; ++r)
                    o[r] += y[r];
            }
        }
        free(scratch);
        free(y);
    }
}

/*
 * Expert-similarity matrix with the Frobenius metric.  For each of the N
 * calibration batches X_i [n][dh]: A_j = E_j(X_i) for all M experts;
 * x_pq = ||A_p - A_q||_F; Sim(p,q) = 1 - x_pq / max over all pairs of that
 * batch; S[p][q] += Sim(p,q).  Finally S /= N.  act is caller scratch of
 * M*n*dh doubles.  If every pair of a batch is identical (max = 0) that
 * batch contributes Sim = 1 everywhere.
 */
void oracle_similarity_frobenius(const void *calib, const void *w_gate_up,
                                 const void *w_down, int dtype, int N, int n,
                                 int dh, int M, int dm, double *act, double *sim)
{
    size_t gu = (size_t)2 * dm * dh, dn = (size_t)dh * dm;
    double *dist = (double *)malloc(sizeof(double) * (size_t)M * M);
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] = 0.0;
    for (int b = 0; b < N; ++b) {
#pragma omp parallel
        {
            double *scratch = (double *)malloc(sizeof(double) * (size_t)dm);
#pragma omp for schedule(dynamic, 1) collapse(2)
            for (int j = 0; j < M; ++j)
                for (int r = 0; r < n; ++r)
                    expert_ffn(elem_ptr(calib, dtype, ((size_t)b * n + r) * dh),
                               elem_ptr(w_gate_up, dtype, (size_t)j * gu),
                               elem_ptr(w_down, dtype, (size_t)j * dn), dtype, dh, dm,
                               scratch, act + ((size_t)j * n + r) * dh);
            free(scratch);
        }
        double max_dist = 0.0;
#pragma omp parallel for schedule(dynamic, 1)
        for (int p = 0; p < M; ++p)
            for (int q = 0; q < M; ++q) {
                double ss = 0.0;
                for (size_t i = 0; i < (size_t)n * dh; ++i) {
                    double d = act[(size_t)p * n * dh + i] - act[(size_t)q * n * dh + i];
                    ss += d * d;
                }
                dist[(size_t)p * M + q] = sqrt(ss);
            }
        for (size_t i = 0; i < (size_t)M * M; ++i)
            if (dist[i] > max_dist)
                max_dist = dist[i];
        for (size_t i = 0; i < (size_t)M * M; ++i)
            sim[i] += max_dist > 0.0 ? 1.0 - dist[i] / max_dist : 1.0;
    }
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] /= (double)N;
    free(dist);
}

/*
 * Expert-similarity matrix with the cosine metric (appendix "Cosine
 * Similarity"): for each calibration batch, Sim(p,q) = (1/n) sum over the n
 * tokens of <A_p[i], A_q[i]> / (||A_p[i]|| ||A_q[i]||), A_j = E_j(X) as above;
 * S[p][q] += Sim(p,q) per batch, finally S /= N (Sec. 3.1.1).  A token for
 * which either output is the zero vector contributes 0 (the quotient is
 * undefined there; reading of this build).  act is caller scratch of M*n*dh
 * doubles.
 */
void oracle_similarity_cosine(const void *calib, const void *w_gate_up, const void *w_down,
                              int dtype, int N, int n, int dh, int M, int dm, double *act,
                              double *sim)
{
    size_t gu = (size_t)2 * dm * dh, dn = (size_t)dh * dm;
    double *norm = (double *)malloc(sizeof(double) * (size_t)M * n);
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] = 0.0;
    for (int b = 0; b < N; ++b) {
#pragma omp parallel
        {
            double *scratch = (double *)malloc(sizeof(double) * (size_t)dm);
#pragma omp for schedule(dynamic, 1) collapse(2)
            for (int j = 0; j < M; ++j)
                for (int r = 0; r < n; ++r)
                    expert_ffn(elem_ptr(calib, dtype, ((size_t)b * n + r) * dh),
                               elem_ptr(w_gate_up, dtype, (size_t)j * gu),
                               elem_ptr(w_down, dtype, (size_t)j * dn), dtype, dh, dm,
                               scratch, act + ((size_t)j * n + r) * dh);
            free(scratch);
        }
        for (int j = 0; j < M; ++j)
            for (int r = 0; r < n; ++r) {
                const double *a = act + ((size_t)j * n + r) * dh;
                double ss = 0.0;
                for (int c = 0; c < dh; ++c)
                    ss += a[c] * a[c];
                norm[(size_t)j * n + r] = sqrt(ss);
            }
#pragma omp parallel for schedule(dynamic, 1)
        for (int p = 0; p < M; ++p)
            for (int q = 0; q < M; ++q) {
                double total = 0.0;
                for (int r = 0; r < n; ++r) {
                    const double *a = act + ((size_t)p * n + r) * dh;
                    const double *c = act + ((size_t)q * n + r) * dh;
                    double dot = 0.0;
                    for (int k = 0; k < dh; ++k)
                        dot += a[k] * c[k];
                    double den = norm[(size_t)p * n + r] * norm[(size_t)q * n + r];
                    if (den > 0.0)
                        total += dot / den;
                }
                sim[(size_t)p * M + q] += total / (double)n;
            }
    }
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] = sim[i] / (double)N;
    free(norm);
}

/*
 * Expert-similarity matrix with linear-kernel CKA (appendix "Centered Kernel
 * Alignment"): for each calibration batch and expert j the n x n Gram matrix
 * K_j = A_j A_j^T of its outputs A_j = E_j(X) [n][dh];
 *   CKA(p,q) = HSIC(K_p,K_q) / sqrt(HSIC(K_p,K_p) HSIC(K_q,K_q)),
 * with the unbiased estimator of HSIC (the appendix names it and refers to the
 * literature for the formula; reading of this build: the estimator of Song et
 * al. 2012, the one minibatch CKA uses): with Kt, Lt = K, L with their
 * diagonals set to zero and 1 the all-ones vector,
 *   HSIC(K,L) = [ tr(Kt Lt) + (1'Kt1)(1'Lt1)/((n-1)(n-2)) - 2 (1'Kt Lt 1)/(n-2) ]
 *               / (n (n-3)),                                   n >= 4.
 * S[p][q] += CKA(p,q) per batch, finally S /= N (Sec. 3.1.1).  If either
 * self-term is not positive the quotient is undefined and the pair contributes
 * 0 (reading of this build).  act: caller scratch of M*n*dh doubles; gram:
 * caller scratch of M*n*n doubles.
 */
static double hsic_unbiased(const double *Kt, const double *Lt, int n)
{
    double tr = 0.0, sk = 0.0, sl = 0.0, cross = 0.0;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            tr += Kt[(size_t)i * n + j] * Lt[(size_t)j * n + i];
            sk += Kt[(size_t)i * n + j];
            sl += Lt[(size_t)i * n + j];
        }
    for (int j = 0; j < n; ++j) {
        double col_k = 0.0, row_l = 0.0; /* (1'Kt)_j and (Lt 1)_j */
        for (int i = 0; i < n; ++i) {
            col_k += Kt[(size_t)i * n + j];
            row_l += Lt[(size_t)j * n + i];
        }
        cross += col_k * row_l;
    }
    double dn = (double)n;
    return (tr + sk * sl / ((dn - 1.0) * (dn - 2.0)) - 2.0 * cross / (dn - 2.0)) / (dn * (dn - 3.0));
}

/*
 * One entry of a Gram matrix for the three kernels of the appendix "Centered
 * Kernel Alignment", x and y being two rows of an expert's outputs:
 *   kernel 0, linear:      <x, y>
 *   kernel 1, RBF:         exp(-||x - y||^2 / (2 sigma^2)),  sigma = p0
 *   kernel 2, polynomial:  (<x, y> + c)^d,  c = p0, d = p1 (a positive integer)
 */
static double cka_kernel_value(const double *x, const double *y, int dh, int kernel, double p0,
                               double p1)
{
    double dot = 0.0, dist2 = 0.0;
    for (int k = 0; k < dh; ++k) {
        dot += x[k] * y[k];
        dist2 += (x[k] - y[k]) * (x[k] - y[k]);
    }
    if (kernel == 1)
        return exp(-dist2 / (2.0 * p0 * p0));
    if (kernel == 2)
        return pow(dot + p0, p1);
    return dot;
}

/* CKA with the kernel chosen by (kernel, p0, p1) as above; everything else as
 * described before hsic_unbiased. */
void oracle_similarity_cka(const void *calib, const void *w_gate_up, const void *w_down,
                           int dtype, int N, int n, int dh, int M, int dm, int kernel, double p0,
                           double p1, double *act, double *gram, double *sim)
{
    size_t gu = (size_t)2 * dm * dh, dn = (size_t)dh * dm;
    double *self = (double *)malloc(sizeof(double) * (size_t)M);
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] = 0.0;
    for (int b = 0; b < N; ++b) {
#pragma omp parallel
        {
            double *scratch = (double *)malloc(sizeof(double) * (size_t)dm);
#pragma omp for schedule(dynamic, 1) collapse(2)
            for (int j = 0; j < M; ++j)
                for (int r = 0; r < n; ++r)
                    expert_ffn(elem_ptr(calib, dtype, ((size_t)b * n + r) * dh),
                               elem_ptr(w_gate_up, dtype, (size_t)j * gu),
                               elem_ptr(w_down, dtype, (size_t)j * dn), dtype, dh, dm,
                               scratch, act + ((size_t)j * n + r) * dh);
            free(scratch);
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int j = 0; j < M; ++j)
            for (int r = 0; r < n; ++r)
                for (int c = 0; c < n; ++c) {
                    const double *x = act + ((size_t)j * n + r) * dh;
                    const double *y = act + ((size_t)j * n + c) * dh;
                    double dot = cka_kernel_value(x, y, dh, kernel, p0, p1);
                    gram[((size_t)j * n + r) * n + c] = (r == c) ? 0.0 : dot;
                }
        for (int j = 0; j < M; ++j)
            self[j] = hsic_unbiased(gram + (size_t)j * n * n, gram + (size_t)j * n * n, n);
#pragma omp parallel for schedule(dynamic, 1)
        for (int p = 0; p < M; ++p)
            for (int q = 0; q < M; ++q) {
                double cka = 0.0;
                if (self[p] > 0.0 && self[q] > 0.0)
                    cka = hsic_unbiased(gram + (size_t)p * n * n, gram + (size_t)q * n * n, n) /
                          sqrt(self[p] * self[q]);
                sim[(size_t)p * M + q] += cka;
            }
    }
    for (size_t i = 0; i < (size_t)M * M; ++i)
        sim[i] = sim[i] * (1.0 / (double)N);
    free(self);
}

/* linear-kernel CKA */
void oracle_similarity_cka_linear(const void *calib, const void *w_gate_up, const void *w_down,
                                  int dtype, int N, int n, int dh, int M, int dm, double *act,
                                  double *gram, double *sim)
{
    oracle_similarity_cka(calib, w_gate_up, w_down, dtype, N, n, dh, M, dm, 0, 0.0, 0.0, act, gram,
                          sim);
}
