/*
 * sere.h - C ABI of the MI355X (gfx950) batch-decode MoE layer with SERE,
 * similarity-based expert re-routing.
 *
 * One call = one decode step of one MoE layer over a batch of T tokens:
 * router top-K, batch-wide primary-expert selection, re-routing of secondary
 * experts onto their most similar primary expert (keeping critical experts),
 * compaction of the token-to-expert map, and the grouped SwiGLU expert FFN
 * over the surviving experts only.
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, at least
 *     16-byte aligned, dense row-major with the last index contiguous.
 *     Inputs are never written.  The library allocates nothing per call and
 *     writes only to `out`, to the non-NULL members of `sere_route_out` and
 *     to `workspace`.
 *   - `dtype` selects the storage of hidden states, router weights, expert
 *     weights and the layer output: SERE_F32 (IEEE binary32) or SERE_BF16
 *     (bfloat16).  The similarity matrix and gate weights are always fp32,
 *     indices int32.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises the device or copies to the
 *     host; results are valid once the caller has synchronised the stream.
 *   - Return value: SERE_OK (0) or a negative SERE_ERR_* code.  All argument
 *     checks happen before anything is enqueued, so a failing call has no
 *     device side effects.  No exception or abort crosses this boundary.
 *   - Not checked on the device (preconditions): hidden states, router
 *     weights and `sim` are finite; `topk_ids` handed to sere_reroute lie in
 *     [0, M) (an id outside that range is read as the nearest one inside it:
 *     the result is then meaningless, but no access leaves its buffer).
 *   - Calls are re-entrant as long as concurrent calls use distinct
 *     workspaces and outputs.
 *   - Expert indices are 0-based.
 */
#ifndef SERE_H
#define SERE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SERE_F32 0
#define SERE_BF16 1

#define SERE_OK 0
#define SERE_ERR_NULL_PTR (-1)            /* a required pointer is NULL                  */
#define SERE_ERR_BAD_SHAPE (-2)           /* a size is out of the supported range        */
#define SERE_ERR_BAD_TOPK (-3)            /* K > M, or S outside [1, K]                  */
#define SERE_ERR_BAD_DTYPE (-4)           /* dtype is neither SERE_F32 nor SERE_BF16     */
#define SERE_ERR_MISALIGNED (-5)          /* a pointer is not 16-byte aligned            */
#define SERE_ERR_WORKSPACE_TOO_SMALL (-6) /* workspace_bytes < sere_workspace_bytes()    */
#define SERE_ERR_BAD_FLAGS (-7)           /* flags has a bit no SERE_FLAG_* names, or two
                                             that exclude each other                     */
#define SERE_ERR_NONFINITE_THRESHOLD (-8) /* threshold is NaN or infinite                */
#define SERE_ERR_HIP (-9)                 /* a HIP launch reported an error              */
#define SERE_ERR_BAD_KERNEL (-10)         /* sere_similarity_cka: unknown kernel or a
                                             parameter outside its range                 */
#define SERE_ERR_SCRATCH_TOO_SMALL (-11)  /* sere_moe_decode_static: the configuration needs
                                             more than SERE_STATIC_SCRATCH_BYTES         */

/* sere_config.flags */
#define SERE_FLAG_RESIDUAL 1 /* sere_moe_decode[_baseline]: out = hidden + layer(hidden), the
                                residual connection around the MoE block of a decoder layer, added
                                in fp32 before the one rounding to the output type; lets a stack
                                of layers be chained with no kernel in between.  `out` must not
                                overlap `hidden`.  Ignored by the routing-only entry points.   */
#define SERE_FLAG_SIM_COSINE 2 /* sere_similarity: the cosine metric instead of the Frobenius one
                                 (appendix on similarity metrics); ignored by the other entry
                                 points                                                        */
#define SERE_FLAG_SIM_CKA_LINEAR 4 /* sere_similarity: linear-kernel CKA instead (same appendix);
                                     excludes SERE_FLAG_SIM_COSINE; ignored by the other entry
                                     points                                                    */

#define SERE_MAX_EXPERTS 256
#define SERE_MAX_SHARED 16
#define SERE_MAX_TOKENS 65536
#define SERE_MAX_ROWS 1048576 /* T * (K + num_shared): rows of the expert-sorted slot list */

/*
 * Problem description.  Names follow the paper: T tokens in the decode batch,
 * d_h hidden size, M routed experts, K experts per token, d_m expert
 * intermediate size (appendix "Preliminaries on MoEs"); S = `select_top_k`,
 * the number of top-ranked experts per token that form the primary set, and
 * rho = `threshold`, the similarity below which a secondary expert is kept as
 * a critical expert (Sec. 3.2.2; the two knobs of the appendix on
 * hyper-parameters).
 */
typedef struct sere_config {
  int32_t num_tokens;   /* T, 1 .. SERE_MAX_TOKENS; T * (K + num_shared) <= SERE_MAX_ROWS */
  int32_t hidden;       /* d_h, positive multiple of 64, at most 65536              */
  int32_t num_experts;  /* M routed experts, 1 .. SERE_MAX_EXPERTS                   */
  int32_t top_k;        /* K, 1 .. M                                                 */
  int32_t inter;        /* d_m, positive multiple of 64, at most 262144             */
  int32_t num_shared;   /* always-on shared experts, 0 .. SERE_MAX_SHARED; they see
                           every token with weight 1 and take no part in routing    */
  int32_t dtype;        /* SERE_F32 | SERE_BF16                                      */
  int32_t select_top_k; /* S, 1 .. K; S == K leaves the routing unchanged            */
  float threshold;      /* rho, finite; rho <= 0 disables the critical-expert test
                           (every secondary expert is re-routed), as in the paper's
                           re-routing algorithm                                     */
  int32_t flags;        /* 0 or an OR of SERE_FLAG_*                                 */
} sere_config;

/*
 * Optional routing outputs; every member may be NULL (then that result stays
 * internal).  A = T*K.  "Slot" k of token t is the k-th ranked expert of the
 * router's ordered list R(t).
 */
typedef struct sere_route_out {
  int32_t *topk_ids;       /* [T,K]  I : router's experts by descending logit; equal
                                      logits: lower index first                      */
  float *topk_weights;     /* [T,K]  W : softmax over the K selected logits           */
  int32_t *rerouted_ids;   /* [T,K]  I': slots k < S unchanged; a slot keeps
                                      duplicates if two slots of a token land on
                                      the same expert                                */
  int32_t *count_before;   /* [M]    slots per expert under I                         */
  int32_t *count_after;    /* [M]    slots per expert under I'                        */
  int32_t *primary_mask;   /* [M]    1 iff the expert is in the primary set           */
  int32_t *num_active;     /* [2]    experts with a non-zero count {under I, under I'} */
  int32_t *expert_offsets; /* [M+1]  exclusive prefix sum of count_after              */
  int32_t *sorted_token;   /* [A]    token of each slot, grouped by expert (ascending
                                      expert, then token, then slot)                 */
  int32_t *sorted_slot;    /* [A]    slot index k of the same entries                 */
} sere_route_out;

/* Bytes of device workspace the calls below need for `cfg` (256-byte aligned
 * base expected); 0 if `cfg` is NULL or invalid. */
size_t sere_workspace_bytes(const sere_config *cfg);

/*
 * Routing half of the layer (Sec. 3.2.2 Steps 1-3 on top of the router):
 * router logits <x_t, Wr_e>, ordered top-K and gate (appendix "Preliminaries
 * on MoEs", top-k gating equation), primary set (primary-set equation), most
 * similar primary expert and threshold test per secondary expert (arg-max and
 * re-routing-condition equations; ties go to the lower index, scan order of
 * the appendix re-routing algorithm), final active set and the re-grouped
 * token-to-expert map (final-set equation).
 *   hidden   [T, d_h]  dtype
 *   router_w [M, d_h]  dtype, row e = router weights of expert e
 *   sim      [M, M]    fp32, sim[u*M + v] = similarity of secondary expert u
 *                      (row) to candidate primary expert v (column); the
 *                      diagonal is never read; need not be symmetric
 * Router logits are accumulated in fp64, so the ordering equals that of exact
 * arithmetic except for logits closer than ~1e-12.
 */
int sere_route(const sere_config *cfg, const void *hidden, const void *router_w,
               const float *sim, const sere_route_out *out, void *workspace,
               size_t workspace_bytes, void *hip_stream);

/*
 * The re-routing step alone, with the signature of the paper's appendix
 * algorithm "CUDA-accelerated SERE": top-K indices in, re-routed indices out.
 *   topk_ids [T, K] int32, already ordered by descending router weight.
 * `out->topk_ids` and `out->topk_weights` are ignored; cfg->hidden, inter,
 * num_shared and dtype are not used but must still be valid.
 */
int sere_reroute(const sere_config *cfg, const int32_t *topk_ids, const float *sim,
                 const sere_route_out *out, void *workspace, size_t workspace_bytes,
                 void *hip_stream);

/*
 * Full decode step with re-routing:
 *   out[t] = sum_k W[t,k] * E_{I'[t,k]}(x_t) + sum_s Eshared_s(x_t)
 * with E(x) = W_down (silu(W_gate x) * (W_up x))  (appendix "Preliminaries on
 * MoEs", layer-output and expert equations).  The gate weights W are the
 * router's and are not changed by re-routing (Sec. 3.2.2 Step 2).  Only the
 * experts that still own a slot under I' (plus the shared experts) are read
 * from memory, each exactly once.
 *   w_gate_up      [M, 2*d_m, d_h]     dtype; rows 0..d_m-1 gate, d_m..2*d_m-1 up
 *   w_down         [M, d_h, d_m]       dtype
 *   shared_gate_up [n_sh, 2*d_m, d_h]  dtype, NULL iff num_shared == 0
 *   shared_down    [n_sh, d_h, d_m]    dtype, NULL iff num_shared == 0
 *   out            [T, d_h]            dtype; fp32 accumulation, one rounding
 *   dbg            optional routing outputs (may be NULL)
 * The intermediate silu(g)*u is kept in fp32 for SERE_F32 and rounded once to
 * bf16 (the matrix cores' input type) for SERE_BF16.
 */
int sere_moe_decode(const sere_config *cfg, const void *hidden, const void *router_w,
                    const void *w_gate_up, const void *w_down, const void *shared_gate_up,
                    const void *shared_down, const float *sim, void *out,
                    const sere_route_out *dbg, void *workspace, size_t workspace_bytes,
                    void *hip_stream);

/*
 * The same step without re-routing: the standard top-K MoE layer (I' = I).
 * cfg->select_top_k and cfg->threshold are validated but have no effect: the
 * call behaves as select_top_k == top_k (so `primary_mask` marks every
 * activated expert).
 */
int sere_moe_decode_baseline(const sere_config *cfg, const void *hidden, const void *router_w,
                             const void *w_gate_up, const void *w_down,
                             const void *shared_gate_up, const void *shared_down, void *out,
                             const sere_route_out *dbg, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * sere_moe_decode for callers that cannot allocate device memory or hand over
 * a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * results as sere_moe_decode, minus the workspace: the intermediate buffers
 * live in a device array of SERE_STATIC_SCRATCH_BYTES bytes that is part of
 * the library image (every GPU the library runs on holds its own copy until
 * the process ends).  The call allocates nothing and frees nothing.
 *   - SERE_ERR_SCRATCH_TOO_SMALL if sere_workspace_bytes(cfg) exceeds
 *     SERE_STATIC_SCRATCH_BYTES (the five reference layer shapes up to a
 *     Mixtral-shaped layer at batch 64 fit); nothing is enqueued then.
 *   - The device that `hip_stream` belongs to must be the current device.  The
 *     first call on a device looks up that device's copy of the array (no
 *     allocation, but a runtime query: make the first call outside graph
 *     capture).
 *   - All calls on one GPU share the one array, which keeps the last call's
 *     contents (nothing in it needs to start at zero).  Two calls whose
 *     execution overlaps on one GPU (different streams, or parallel branches
 *     of a graph) race; calls ordered on one stream do not.
 */
#define SERE_STATIC_SCRATCH_BYTES (32u << 20)
int sere_moe_decode_static(const sere_config *cfg, const void *hidden, const void *router_w,
                           const void *w_gate_up, const void *w_down, const void *shared_gate_up,
                           const void *shared_down, const float *sim, void *out,
                           const sere_route_out *dbg, void *hip_stream);

/*
 * Expert-similarity matrix of one layer from calibration tokens, with the
 * Frobenius metric (Sec. 3.1.1 accumulation equation; appendix "Frobenius
 * Similarity"; appendix algorithm "Expert Similarity Estimation"): for each of
 * `num_batches` batches of `batch_tokens` tokens every routed expert is run on
 * every token, x_pq = ||A_p - A_q||_F, Sim(p,q) = 1 - x_pq / max over all pairs
 * of that batch, and sim = the mean of Sim over the batches (diagonal 1).  The
 * distances come from the Gram matrix of the experts' flattened outputs,
 * x_pq^2 = <A_p,A_p> + <A_q,A_q> - 2 <A_p,A_q>, formed in fp64 on the matrix
 * cores; pairs whose squared distance is below 1e-9 of <A_p,A_p> + <A_q,A_q>
 * (near-identical experts) are recomputed as a direct difference.
 * With SERE_FLAG_SIM_COSINE in cfg->flags the metric is the cosine one of the
 * appendix "Cosine Similarity" instead: Sim(p,q) = the mean over the batch's
 * tokens of the cosine between the two experts' outputs for that token (a
 * token where either output is the zero vector contributes 0); values lie in
 * [-1, 1].  With SERE_FLAG_SIM_CKA_LINEAR it is centered kernel alignment with
 * the linear kernel (appendix "Centered Kernel Alignment"): K_p = A_p A_p^T
 * [batch_tokens, batch_tokens] per expert, Sim(p,q) = HSIC(K_p,K_q) /
 * sqrt(HSIC(K_p,K_p) HSIC(K_q,K_q)) with the unbiased O(n^2) estimator of HSIC
 * that the appendix refers to (on the Gram matrices with zeroed diagonals Kt:
 * [tr(Kt_p Kt_q) + (1'Kt_p 1)(1'Kt_q 1)/((n-1)(n-2)) - 2 (1'Kt_p Kt_q 1)/(n-2)]
 * / (n(n-3))); a pair with a non-positive self-term contributes 0; needs
 * 4 <= batch_tokens <= 512 (else SERE_ERR_BAD_SHAPE).  The RBF and polynomial
 * kernels of that appendix: sere_similarity_cka below.
 *   calib [num_batches, batch_tokens, d_h]  dtype, device
 *   sim   [M, M] fp32, device, written
 * Uses cfg->hidden, num_experts, inter, dtype (the other fields must be valid
 * but are not used).  The experts run through the decode path's own FFN
 * kernels, so for SERE_BF16 the activations carry bf16-level rounding (as a
 * bf16 model forward does); similarities agree with an fp64 evaluation to a
 * few 1e-3.  batch_tokens: 1 .. 4096, num_batches: 1 .. 4096.
 * Workspace: sere_similarity_workspace_bytes(cfg, batch_tokens).
 */
size_t sere_similarity_workspace_bytes(const sere_config *cfg, int32_t batch_tokens);
int sere_similarity(const sere_config *cfg, const void *calib, int32_t num_batches,
                    int32_t batch_tokens, const void *w_gate_up, const void *w_down, float *sim,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same estimate with centered kernel alignment and any of the three
 * kernels of the appendix "Centered Kernel Alignment" (cfg->flags' metric bits
 * are ignored): K_p[i][j] = k(A_p[i], A_p[j]) over the batch's tokens with
 *   SERE_CKA_LINEAR  k(x, y) = <x, y>                          (no parameter)
 *   SERE_CKA_RBF     k(x, y) = exp(-|x - y|^2 / (2 sigma^2))   param0 = sigma > 0
 *   SERE_CKA_POLY    k(x, y) = (<x, y> + c)^d                  param0 = c, param1 = d,
 *                                                              an integer in 1 .. 16
 * and Sim(p,q) = HSIC(K_p,K_q) / sqrt(HSIC(K_p,K_p) HSIC(K_q,K_q)) with the
 * unbiased estimator described above.  The paper does not state the kernel
 * parameters it used; they are the caller's.  4 <= batch_tokens <= 512.
 * SERE_ERR_BAD_KERNEL for an unknown kernel or a parameter outside its range.
 * Workspace: sere_similarity_cka_workspace_bytes(cfg, batch_tokens).
 */
#define SERE_CKA_LINEAR 0
#define SERE_CKA_RBF 1
#define SERE_CKA_POLY 2
size_t sere_similarity_cka_workspace_bytes(const sere_config *cfg, int32_t batch_tokens);
int sere_similarity_cka(const sere_config *cfg, const void *calib, int32_t num_batches,
                        int32_t batch_tokens, const void *w_gate_up, const void *w_down,
                        int32_t kernel, double param0, double param1, float *sim, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel the calls
 * above enqueue carries a pair of HIP events attached to its own dispatch on
 * the caller's stream: they take the kernel's start and end time stamps, so
 * the elapsed time is the kernel's duration as a profiler's kernel trace
 * reports it, without the gap to its neighbours (at most
 * SERE_TIMING_MAX_RECORDS launches are kept, later ones are not recorded).
 * Do not enable it on a stream that is being captured into a HIP graph.
 * sere_stage_timing_read waits for the recorded events, adds the elapsed
 * milliseconds and launch counts per stage into the two arrays of
 * SERE_NUM_STAGES entries, and clears the records.  Process-global, not
 * thread-safe, and slower than normal operation: never enable it while
 * measuring whole-step latency.
 */
#define SERE_STAGE_ROUTER 0   /* router logits                           */
#define SERE_STAGE_ROUTE 1    /* top-K, gate, re-route, compaction       */
#define SERE_STAGE_GATE_UP 2  /* gate/up projections + SiLU * up         */
#define SERE_STAGE_DOWN 3     /* down projection                         */
#define SERE_STAGE_COMBINE 4  /* weighted sum over slots, output store   */
#define SERE_STAGE_SIM_PAIRS 5 /* sere_similarity*: everything after the experts' forward pass
                                  (Gram matrices, pairwise metric, accumulation)              */
#define SERE_NUM_STAGES 6
#define SERE_TIMING_MAX_RECORDS 8192
int sere_stage_timing(int enable);
int sere_stage_timing_read(double *total_ms, int32_t *launches);

/*
 * Benchmark helper: a plain streaming read of `bytes` bytes of device memory at
 * `src` (a multiple of 16, 16-byte aligned) with non-temporal 128-bit loads,
 * enqueued on the stream; nothing is computed but a checksum that is stored to
 * sink[0] (device, 4 bytes) only if it equals a value no real data gives.  It
 * measures what the memory system delivers for a read of that size on this
 * machine, to set beside the published peak.  SERE_ERR_BAD_SHAPE for a size
 * that is 0 or not a multiple of 16.
 */
int sere_stream_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);

/* Static, human-readable text for a status code. */
const char *sere_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SERE_H */
