// Expert-similarity estimation (Sec. 3.1.1, the appendix on similarity metrics
// and the appendix algorithm "Expert Similarity Estimation"): every expert
// runs on every calibration token through the same grouped FFN kernels the
// decode path uses (a work list in which each expert owns all tokens of the
// batch); then, with the Frobenius metric, x_pq = ||A_p - A_q||_F for all
// pairs and Sim = 1 - x / max(x) per batch, or, with the cosine metric, the
// mean over tokens of the cosine between the two experts' outputs, or linear
// CKA of the experts' Gram matrices; Sim is accumulated over batches and
// averaged.
#pragma once

#include "common.hpp"

namespace sere {

// work list "every expert, all n tokens": grid ceil(M*n/256), 256 threads
__global__ __launch_bounds__(256) void similarity_worklist_kernel(int M, int n, int32_t* sorted_token,
                                                                  int32_t* work_expert, int32_t* work_off,
                                                                  int32_t* work_cnt, int32_t* n_work) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < M * n) sorted_token[i] = i % n;
  if (i < M) {
    work_expert[i] = i;
    work_off[i] = i * n;
    work_cnt[i] = n;
  }
  if (i == 0) {
    n_work[0] = M;
    n_work[1] = 0;  // many long items: coarse cut
  }
}

// Frobenius distances of all pairs (appendix "Frobenius Similarity"), x_pq = ||A_p - A_q||_F, from
// the Gram matrix of the experts' outputs: with V_e the output of expert e on the batch, flattened
// to one vector of L = n * d_h numbers (A_e = sum over slices of y[slice][e*n .. e*n+n) rows),
//   x_pq^2 = <V_p, V_p> + <V_q, V_q> - 2 <V_p, V_q>.
// The Gram matrix is a dense contraction over L and runs on the matrix cores in fp64
// (v_mfma_f64_16x16x4: products of fp32 numbers are exact in fp64, sums carry ~1e-16 relative
// rounding each), so the cancellation in the formula above costs at most ~1e-15 of an output's
// squared norm: harmless for every pair but near-identical twins, which are recomputed as a
// direct difference by the wavefront that finds them.
typedef double f64x4 __attribute__((ext_vector_type(4)));
constexpr int kGramBlock = 64;     // experts per side of a workgroup's block: 2 x 2 wavefronts, each 2 x 2 tiles of 16 x 16
constexpr int kGramSteps = 2;      // 16-wide k steps per load group (two groups are in flight)
// partial Gram matrices lie M * M + kGramPad doubles apart: a power-of-two distance would put the
// same entry of every split on the same memory channel
constexpr int kGramPad = 96;
__host__ __device__ inline size_t gram_part_stride(int M) { return static_cast<size_t>(M) * M + kGramPad; }
constexpr double kGramTwinThreshold = 1e-9;  // x_pq^2 below this fraction of <V_p,V_p> + <V_q,V_q>: recompute directly

// upper-triangular blocks (bp <= bq) numbered row by row
__device__ __forceinline__ void gram_block_of(int index, int nb, int& bp, int& bq) {
  bp = 0;
  while (index >= nb - bp) {
    index -= nb - bp;
    ++bp;
  }
  bq = bp + index;
}

// part[split][p][q] = sum over the split's range of L of V_p[k] * V_q[k], for every (p, q) of the
// upper-triangular 64 x 64 blocks.  grid (nb (nb + 1) / 2, nsplit), 256 threads; lane l of a
// wavefront holds row l % 16 of each of its tiles, and of every 16 consecutive k the four
// 4 (l / 16) ... + 3 (the order of k inside the sum is free as long as both operands agree).
// `chunk` (the split's length) is a multiple of 2 * 16 * kGramSteps (= 64, as L is).
__global__ __launch_bounds__(256) void frobenius_gram_kernel(const float* __restrict__ y, int ksplit, int rows, int n,
                                                             int dh, int M, long long chunk,
                                                             double* __restrict__ part,
                                                             unsigned long long* __restrict__ max_bits) {
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *max_bits = 0ull;   // for frobenius_distance_kernel
  const int nb = (M + kGramBlock - 1) / kGramBlock;
  int bp, bq;
  gram_block_of(blockIdx.x, nb, bp, bq);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r16 = lane & 15, kq = lane >> 4;
  const int p0 = bp * kGramBlock + (wave >> 1) * 32, q0 = bq * kGramBlock + (wave & 1) * 32;
  const long long L = static_cast<long long>(n) * dh;             // multiple of 64
  const size_t slice = static_cast<size_t>(rows) * dh;
  const float* ap[2];
  const float* aq[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {   // rows beyond M repeat the last one (their results are not stored)
    ap[t] = y + static_cast<size_t>(min(p0 + 16 * t + r16, M - 1)) * L + 4 * kq;
    aq[t] = y + static_cast<size_t>(min(q0 + 16 * t + r16, M - 1)) * L + 4 * kq;
  }
  const long long kbeg = blockIdx.y * chunk, kend = min(kbeg + chunk, L);
  auto fetch = [&](const float* row, long long k) {
    float4 v = *reinterpret_cast<const float4*>(row + k);
    for (int s = 1; s < ksplit; ++s) {
      const float4 v2 = *reinterpret_cast<const float4*>(row + s * slice + k);
      v.x += v2.x; v.y += v2.y; v.z += v2.z; v.w += v2.w;
    }
    return v;
  };
  f64x4 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};
  // groups of kGramSteps steps, double buffered: the loads of the next group are in flight while
  // the current one is multiplied (the split's length is a multiple of 2 * 16 * kGramSteps)
  float4 va[2][kGramSteps][2], vb[2][kGramSteps][2];
  auto fetch_group = [&](int buf, long long k) {
#pragma unroll
    for (int st = 0; st < kGramSteps; ++st)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        va[buf][st][t] = fetch(ap[t], k + 16 * st);
        vb[buf][st][t] = fetch(aq[t], k + 16 * st);
      }
  };
  auto multiply_group = [&](int buf) {
#pragma unroll
    for (int st = 0; st < kGramSteps; ++st)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const float4 x = va[buf][st][a], w = vb[buf][st][b];
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(x.x), static_cast<double>(w.x), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(x.y), static_cast<double>(w.y), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(x.z), static_cast<double>(w.z), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(x.w), static_cast<double>(w.w), acc[a][b], 0, 0, 0);
        }
  };
  constexpr int kGroup = 16 * kGramSteps;
  fetch_group(0, kbeg);
  for (long long k = kbeg; k < kend; k += 2 * kGroup) {
    fetch_group(1, k + kGroup);                               // in range: the split holds whole pairs of groups
    multiply_group(0);
    fetch_group(0, k + 2 * kGroup < kend ? k + 2 * kGroup : kbeg);   // after the last pair: a harmless re-read
    multiply_group(1);
  }
  // lane l holds D[l / 16 + 4 r][l % 16], r = 0..3 (the fp64 tile interleaves its row blocks)
  double* out = part + static_cast<size_t>(blockIdx.y) * gram_part_stride(M);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int pp = p0 + 16 * a + kq + 4 * r, qq = q0 + 16 * b + r16;
        if (pp < M && qq < M) out[static_cast<size_t>(pp) * M + qq] = acc[a][b][r];
      }
}

// The partial Gram matrices are added in two fixed-order levels: group r of kGramGroups takes the
// splits r, r + kGramGroups, ... (this kernel; entries below the block diagonal are read from
// their mirror image), and the distance kernel adds the kGramGroups group sums.
// grid (ceil(M * M / 256), kGramGroups), 256 threads.
constexpr int kGramGroups = 8;
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ part, int nsplit, int M,
                                                          double* __restrict__ gram) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * M) return;
  int a = idx / M, b = idx % M;
  if (a / kGramBlock > b / kGramBlock) {
    const int t = a;
    a = b;
    b = t;
  }
  const size_t mm = gram_part_stride(M);
  const double* src = part + static_cast<size_t>(a) * M + b;
  double g = 0.0;
  for (int s = blockIdx.y; s < nsplit; s += kGramGroups) g += src[s * mm];
  gram[static_cast<size_t>(blockIdx.y) * M * M + idx] = g;
}

// dist[p][q] = sqrt(G_pp + G_qq - 2 G_pq), G = the sum of the group sums `gram`.  A pair whose squared distance is below
// kGramTwinThreshold of G_pp + G_qq (near-identical outputs: the subtraction has cancelled most
// digits) is recomputed as a direct difference sqrt(sum_i (A_p[i] - A_q[i])^2) by the whole
// wavefront, one such pair after the other.  The largest distance of the batch is gathered in
// *max_bits (the bits of a non-negative double order like the number; cleared by the Gram kernel).
// grid ceil(M * M / 256), 256 threads.
__global__ __launch_bounds__(256) void frobenius_distance_kernel(const double* __restrict__ gram,
                                                                 const float* __restrict__ y, int ksplit, int rows,
                                                                 int n, int dh, int M, double* __restrict__ dist,
                                                                 unsigned long long* __restrict__ max_bits) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int lane = threadIdx.x & 63;
  const bool valid = idx < M * M;
  const int p = valid ? idx / M : 0, q = valid ? idx % M : 0;
  double d = 0.0;
  bool twin = false;
  auto entry = [&](int at) {   // the group sums of one entry, in fixed order
    double g = 0.0;
#pragma unroll
    for (int r = 0; r < kGramGroups; ++r) g += gram[static_cast<size_t>(r) * M * M + at];
    return g;
  };
  if (valid && p != q) {
    const double gpp = entry(p * M + p), gqq = entry(q * M + q);
    const double d2 = (gpp + gqq) - 2.0 * entry(idx);
    twin = d2 < kGramTwinThreshold * (gpp + gqq);
    if (!twin) d = sqrt(d2);
  }
  unsigned long long todo = __ballot(twin);
  const size_t len = static_cast<size_t>(n) * dh;          // multiple of 64
  const size_t slice = static_cast<size_t>(rows) * dh;
  while (todo != 0ull) {                                   // wave-uniform
    const int src = __ffsll(static_cast<long long>(todo)) - 1;
    todo &= todo - 1ull;
    const int tp = __shfl(p, src, kWave), tq = __shfl(q, src, kWave);
    const float* ap = y + static_cast<size_t>(tp) * len;
    const float* aq = y + static_cast<size_t>(tq) * len;
    double acc = 0.0;
    for (size_t i = static_cast<size_t>(lane) * 4; i < len; i += 256) {
      float4 a = *reinterpret_cast<const float4*>(ap + i), b = *reinterpret_cast<const float4*>(aq + i);
      for (int s = 1; s < ksplit; ++s) {
        const float4 a2 = *reinterpret_cast<const float4*>(ap + s * slice + i);
        const float4 b2 = *reinterpret_cast<const float4*>(aq + s * slice + i);
        a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
        b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
      }
      const double dx = static_cast<double>(a.x) - b.x, dy = static_cast<double>(a.y) - b.y;
      const double dz = static_cast<double>(a.z) - b.z, dw = static_cast<double>(a.w) - b.w;
      acc += dx * dx + dy * dy + dz * dz + dw * dw;
    }
    acc = wave_sum(acc);
    if (lane == src) d = sqrt(acc);
  }
  if (valid) dist[idx] = d;
  double m = d;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, kWave));
  if (lane == 0 && m > 0.0) atomicMax(max_bits, static_cast<unsigned long long>(__double_as_longlong(m)));
}

// Cosine metric (appendix "Cosine Similarity"): out[p][q] = (1/n) sum over tokens i of
// <A_p[i], A_q[i]> / (|A_p[i]| |A_q[i]|); a token where either output is the zero vector
// contributes 0.  A_e as above.  grid (M, M), 256 threads: wavefront w takes tokens w, w+4, ...;
// fp64 accumulation, the four partial sums added in fixed order.
__global__ __launch_bounds__(256) void pair_cosine_kernel(const float* __restrict__ y, int ksplit, int rows, int n,
                                                          int dh, int M, double* __restrict__ out) {
  __shared__ double part[4];
  const int p = blockIdx.y, q = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const size_t slice = static_cast<size_t>(rows) * dh;
  double total = 0.0;
  for (int i = wave; i < n; i += 4) {
    const float* ap = y + (static_cast<size_t>(p) * n + i) * dh;
    const float* aq = y + (static_cast<size_t>(q) * n + i) * dh;
    double dot = 0.0, np2 = 0.0, nq2 = 0.0;
    for (int c = lane * 4; c < dh; c += 256) {
      float4 a = *reinterpret_cast<const float4*>(ap + c), b = *reinterpret_cast<const float4*>(aq + c);
      for (int s = 1; s < ksplit; ++s) {
        const float4 a2 = *reinterpret_cast<const float4*>(ap + s * slice + c);
        const float4 b2 = *reinterpret_cast<const float4*>(aq + s * slice + c);
        a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
        b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
      }
      const double ax = a.x, ay = a.y, az = a.z, aw = a.w, bx = b.x, by = b.y, bz = b.z, bw = b.w;
      dot += ax * bx + ay * by + az * bz + aw * bw;
      np2 += ax * ax + ay * ay + az * az + aw * aw;
      nq2 += bx * bx + by * by + bz * bz + bw * bw;
    }
    dot = wave_sum(dot);
    np2 = wave_sum(np2);
    nq2 = wave_sum(nq2);
    const double den = sqrt(np2) * sqrt(nq2);
    if (den > 0.0) total += dot / den;
  }
  if (lane == 0) part[wave] = total;
  __syncthreads();
  if (threadIdx.x == 0) out[static_cast<size_t>(p) * M + q] = ((part[0] + part[1]) + (part[2] + part[3])) / n;
}

// Linear CKA (appendix "Centered Kernel Alignment"), step 1: the Gram matrix of every expert's
// outputs with its diagonal set to zero, gram[e][i][j] = <A_e[i], A_e[j]> (i != j), and its row
// sums.  Entries (i, j) and (j, i) are formed by the same operations in the same order, so the
// matrix is symmetric to the bit.  grid (n, M), 256 threads: wavefront w takes j = w, w+4, ...;
// fp64 accumulation.
// With `diag` (RBF and polynomial kernels) the diagonal <A_e[i], A_e[i]> goes there and the row
// sums are left to gram_transform_kernel (rowsum == nullptr).
__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ y, int ksplit, int rows, int n, int dh,
                                                   double* __restrict__ gram, double* __restrict__ rowsum,
                                                   double* __restrict__ diag) {
  __shared__ double part[4];
  const int i = blockIdx.x, e = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const size_t slice = static_cast<size_t>(rows) * dh;
  const float* ai = y + (static_cast<size_t>(e) * n + i) * dh;
  double row = 0.0;
  for (int j = wave; j < n; j += 4) {
    const float* aj = y + (static_cast<size_t>(e) * n + j) * dh;
    double dot = 0.0;
    for (int c = lane * 4; c < dh; c += 256) {
      float4 a = *reinterpret_cast<const float4*>(ai + c), b = *reinterpret_cast<const float4*>(aj + c);
      for (int s = 1; s < ksplit; ++s) {
        const float4 a2 = *reinterpret_cast<const float4*>(ai + s * slice + c);
        const float4 b2 = *reinterpret_cast<const float4*>(aj + s * slice + c);
        a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
        b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
      }
      const double ax = a.x, ay = a.y, az = a.z, aw = a.w, bx = b.x, by = b.y, bz = b.z, bw = b.w;
      dot += (ax * bx + ay * by) + (az * bz + aw * bw);
    }
    dot = wave_sum(dot);
    if (j == i) {
      if (diag != nullptr && lane == 0) diag[static_cast<size_t>(e) * n + i] = dot;
      dot = 0.0;
    }
    if (lane == 0) gram[(static_cast<size_t>(e) * n + i) * n + j] = dot;
    row += dot;
  }
  if (lane == 0) part[wave] = row;
  __syncthreads();
  if (threadIdx.x == 0 && rowsum != nullptr)
    rowsum[static_cast<size_t>(e) * n + i] = (part[0] + part[1]) + (part[2] + part[3]);
}

constexpr int kCkaLinear = 0, kCkaRbf = 1, kCkaPoly = 2;  // SERE_CKA_* of the header

// The other two kernels of that appendix, from the linear Gram matrix G (off-diagonal entries in
// `gram`, diagonal in `diag`), in place, with the row sums of the result:
//   RBF:        K_ij = exp(-(G_ii + G_jj - 2 G_ij) / (2 sigma^2)),  sigma = p0
//   polynomial: K_ij = (G_ij + c)^d,  c = p0, d = degree (repeated multiplication)
// The diagonal stays 0 (the HSIC estimator ignores it); (i, j) and (j, i) take the same operations
// on the same values, so the matrix stays symmetric to the bit.  grid (n, M), 256 threads.
__global__ __launch_bounds__(256) void gram_transform_kernel(double* __restrict__ gram,
                                                             const double* __restrict__ diag, int n, int kernel,
                                                             double p0, int degree,
                                                             double* __restrict__ rowsum) {
  __shared__ double part[4];
  const int i = blockIdx.x, e = blockIdx.y;
  double* row = gram + (static_cast<size_t>(e) * n + i) * n;
  const double* d = diag + static_cast<size_t>(e) * n;
  const double di = d[i];
  double sum = 0.0;
  for (int j = threadIdx.x; j < n; j += 256) {
    double v = 0.0;
    if (j != i) {
      const double g = row[j];
      if (kernel == kCkaRbf) {
        v = exp(-((di + d[j]) - 2.0 * g) / (2.0 * p0 * p0));
      } else {
        const double base = g + p0;
        v = base;
        for (int k = 1; k < degree; ++k) v *= base;
      }
    }
    row[j] = v;
    sum += v;
  }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) rowsum[static_cast<size_t>(e) * n + i] = (part[0] + part[1]) + (part[2] + part[3]);
}

// Linear CKA, step 2: the unbiased estimator of HSIC for every pair of experts (Song et al. 2012,
// the O(n^2) estimator the appendix refers to), from the zero-diagonal Gram matrices Kt_p, Kt_q:
//   hsic[p][q] = [ tr(Kt_p Kt_q) + (1'Kt_p 1)(1'Kt_q 1) / ((n-1)(n-2)) - 2 (1'Kt_p Kt_q 1) / (n-2) ] / (n (n-3))
// with tr(Kt_p Kt_q) = sum_ij Kt_p[i][j] Kt_q[i][j] (symmetric matrices) and 1'Kt_p Kt_q 1 = the
// dot product of the two row-sum vectors.  grid (M, M), 256 threads; n >= 4.
__global__ __launch_bounds__(256) void pair_hsic_kernel(const double* __restrict__ gram,
                                                        const double* __restrict__ rowsum, int n, int M,
                                                        double* __restrict__ hsic) {
  __shared__ double part[4][4];
  const int p = blockIdx.y, q = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const double* kp = gram + static_cast<size_t>(p) * n * n;
  const double* kq = gram + static_cast<size_t>(q) * n * n;
  double tr = 0.0, cross = 0.0, sp = 0.0, sq = 0.0;
  for (int i = threadIdx.x; i < n * n; i += 256) tr += kp[i] * kq[i];
  for (int i = threadIdx.x; i < n; i += 256) {
    const double rp = rowsum[static_cast<size_t>(p) * n + i], rq = rowsum[static_cast<size_t>(q) * n + i];
    cross += rp * rq;
    sp += rp;
    sq += rq;
  }
  tr = wave_sum(tr);
  cross = wave_sum(cross);
  sp = wave_sum(sp);
  sq = wave_sum(sq);
  if (lane == 0) {
    part[0][wave] = tr;
    part[1][wave] = cross;
    part[2][wave] = sp;
    part[3][wave] = sq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double v[4];
    for (int k = 0; k < 4; ++k) v[k] = (part[k][0] + part[k][1]) + (part[k][2] + part[k][3]);
    const double dn = n;
    hsic[static_cast<size_t>(p) * M + q] =
        (v[0] + v[2] * v[3] / ((dn - 1.0) * (dn - 2.0)) - 2.0 * v[1] / (dn - 2.0)) / (dn * (dn - 3.0));
  }
}

constexpr int kMetricFrobenius = 0, kMetricCosine = 1, kMetricCkaLinear = 2;

// Frobenius: acc[p][q] (+)= 1 - dist/max(dist), the maximum of the batch given as the bits of a
// double in *max_bits; cosine: acc[p][q] (+)= dist[p][q] (the pair kernel's value as it is); linear
// CKA: acc[p][q] (+)= dist[p][q] / sqrt(dist[p][p] dist[q][q]), dist holding the HSIC estimates (0
// where a self-term is not positive: the quotient is undefined there).  On the last batch
// sim = acc / N.  grid ceil(M * M / 256), 256 threads.
__global__ __launch_bounds__(256) void similarity_accumulate_kernel(const double* __restrict__ dist, int M,
                                                                    int batch, int num_batches, int metric,
                                                                    const unsigned long long* __restrict__ max_bits,
                                                                    double* __restrict__ acc,
                                                                    float* __restrict__ sim) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M * M) return;
  double sv;
  if (metric == kMetricCosine) {
    sv = dist[i];
  } else if (metric == kMetricCkaLinear) {
    const double hp = dist[static_cast<size_t>(i / M) * M + i / M], hq = dist[static_cast<size_t>(i % M) * M + i % M];
    sv = (hp > 0.0 && hq > 0.0) ? dist[i] / sqrt(hp * hq) : 0.0;
  } else {
    const double mx = __longlong_as_double(static_cast<long long>(*max_bits));
    sv = mx > 0.0 ? 1.0 - dist[i] / mx : 1.0;  // all pairs identical: Sim = 1
  }
  const double a = (batch == 0 ? 0.0 : acc[i]) + sv;
  acc[i] = a;
  if (batch == num_batches - 1) sim[i] = static_cast<float>(a / num_batches);
}

}  // namespace sere
