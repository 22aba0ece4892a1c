// Expert-similarity estimation (Sec. 3.1.1, the appendix on similarity metrics
// and the appendix algorithm "Expert Similarity Estimation"): every expert
// runs on every calibration token through the same grouped FFN kernels the
// decode path uses (a work list in which each expert owns all tokens of the
// batch); then, with the Frobenius metric, x_pq = ||A_p - A_q||_F for all
// pairs and Sim = 1 - x / max(x) per batch, or, with the cosine metric, the
// mean over tokens of the cosine between the two experts' outputs; Sim is
// accumulated over batches and averaged.
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

// dist[p][q] = sqrt(sum_i (A_p[i] - A_q[i])^2), A_e = sum over slices of y[slice][e*n .. e*n+n) rows.
// grid (M, M), 256 threads; fp64 accumulation.
__global__ __launch_bounds__(256) void pair_distance_kernel(const float* __restrict__ y, int ksplit, int rows,
                                                            int n, int dh, int M, double* __restrict__ dist) {
  __shared__ double part[4];
  const int p = blockIdx.y, q = blockIdx.x;
  const size_t len = static_cast<size_t>(n) * dh;          // multiple of 64
  const size_t slice = static_cast<size_t>(rows) * dh;
  const float* ap = y + static_cast<size_t>(p) * len;
  const float* aq = y + static_cast<size_t>(q) * len;
  double acc = 0.0;
  if (p != q) {
    for (size_t i = static_cast<size_t>(threadIdx.x) * 4; i < len; i += 1024) {
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
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) dist[static_cast<size_t>(p) * M + q] = sqrt((part[0] + part[1]) + (part[2] + part[3]));
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

// Frobenius: acc[p][q] (+)= 1 - dist/max(dist); cosine: acc[p][q] (+)= dist[p][q] (the pair
// kernel's value as it is); on the last batch sim = acc / N.  One block of 1024 threads.
__global__ __launch_bounds__(1024) void similarity_accumulate_kernel(const double* __restrict__ dist, int M,
                                                                     int batch, int num_batches, int cosine,
                                                                     double* __restrict__ acc,
                                                                     float* __restrict__ sim) {
  __shared__ double smax[16];
  const int total = M * M;
  double m = 0.0;
  for (int i = threadIdx.x; i < total; i += 1024) m = fmax(m, dist[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, kWave));
  if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = m;
  __syncthreads();
  double mx = 0.0;
  for (int w = 0; w < 16; ++w) mx = fmax(mx, smax[w]);
  for (int i = threadIdx.x; i < total; i += 1024) {
    const double sv = cosine ? dist[i] : (mx > 0.0 ? 1.0 - dist[i] / mx : 1.0);  // all pairs identical: Sim = 1
    const double a = (batch == 0 ? 0.0 : acc[i]) + sv;
    acc[i] = a;
    if (batch == num_batches - 1) sim[i] = static_cast<float>(a / num_batches);
  }
}

}  // namespace sere
