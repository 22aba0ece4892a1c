// Routing kernels: router logits, ordered top-K + gate, and the batch-wide
// re-routing / compaction kernel.
//
// Paper anchors: router logits R(x) and the top-k gate of the appendix
// "Preliminaries on MoEs"; primary set, most-similar primary, re-routing
// condition and final set of Sec. 3.2.2 (Steps 1-3).  The appendix algorithm
// "CUDA-accelerated SERE" gives one thread to every (token, secondary slot)
// and lets each scan all M experts; here the scan is done once per secondary
// EXPERT (its result depends only on the expert and the primary mask), by one
// 64-lane wavefront, and the rewritten map is counted, prefix-summed and
// regrouped per expert in the same workgroup, in LDS.
#pragma once

#include "common.hpp"

namespace sere {

// ---------------------------------------------------------------------------
// Router logits in fp64.  grid (ceil(M/16), T), 256 threads; wave w of block
// (bx, t) computes experts bx*16 + 4w .. +3 for token t.  Every logit is
// reduced in the same lane pattern, so bit-identical router rows give
// bit-identical logits (ties then resolve by index, as in exact arithmetic).
// Block (0,0) also clears the int32 word at `clear_word` (may be NULL).
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void router_logits_kernel(
    const void* __restrict__ hidden, const void* __restrict__ router_w, double* __restrict__ logits,
    int T, int M, int dh, int32_t* clear_word) {
  const int t = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (clear_word != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *clear_word = 0;
  const int e0 = blockIdx.x * 16 + wave * 4;
  for (int q = 0; q < 4; ++q) {
    const int e = e0 + q;
    if (e >= M) break;
    double acc = 0.0;
    for (int i = lane * 8; i < dh; i += 512) {
      float xv[8], wv[8];
      load8<DT>(hidden, static_cast<size_t>(t) * dh + i, xv);
      load8<DT>(router_w, static_cast<size_t>(e) * dh + i, wv);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = fma(static_cast<double>(xv[j]), static_cast<double>(wv[j]), acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) logits[static_cast<size_t>(t) * M + e] = acc;
  }
}

// ---------------------------------------------------------------------------
// Ordered top-K and gate, one wavefront per token (4 tokens per block).
// K rounds of arg-max over the not-yet-taken logits; a larger logit wins,
// equal logits go to the lower expert index.  Gate = softmax over the K
// selected logits (fp64 internally, stored fp32).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void topk_gate_kernel(const double* __restrict__ logits,
                                                        int32_t* __restrict__ topk_ids,
                                                        float* __restrict__ topk_w, int T, int M,
                                                        int K) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;  // whole wavefront leaves; the kernel has no barrier

  double cand[4];
  double mysel[4] = {0.0, 0.0, 0.0, 0.0};  // selected logit of rank k = lane + 64*c
  double top = 0.0;
  unsigned taken = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int e = lane + 64 * c;
    if (e < M) {
      cand[c] = logits[static_cast<size_t>(t) * M + e];
    } else {
      cand[c] = 0.0;
      taken |= 1u << c;
    }
  }
  for (int k = 0; k < K; ++k) {
    double bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool ok = !((taken >> c) & 1u);
      if (ok && (bi == 0x7fffffff || cand[c] > bv)) {
        bv = cand[c];
        bi = lane + 64 * c;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const double ov = __shfl_xor(bv, off, kWave);
      const int oi = __shfl_xor(bi, off, kWave);
      const bool mine_valid = bi != 0x7fffffff, other_valid = oi != 0x7fffffff;
      const bool take = other_valid && (!mine_valid || ov > bv || (ov == bv && oi < bi));
      if (take) {
        bv = ov;
        bi = oi;
      }
    }
    // every lane now holds the winner (bv, bi)
    if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
    if (k == 0) top = bv;
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (k == lane + 64 * c) mysel[c] = bv;
    if (lane == 0) topk_ids[static_cast<size_t>(t) * K + k] = bi;
  }
  double ex[4];
  double part = 0.0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    ex[c] = (lane + 64 * c < K) ? exp(mysel[c] - top) : 0.0;
    part += ex[c];
  }
  const double denom = wave_sum(part);
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (lane + 64 * c < K)
      topk_w[static_cast<size_t>(t) * K + lane + 64 * c] = static_cast<float>(ex[c] / denom);
}

// ---------------------------------------------------------------------------
// Batch-wide re-routing and compaction: ONE workgroup of 1024 threads.
// ---------------------------------------------------------------------------
struct RouteArgs {
  const int32_t* topk_ids;  // [A]  I
  const float* sim;         // [M,M] (unused when reroute == 0)
  int T, K, M, S, n_sh;
  float rho;
  int reroute;              // 0: identity map (standard top-K MoE)
  int32_t* rerouted_ids;    // [A]  I'
  int32_t* count_before;    // [M]
  int32_t* count_after;     // [M]
  int32_t* primary_mask;    // [M]
  int32_t* num_active;      // [2]
  int32_t* expert_offsets;  // [M+1]
  int32_t* sorted_token;    // [A + n_sh*T]
  int32_t* sorted_slot;     // [A]
  int32_t* slot_pos;        // [A]  position of slot a = t*K+k in the sorted list
  int32_t* work_expert;     // [M + n_sh] surviving experts ascending, then M+s per shared
  int32_t* work_off;        // [M + n_sh] first row of the item in the sorted list
  int32_t* work_cnt;        // [M + n_sh] rows of the item
  int32_t* n_work;          // [1]
};

constexpr int kRouteThreads = 1024;
constexpr int kRouteWaves = kRouteThreads / kWave;

__global__ __launch_bounds__(kRouteThreads) void route_kernel(RouteArgs p) {
  __shared__ int s_cnt_b[SERE_MAX_EXPERTS];
  __shared__ int s_cnt_a[SERE_MAX_EXPERTS];
  __shared__ int s_prim[SERE_MAX_EXPERTS];
  __shared__ int s_remap[SERE_MAX_EXPERTS];
  __shared__ int s_scan_cnt[SERE_MAX_EXPERTS];
  __shared__ int s_scan_act[SERE_MAX_EXPERTS];
  __shared__ int s_cursor[SERE_MAX_EXPERTS];
  __shared__ int s_round[kRouteWaves][SERE_MAX_EXPERTS];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int M = p.M, K = p.K, S = p.S;
  const int A = p.T * K;

  if (tid < SERE_MAX_EXPERTS) {
    s_cnt_b[tid] = 0;
    s_cnt_a[tid] = 0;
    s_prim[tid] = 0;
    s_remap[tid] = tid;
  }
  for (int i = tid; i < kRouteWaves * SERE_MAX_EXPERTS; i += kRouteThreads) (&s_round[0][0])[i] = 0;
  __syncthreads();

  // Step 1: activation histogram and primary mask (union of every token's top-S)
  for (int a = tid; a < A; a += kRouteThreads) {
    const int e = p.topk_ids[a];
    atomicAdd(&s_cnt_b[e], 1);
    if (a % K < S) s_prim[e] = 1;
  }
  __syncthreads();

  // Step 2: per secondary expert u (activated, not primary): most similar
  // primary v*, ascending scan with strict '>' (lowest index wins a tie, start
  // value (-inf, expert 0)); kept as critical iff rho > 0 and sim* < rho.
  if (p.reroute) {
    for (int u = wave; u < M; u += kRouteWaves) {
      if (s_cnt_b[u] == 0 || s_prim[u]) continue;  // wave-uniform
      float bs = -INFINITY;
      int bv = 0;
      for (int v = lane; v < M; v += kWave) {
        if (s_prim[v]) {
          const float s = p.sim[static_cast<size_t>(u) * M + v];
          if (s > bs) {
            bs = s;
            bv = v;
          }
        }
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const float os = __shfl_xor(bs, off, kWave);
        const int ov = __shfl_xor(bv, off, kWave);
        if (os > bs || (os == bs && ov < bv)) {
          bs = os;
          bv = ov;
        }
      }
      if (lane == 0) s_remap[u] = (p.rho > 0.0f && bs < p.rho) ? u : bv;
    }
  }
  __syncthreads();

  // Step 3: rewrite secondary slots, count the new map
  for (int a = tid; a < A; a += kRouteThreads) {
    const int e = p.topk_ids[a];
    const int e2 = (a % K >= S) ? s_remap[e] : e;
    p.rerouted_ids[a] = e2;
    atomicAdd(&s_cnt_a[e2], 1);
  }
  __syncthreads();

  // inclusive scans over experts: slots (-> offsets) and activity (-> work list rank)
  const bool is_e = tid < SERE_MAX_EXPERTS;
  const int my_cnt = (is_e && tid < M) ? s_cnt_a[tid] : 0;
  const int my_act = my_cnt > 0 ? 1 : 0;
  const int n_before = __syncthreads_count(is_e && tid < M && s_cnt_b[tid] > 0);
  if (is_e) {
    s_scan_cnt[tid] = my_cnt;
    s_scan_act[tid] = my_act;
  }
  __syncthreads();
  for (int d = 1; d < SERE_MAX_EXPERTS; d <<= 1) {
    int add_c = 0, add_a = 0;
    if (is_e && tid >= d) {
      add_c = s_scan_cnt[tid - d];
      add_a = s_scan_act[tid - d];
    }
    __syncthreads();
    if (is_e) {
      s_scan_cnt[tid] += add_c;
      s_scan_act[tid] += add_a;
    }
    __syncthreads();
  }
  const int n_after = s_scan_act[SERE_MAX_EXPERTS - 1];
  if (is_e && tid < M) {
    const int off = s_scan_cnt[tid] - my_cnt;
    s_cursor[tid] = off;
    p.expert_offsets[tid] = off;
    p.count_before[tid] = s_cnt_b[tid];
    p.count_after[tid] = my_cnt;
    p.primary_mask[tid] = s_prim[tid];
    if (my_act) {
      const int i = s_scan_act[tid] - 1;
      p.work_expert[i] = tid;
      p.work_off[i] = off;
      p.work_cnt[i] = my_cnt;
    }
  }
  if (tid == 0) {
    p.expert_offsets[M] = A;
    p.num_active[0] = n_before;
    p.num_active[1] = n_after;
    p.n_work[0] = n_after + p.n_sh;
  }
  if (tid < p.n_sh) {
    p.work_expert[n_after + tid] = M + tid;
    p.work_off[n_after + tid] = A + tid * p.T;
    p.work_cnt[n_after + tid] = p.T;
  }
  for (int i = tid; i < p.n_sh * p.T; i += kRouteThreads) p.sorted_token[A + i] = i % p.T;
  __syncthreads();

  // Stable regrouping by expert: slots keep ascending (token, slot) order
  // inside each expert.  A round covers 1024 consecutive slots, one wavefront
  // per 64; rank inside the wavefront by comparing against every lane, rank
  // across wavefronts through the per-round table.
  for (int base = 0; base < A; base += kRouteThreads) {
    const int a = base + tid;
    const bool valid = a < A;
    int e = -1;
    if (valid) {
      const int e0 = p.topk_ids[a];
      e = (a % K >= S) ? s_remap[e0] : e0;
    }
    int rank = 0, same = 0;
    for (int j = 0; j < kWave; ++j) {
      const int ej = __builtin_amdgcn_readlane(e, j);
      const int eq = (ej == e) ? 1 : 0;
      same += eq;
      rank += (j < lane) ? eq : 0;
    }
    if (valid && rank == 0) s_round[wave][e] = same;
    __syncthreads();
    if (valid) {
      int pos = s_cursor[e] + rank;
      for (int w = 0; w < wave; ++w) pos += s_round[w][e];
      p.sorted_token[pos] = a / K;
      p.sorted_slot[pos] = a % K;
      p.slot_pos[a] = pos;
    }
    __syncthreads();
    if (is_e && tid < M) {
      int add = 0;
      for (int w = 0; w < kRouteWaves; ++w) {
        add += s_round[w][tid];
        s_round[w][tid] = 0;
      }
      s_cursor[tid] += add;
    }
    __syncthreads();
  }
}

}  // namespace sere
