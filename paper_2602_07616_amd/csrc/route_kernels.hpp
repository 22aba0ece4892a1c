// Routing kernels: router logits, ordered top-K + gate, and the batch-wide
// re-routing / compaction step.
//
// Paper anchors: router logits R(x) and the top-k gate of the appendix
// "Preliminaries on MoEs"; primary set, most-similar primary, re-routing
// condition and final set of Sec. 3.2.2 (Steps 1-3).  The appendix algorithm
// "CUDA-accelerated SERE" gives one thread to every (token, secondary slot)
// and lets each scan all M experts; here the scan is done once per secondary
// EXPERT (its result depends only on the expert and the primary mask), and the
// rewritten map is counted, prefix-summed and regrouped per expert by the
// same workgroup, in LDS.
//
// Two launches: (1) router logits, delivered per token as sorted lists of 16;
// (2) top-K per token as a merge of the list heads; the workgroup that finishes
// last (a ticket in global memory, cleared by launch 1) then runs the
// batch-wide step, so no third launch is needed.
#pragma once

#include "common.hpp"

namespace sere {

// ------------------------------------------------------------ wave helpers ---
// Value of lane (l ^ 1), (l ^ 2), mirrored inside 8, mirrored inside 16: four
// DPP exchanges that together reach every lane of a 16-lane row.
template <int STEP>
__device__ __forceinline__ uint32_t row_xchg(uint32_t v) {
  constexpr int ctrl = STEP == 0 ? 0xB1 : STEP == 1 ? 0x4E : STEP == 2 ? 0x141 : 0x140;
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), ctrl, 0xF, 0xF, true));
}
template <int STEP>
__device__ __forceinline__ double row_xchg(double v) {
  const uint64_t b = static_cast<uint64_t>(__double_as_longlong(v));
  const uint64_t r = (static_cast<uint64_t>(row_xchg<STEP>(static_cast<uint32_t>(b >> 32))) << 32) |
                     row_xchg<STEP>(static_cast<uint32_t>(b));
  return __longlong_as_double(static_cast<long long>(r));
}

// sum over the 16 lanes of a row; every lane of the row gets it
__device__ __forceinline__ double row_sum(double v) {
  v += row_xchg<0>(v);
  v += row_xchg<1>(v);
  v += row_xchg<2>(v);
  v += row_xchg<3>(v);
  return v;
}

// sum over the wavefront (rows through scalar registers); wave-uniform result.
// The association order is fixed, so equal inputs give bit-equal sums.
__device__ __forceinline__ double wave_sum_dpp(double v) {
  v = row_sum(v);
  const uint64_t b = static_cast<uint64_t>(__double_as_longlong(v));
  const int lo = static_cast<int>(b), hi = static_cast<int>(b >> 32);
  double r[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint64_t x = (static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readlane(hi, 16 * q))) << 32) |
                       static_cast<uint32_t>(__builtin_amdgcn_readlane(lo, 16 * q));
    r[q] = __longlong_as_double(static_cast<long long>(x));
  }
  return (r[0] + r[1]) + (r[2] + r[3]);
}

// Barrier that orders LDS traffic only: global stores issued earlier (results
// that nobody in this workgroup reads back) need not have completed.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// order-preserving map double -> uint64 (larger double <=> larger key; -0 == +0)
__device__ __forceinline__ uint64_t sortable_key(double v) {
  uint64_t b = static_cast<uint64_t>(__double_as_longlong(v));
  if (b == 0x8000000000000000ull) b = 0;
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_to_double(uint64_t k) {
  const uint64_t b = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
  return __longlong_as_double(static_cast<long long>(b));
}

// value of the lane D places further round in the 16-lane row (DPP row rotate)
template <int D>
__device__ __forceinline__ uint32_t row_rot(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x120 + D, 0xF, 0xF, true));
}
template <int D>
__device__ __forceinline__ void rank_step(uint64_t key, uint32_t id, uint32_t& rank) {
  const uint64_t okey = (static_cast<uint64_t>(row_rot<D>(static_cast<uint32_t>(key >> 32))) << 32) |
                        row_rot<D>(static_cast<uint32_t>(key));
  const uint32_t oid = row_rot<D>(id);
  rank += (okey > key || (okey == key && oid < id)) ? 1u : 0u;
  if constexpr (D < 15) rank_step<D + 1>(key, id, rank);
}

// ---------------------------------------------------------------------------
// Router logits in fp64, delivered as SORTED LISTS.  grid (ceil(M/16), T),
// 256 threads; wave w of block (bx, t) computes experts bx*16 + 4w .. +3 for
// token t, the four dot products interleaved.  Every logit is reduced in the
// same lane pattern, so bit-identical router rows give bit-identical logits
// (ties then resolve by index, as in exact arithmetic).  The block then ranks
// its 16 logits (larger first, equal: lower expert first) and writes them as
// order-preserving keys with their expert ids:
//   list_key[(t*L + bx)*16 + rank], list_id[(t*L + bx)*16 + rank],  L = gridDim.x;
// places of experts >= M hold key 0 (below every real key).
// Block (0,0) clears the int32 at clear_word.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void router_logits_kernel(
    const void* __restrict__ hidden, const void* __restrict__ router_w, uint64_t* __restrict__ list_key,
    uint8_t* __restrict__ list_id, int /*T: one workgroup row per token, see grid*/, int M, int dh,
    int32_t* clear_word) {
  __shared__ double s_logit[16];
  const int t = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (clear_word != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *clear_word = 0;
  const int e0 = blockIdx.x * 16 + wave * 4;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  // four 512-wide chunks per pass, all loads of a pass issued before any arithmetic
  // (the router weights come cold from HBM on every step; one round trip instead of four)
  for (int i0 = lane * 8; i0 < dh; i0 += 2048) {
    Raw8<DT> xr[4], wr[4][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int i = i0 + 512 * c;
      if (i < dh) {
        xr[c].load(hidden, static_cast<size_t>(t) * dh + i);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (e0 + q < M) wr[c][q].load(router_w, static_cast<size_t>(e0 + q) * dh + i);  // wave-uniform
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (i0 + 512 * c < dh) {
        float xv[8];
        xr[c].widen(xv);
        double xd[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) xd[j] = static_cast<double>(xv[j]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (e0 + q < M) {
            float wv[8];
            wr[c][q].widen(wv);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[q] = fma(xd[j], static_cast<double>(wv[j]), acc[q]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const double sum = wave_sum_dpp(acc[q]);
    if (lane == 0) s_logit[wave * 4 + q] = sum;
  }
  __syncthreads();
  if (threadIdx.x < 16) {  // one 16-lane row; the other rows of the wavefront idle
    const int e = blockIdx.x * 16 + threadIdx.x;
    const uint64_t key = e < M ? sortable_key(s_logit[threadIdx.x]) : 0ull;
    uint32_t rank = 0;
    rank_step<1>(key, static_cast<uint32_t>(e), rank);
    const size_t at = (static_cast<size_t>(t) * gridDim.x + blockIdx.x) * 16 + rank;
    list_key[at] = key;
    list_id[at] = static_cast<uint8_t>(e);
  }
}

// The same for batches of many tokens: a workgroup serves TB tokens with its 16 experts, so a
// router row is fetched once per TB tokens (at 2048 tokens the one-token kernel reads the
// router weights 2048 times from cache).  Wave w: experts bx*16 + 4w .. +3 x tokens
// by*TB .. +TB-1, one 512-wide chunk of the rows at a time.  Same lane pattern per logit as
// above.  grid (ceil(M/16), ceil(T/TB)), 256 threads.
template <int DT, int TB>
__global__ __launch_bounds__(256) void router_logits_tokens_kernel(
    const void* __restrict__ hidden, const void* __restrict__ router_w, uint64_t* __restrict__ list_key,
    uint8_t* __restrict__ list_id, int T, int M, int dh, int32_t* clear_word) {
  __shared__ double s_logit[TB][16];
  const int t0 = blockIdx.y * TB;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (clear_word != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *clear_word = 0;
  const int e0 = blockIdx.x * 16 + wave * 4;
  double acc[4][TB];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int b = 0; b < TB; ++b) acc[q][b] = 0.0;
  // passes of up to four 512-wide chunks, all loads of a pass issued before any arithmetic (the
  // router weights come cold from HBM on every step: one round trip per pass instead of one per chunk)
  constexpr int kChunks = TB <= 2 ? 4 : 2;
  for (int i0 = lane * 8; i0 < dh; i0 += 512 * kChunks) {
    Raw8<DT> xr[kChunks][TB], wr[kChunks][4];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int i = min(i0 + 512 * c, dh - 8);   // a chunk beyond d_h re-reads the row's end and is not used
#pragma unroll
      for (int b = 0; b < TB; ++b) xr[c][b].load(hidden, static_cast<size_t>(min(t0 + b, T - 1)) * dh + i);
#pragma unroll
      for (int q = 0; q < 4; ++q) wr[c][q].load(router_w, static_cast<size_t>(min(e0 + q, M - 1)) * dh + i);
    }
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      if (i0 + 512 * c < dh) {
        double wd[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float wv[8];
          wr[c][q].widen(wv);
#pragma unroll
          for (int j = 0; j < 8; ++j) wd[q][j] = static_cast<double>(wv[j]);
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
          float xv[8];
          xr[c][b].widen(xv);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const double xd = static_cast<double>(xv[j]);
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q][b] = fma(xd, wd[q][j], acc[q][b]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int b = 0; b < TB; ++b) {
      const double sum = wave_sum_dpp(acc[q][b]);
      if (lane == 0) s_logit[b][wave * 4 + q] = sum;
    }
  __syncthreads();
  if (threadIdx.x < 16 * TB) {  // one 16-lane row per token
    const int b = threadIdx.x >> 4, t = t0 + b;
    const int e = blockIdx.x * 16 + (threadIdx.x & 15);
    const uint64_t key = e < M ? sortable_key(s_logit[b][threadIdx.x & 15]) : 0ull;
    uint32_t rank = 0;
    rank_step<1>(key, static_cast<uint32_t>(e), rank);
    if (t < T) {
      const size_t at = (static_cast<size_t>(t) * gridDim.x + blockIdx.x) * 16 + rank;
      list_key[at] = key;
      list_id[at] = static_cast<uint8_t>(e);
    }
  }
}

// The same for batches of hundreds of tokens and more, where the logits are a dense contraction
// ([T x d_h] x [d_h x M]) and the vector ALU (fp64 FMAs plus the conversions around them) bounds
// the kernels above: the fp64 matrix cores (v_mfma_f64_16x16x4) multiply a tile of 16 tokens x 16
// experts, fed from registers.  A workgroup owns one tile; its four wavefronts take every fourth
// 32-wide chunk of d_h each, and their partial tiles are added in a fixed order through LDS.
// Lane l of a wavefront holds row l % 16 of both operands (a token, an expert) and, of every 32
// consecutive k, the eight from 8 (l / 16) on: one 128-bit load per operand and chunk feeds eight
// MFMAs (the order of k inside a sum is free as long as both operands agree).  Every logit is the
// same sequence of operations on its two rows, so bit-identical router rows still give
// bit-identical logits.  The result tile has lane l hold D[l / 16 + 4 r][l % 16], r = 0..3: with
// the tokens as rows, a 16-lane row of register r holds one token's 16 logits, which is what the
// ranking wants.  grid (ceil(M/16), ceil(T/16)), 256 threads.
typedef double route_f64x4 __attribute__((ext_vector_type(4)));
template <int DT>
__global__ __launch_bounds__(256) void router_logits_mfma_kernel(
    const void* __restrict__ hidden, const void* __restrict__ router_w, uint64_t* __restrict__ list_key,
    uint8_t* __restrict__ list_id, int T, int M, int dh, int32_t* clear_word) {
  __shared__ double s_part[4][4][kWave];  // [wavefront][register r][lane]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r16 = lane & 15, kq = lane >> 4;
  if (clear_word != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *clear_word = 0;
  const int t0 = blockIdx.y * 16, e0 = blockIdx.x * 16;
  // rows beyond T or M repeat the last one; their results are not stored
  const size_t xrow = static_cast<size_t>(min(t0 + r16, T - 1)) * dh + 8 * kq;
  const size_t wrow = static_cast<size_t>(min(e0 + r16, M - 1)) * dh + 8 * kq;
  route_f64x4 acc = {0.0, 0.0, 0.0, 0.0};
  const int nch = dh >> 5;  // 32-wide chunks; this wavefront takes chunks wave, wave + 4, ...
  constexpr int kAhead = 4; // chunks whose loads are issued together
  for (int c0 = wave; c0 < nch; c0 += 4 * kAhead) {
    Raw8<DT> xr[kAhead], wr[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const int c = min(c0 + 4 * u, nch - 1);  // a chunk beyond the row re-reads its end and is not used
      xr[u].load(hidden, xrow + 32 * static_cast<size_t>(c));
      wr[u].load(router_w, wrow + 32 * static_cast<size_t>(c));
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      if (c0 + 4 * u < nch) {  // wave-uniform
        float xv[8], wv[8];
        xr[u].widen(xv);
        wr[u].widen(wv);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(xv[j]), static_cast<double>(wv[j]), acc, 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) s_part[wave][r][lane] = acc[r];
  __syncthreads();
  // wavefront w finishes register w: tokens t0 + kq + 4 w, one per 16-lane row
  const double logit = ((s_part[0][wave][lane] + s_part[1][wave][lane]) + s_part[2][wave][lane]) + s_part[3][wave][lane];
  const int t = t0 + kq + 4 * wave, e = e0 + r16;
  const uint64_t key = e < M ? sortable_key(logit) : 0ull;
  uint32_t rank = 0;
  rank_step<1>(key, static_cast<uint32_t>(e), rank);
  if (t < T) {
    const size_t at = (static_cast<size_t>(t) * gridDim.x + blockIdx.x) * 16 + rank;
    list_key[at] = key;
    list_id[at] = static_cast<uint8_t>(e);
  }
}

// ---------------------------------------------------------------------------
// Ordered top-K and gate by merging the sorted lists.  LP (4, 8 or 16) adjacent
// lanes own one token, lane l of the group holds list l (all 16 entries, in
// registers).  K rounds: the group's arg-max over the list heads (log2 LP DPP
// exchanges; larger key wins, equal keys go to the lower expert id), the
// winning lane pops its head.  Gate = softmax over the K selected logits (fp64
// internally, stored fp32); lane l keeps the selected logits of ranks
// l, l + LP, ... (KS of them, K <= KS*LP).  `active` is false for a group
// without a token.  ids8 (may be NULL) receives the ids as bytes for the
// workgroup's own use.
// ---------------------------------------------------------------------------
template <int STEP>
__device__ __forceinline__ void argmax_step(uint64_t& key, uint32_t& idx) {
  const uint32_t ohi = row_xchg<STEP>(static_cast<uint32_t>(key >> 32));
  const uint32_t olo = row_xchg<STEP>(static_cast<uint32_t>(key));
  const uint32_t oidx = row_xchg<STEP>(idx);
  const uint64_t okey = (static_cast<uint64_t>(ohi) << 32) | olo;
  if (okey > key || (okey == key && oidx < idx)) {
    key = okey;
    idx = oidx;
  }
}

template <int LP>
__device__ __forceinline__ double group_sum(double v) {
  v += row_xchg<0>(v);
  v += row_xchg<1>(v);
  if constexpr (LP >= 8) v += row_xchg<2>(v);
  if constexpr (LP >= 16) v += row_xchg<3>(v);
  return v;
}

// KEEP (8 or 16, >= min(K, 16)): list entries held per lane; a sorted list cannot
// contribute more than K entries to the top K, so for K <= 8 half a list is enough.
template <int LP, int KS, int KEEP>
__device__ __forceinline__ void topk_merge(const uint64_t* __restrict__ list_key,
                                           const uint8_t* __restrict__ list_id, bool active, int nlists,
                                           int32_t* __restrict__ ids, float* __restrict__ w, uint8_t* ids8, int K) {
  const int l = threadIdx.x & (LP - 1);
  const bool has_list = active && l < nlists;
  static_assert(KEEP == 8 || KEEP == 16, "half a list or a whole one");
  uint64_t key[KEEP];
  uint32_t idw[4];  // expert ids, one byte each (the upper two words stay 0 for KEEP == 8)
  idw[0] = idw[1] = idw[2] = idw[3] = 0;
  if (has_list) {
    const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(list_key + static_cast<size_t>(l) * 16);
#pragma unroll
    for (int j = 0; j < KEEP / 2; ++j) {
      const ulonglong2 v = kp[j];
      key[2 * j] = v.x;
      key[2 * j + 1] = v.y;
    }
    if (KEEP == 16) {
      const uint4 iv = *reinterpret_cast<const uint4*>(list_id + static_cast<size_t>(l) * 16);
      idw[0] = iv.x; idw[1] = iv.y; idw[2] = iv.z; idw[3] = iv.w;
    } else {
      const uint2 iv = *reinterpret_cast<const uint2*>(list_id + static_cast<size_t>(l) * 16);
      idw[0] = iv.x; idw[1] = iv.y;
    }
  } else {
#pragma unroll
    for (int j = 0; j < KEEP; ++j) key[j] = 0;
  }
  double mysel[KS];
#pragma unroll
  for (int c = 0; c < KS; ++c) mysel[c] = 0.0;
  double top = 0.0;
  for (int k = 0; k < K; ++k) {
    uint64_t wkey = key[0];
    uint32_t wid = key[0] != 0 ? (idw[0] & 0xffu) : 0x7fffffffu;
    argmax_step<0>(wkey, wid);
    argmax_step<1>(wkey, wid);
    if constexpr (LP >= 8) argmax_step<2>(wkey, wid);
    if constexpr (LP >= 16) argmax_step<3>(wkey, wid);
    // every lane of the group now holds the winner; its owner pops
    if (key[0] != 0 && (idw[0] & 0xffu) == wid) {
#pragma unroll
      for (int j = 0; j < KEEP - 1; ++j) key[j] = key[j + 1];
      key[KEEP - 1] = 0;
      idw[0] = (idw[0] >> 8) | (idw[1] << 24);
      idw[1] = (idw[1] >> 8) | (idw[2] << 24);
      idw[2] = (idw[2] >> 8) | (idw[3] << 24);
      idw[3] >>= 8;
    }
    const double val = key_to_double(wkey);
    if (k == 0) top = val;
#pragma unroll
    for (int c = 0; c < KS; ++c)
      if (k == l + LP * c) mysel[c] = val;
    if (l == 0 && active) {
      // a device-scope store: with several workgroups the ids are read by another one of this launch
      __hip_atomic_store(ids + k, static_cast<int32_t>(wid), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ids8 != nullptr) ids8[k] = static_cast<uint8_t>(wid);
    }
  }
  double ex[KS];
  double part = 0.0;
#pragma unroll
  for (int c = 0; c < KS; ++c) {
    ex[c] = 0.0;
    if (LP * c < K) {  // uniform
      ex[c] = (l + LP * c < K) ? exp(mysel[c] - top) : 0.0;
      part += ex[c];
    }
  }
  const double denom = group_sum<LP>(part);
#pragma unroll
  for (int c = 0; c < KS; ++c)
    if (l + LP * c < K && active) w[l + LP * c] = static_cast<float>(ex[c] / denom);
}

// ---------------------------------------------------------------------------
// Batch-wide re-routing and compaction by ONE workgroup of 1024 threads.
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
  int32_t* work_expert;     // [max items] expert of each work item (M+s for shared expert s); experts
                            //             ascending, an expert's rows cut into items of <= kItemRows
  int32_t* work_off;        // [max items] first row of the item in the sorted list
  int32_t* work_cnt;        // [max items] rows of the item (1 .. kItemRows)
  int32_t* n_work;          // [2]: number of items; 1 if the FFN kernels are to cut them fine
  int fine_items;           // ... which they do while there are at most this many items
  int topk_threads;         // threads of a workgroup that take part in the top-K merge (256 or 1024)
  int item_rows;            // rows per work item: kItemRows, or twice that for batches with many rows per expert
};

constexpr int kRouteThreads = 1024;
constexpr int kTopkThreadsMulti = 256;   // threads of a workgroup that merge lists when several workgroups share the batch
constexpr int kTopkLoneThreads = 512;    // one workgroup serves the whole batch up to this many merging threads
                                         // (measured: 1024 threads on one compute unit take 14.5 us, four
                                         // workgroups of 256 take 11.6 us)
constexpr int kTopkMaxSmallGroups = 64;  // groups of 256 threads up to this many workgroups, of 1024 beyond
constexpr int kSimPrefetchMaxGroups = 8;  // workgroups of a top-K launch that all prefetch their similarity rows
constexpr int kRouteWaves = kRouteThreads / kWave;
constexpr int kItemRows = 32;                     // rows of the sorted slot list per FFN work item (RouteArgs::item_rows may double it)
constexpr int kIdsInLds = 4096;                   // slots whose ids a lone workgroup keeps in LDS

struct RouteShared {
  int cnt_b[SERE_MAX_EXPERTS];
  int cnt_a[SERE_MAX_EXPERTS];
  int prim[SERE_MAX_EXPERTS];
  int remap[SERE_MAX_EXPERTS];
  int scan_cnt[SERE_MAX_EXPERTS / kWave];
  int scan_act[SERE_MAX_EXPERTS / kWave];
  int scan_before[SERE_MAX_EXPERTS / kWave];
  int scan_items[SERE_MAX_EXPERTS / kWave];
  int cursor[SERE_MAX_EXPERTS];
  int round_cnt[kRouteWaves][SERE_MAX_EXPERTS];
  uint8_t ids8[kIdsInLds];
  int flag;
};

// Rows of sim are scanned by 16-lane rows of a wavefront: row group q = lane/16
// of wavefront w owns experts u = 4*w + q + 64*r (r = 0, 1, ...); lane i of the
// group reads sim[u][i], sim[u][i + 16], ...: a load instruction touches four
// 64-byte segments, and the arg-max of a row needs only the four in-row DPP
// exchanges.  NC (4, 8 or 16) bounds M <= 16*NC.  The first values of a lane
// are loaded up front, before it is known which experts are secondary at all,
// so that their latency hides behind the top-K.
template <int NC>
struct SimPrefetch {
  static constexpr int NR = NC / 4;              // rounds of 64 experts
  static constexpr int PR = NC == 16 ? 1 : NR;   // rounds fetched ahead (at most 16 values per lane)
  float v[PR * NC];
};
template <int NC>
__device__ __forceinline__ void prefetch_sim(const RouteArgs& p, SimPrefetch<NC>& pf, bool enabled = true) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int q = lane >> 4, i = lane & 15;
#pragma unroll
  for (int r = 0; r < SimPrefetch<NC>::PR; ++r) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int u = 4 * wave + q + 64 * r, v = i + 16 * c;
      pf.v[r * NC + c] = (enabled && p.reroute && u < p.M && v < p.M) ? p.sim[static_cast<size_t>(u) * p.M + v] : 0.0f;
    }
  }
}

// arg-max step over (similarity, index): larger similarity wins, equal goes to the lower index
template <int STEP>
__device__ __forceinline__ void simmax_step(float& sv, int& iv) {
  const float os = __uint_as_float(row_xchg<STEP>(__float_as_uint(sv)));
  const int oi = static_cast<int>(row_xchg<STEP>(static_cast<uint32_t>(iv)));
  if (os > sv || (os == sv && oi < iv)) {
    sv = os;
    iv = oi;
  }
}

template <bool IDS_IN_LDS, int NC>
__device__ __forceinline__ void route_phase(const RouteArgs& p, RouteShared& s, const SimPrefetch<NC>& pf,
                                            bool prefetched = true) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int M = p.M, K = p.K, S = p.S;
  const int A = p.T * K;
  // ids read from memory may be a caller's (sere_reroute): clamped into [0, M) so that an id outside
  // that range, a broken precondition, cannot send any access out of bounds
  // (device-scope loads: the ids may have been written by other workgroups of this launch)
  auto id_at = [&](int a) -> int {
    return IDS_IN_LDS ? static_cast<int>(s.ids8[a])
                      : min(max(__hip_atomic_load(p.topk_ids + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0), M - 1);
  };

  if (tid < SERE_MAX_EXPERTS) {
    s.cnt_b[tid] = 0;
    s.cnt_a[tid] = 0;
    s.prim[tid] = 0;
    s.remap[tid] = tid;
  }
  for (int i = tid; i < kRouteWaves * SERE_MAX_EXPERTS; i += kRouteThreads) (&s.round_cnt[0][0])[i] = 0;
  lds_barrier();

  // Step 1: activation histogram and primary mask (union of every token's top-S)
  for (int a = tid; a < A; a += kRouteThreads) {
    const int e = id_at(a);
    atomicAdd(&s.cnt_b[e], 1);
    if (a % K < S) s.prim[e] = 1;
  }
  lds_barrier();

  // Step 2: per secondary expert u (activated, not primary): most similar
  // primary v*.  Each lane keeps the first maximum of its own columns in
  // ascending order with strict '>' (start value (-inf, expert 0)); lanes are
  // merged preferring the larger similarity, then the lower index: together
  // the first maximum of an ascending scan, as the paper's algorithm finds it.
  // The expert is kept as critical iff rho > 0 and sim* < rho.
  if (p.reroute) {
    const int q = lane >> 4, i = lane & 15;
#pragma unroll
    for (int r = 0; r < SimPrefetch<NC>::NR; ++r) {
      const int u = 4 * wave + q + 64 * r;
      const bool sec = u < M && s.cnt_b[u] > 0 && !s.prim[u];
      if (__ballot(sec) == 0) continue;  // wave-uniform
      float bs = -INFINITY;
      int bv = 0;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int v = i + 16 * c;
        if (v < M) {
          float sv;
          if (r < SimPrefetch<NC>::PR && prefetched)   // prefetched: uniform over the workgroup
            sv = pf.v[(r < SimPrefetch<NC>::PR ? r : 0) * NC + c];
          else
            sv = sec ? p.sim[static_cast<size_t>(u) * M + v] : 0.0f;
          if (s.prim[v] && sv > bs) {
            bs = sv;
            bv = v;
          }
        }
      }
      simmax_step<0>(bs, bv);
      simmax_step<1>(bs, bv);
      simmax_step<2>(bs, bv);
      simmax_step<3>(bs, bv);
      if (sec && i == 0) s.remap[u] = (p.rho > 0.0f && bs < p.rho) ? u : bv;
    }
  }
  lds_barrier();

  // Step 3: rewrite secondary slots, count the new map
  for (int a = tid; a < A; a += kRouteThreads) {
    const int e = id_at(a);
    const int e2 = (a % K >= S) ? s.remap[e] : e;
    p.rerouted_ids[a] = e2;
    atomicAdd(&s.cnt_a[e2], 1);
  }
  lds_barrier();

  // inclusive scans over experts: slots (-> offsets), activity (-> active
  // count) and work items (an expert's rows are cut into items of at most
  // kItemRows rows, so that one long expert cannot hold up the FFN kernels);
  // inside each of the first four wavefronts by shuffles, across them through
  // four totals in LDS
  const bool is_e = tid < SERE_MAX_EXPERTS;
  const int my_cnt = (is_e && tid < M) ? s.cnt_a[tid] : 0;
  const int my_act = my_cnt > 0 ? 1 : 0;
  const int item_rows = p.item_rows;
  const int my_items = (my_cnt + item_rows - 1) / item_rows;
  int inc_cnt = my_cnt, inc_act = my_act, inc_items = my_items;
  if (is_e) {  // wave-uniform (waves 0-3)
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int uc = __shfl_up(inc_cnt, d, kWave), ua = __shfl_up(inc_act, d, kWave);
      const int ui = __shfl_up(inc_items, d, kWave);
      if (lane >= d) {
        inc_cnt += uc;
        inc_act += ua;
        inc_items += ui;
      }
    }
    if (lane == kWave - 1) {
      s.scan_cnt[wave] = inc_cnt;
      s.scan_act[wave] = inc_act;
      s.scan_items[wave] = inc_items;
    }
    const int nb = __popcll(__ballot(tid < M && s.cnt_b[tid] > 0));
    if (lane == 0) s.scan_before[wave] = nb;
  }
  lds_barrier();
  int n_after = 0, n_before = 0, n_items = 0;
#pragma unroll
  for (int w = 0; w < SERE_MAX_EXPERTS / kWave; ++w) {
    if (is_e && w < wave) {
      inc_cnt += s.scan_cnt[w];
      inc_items += s.scan_items[w];
    }
    n_after += s.scan_act[w];
    n_before += s.scan_before[w];
    n_items += s.scan_items[w];
  }
  if (is_e && tid < M) {
    const int off = inc_cnt - my_cnt;
    s.cursor[tid] = off;
    p.expert_offsets[tid] = off;
    p.count_before[tid] = s.cnt_b[tid];
    p.count_after[tid] = my_cnt;
    p.primary_mask[tid] = s.prim[tid];
    const int first = inc_items - my_items;
    // Items of 128 rows (prefill-sized batches): an expert with a few rows more than one item
    // holds is cut into items of about equal size (multiples of a 16-row tile) instead of a full
    // one and a remnant: its items then take about equally long, and as they are numbered next
    // to each other they stream the expert's weights side by side, the later one from cache.
    int per = item_rows;
    if (item_rows >= 4 * kItemRows && my_items >= 2 && my_items <= 4)
      per = ((my_cnt + my_items - 1) / my_items + 15) & ~15;
    for (int j = 0; j < my_items; ++j) {
      p.work_expert[first + j] = tid;
      p.work_off[first + j] = off + j * per;
      p.work_cnt[first + j] = min(per, my_cnt - j * per);
    }
  }
  const int sh_items = (p.T + item_rows - 1) / item_rows;  // per shared expert
  if (tid == 0) {
    p.expert_offsets[M] = A;
    p.num_active[0] = n_before;
    p.num_active[1] = n_after;
    p.n_work[0] = n_items + p.n_sh * sh_items;
    p.n_work[1] = (item_rows == kItemRows && n_items + p.n_sh * sh_items <= p.fine_items) ? 1 : 0;
  }
  for (int i = tid; i < p.n_sh * sh_items; i += kRouteThreads) {
    const int sh = i / sh_items, j = i % sh_items;
    p.work_expert[n_items + i] = M + sh;
    p.work_off[n_items + i] = A + sh * p.T + j * item_rows;
    p.work_cnt[n_items + i] = min(item_rows, p.T - j * item_rows);
  }
  for (int i = tid; i < p.n_sh * p.T; i += kRouteThreads) p.sorted_token[A + i] = i % p.T;
  lds_barrier();

  // Stable regrouping by expert: slots keep ascending (token, slot) order
  // inside each expert.  A round covers 1024 consecutive slots, one wavefront
  // per 64; rank inside the wavefront from ballots, rank across wavefronts
  // through the per-round table.
  for (int base = 0; base < A; base += kRouteThreads) {
    const int a = base + tid;
    const bool valid = a < A;
    int e = 0;
    if (valid) {
      const int e0 = id_at(a);
      e = (a % K >= S) ? s.remap[e0] : e0;
    }
    // lanes of this wavefront holding the same expert: intersect, over the 8
    // bits of e, the ballot of lanes that agree with this lane on that bit
    int rank = 0, same = 0;
    if (base + wave * kWave < A) {  // wave-uniform: this wavefront has slots
      uint64_t peers = __ballot(valid);
#pragma unroll
      for (int bit = 0; bit < 8; ++bit) {
        const bool set = (e >> bit) & 1;
        const uint64_t with = __ballot(set);
        peers &= set ? with : ~with;
      }
      same = __popcll(peers);
      rank = __popcll(peers & ((1ull << lane) - 1ull));
    }
    if (valid && rank == 0) s.round_cnt[wave][e] = same;
    lds_barrier();
    if (valid) {
      int pos = s.cursor[e] + rank;
      for (int w = 0; w < wave; ++w) pos += s.round_cnt[w][e];
      p.sorted_token[pos] = a / K;
      p.sorted_slot[pos] = a % K;
      p.slot_pos[a] = pos;
    }
    if (base + kRouteThreads < A) {  // another round follows: advance the cursors
      lds_barrier();
      if (is_e && tid < M) {
        int add = 0;
        for (int w = 0; w < kRouteWaves; ++w) {
          add += s.round_cnt[w][tid];
          s.round_cnt[w][tid] = 0;
        }
        s.cursor[tid] += add;
      }
      lds_barrier();
    }
  }
}

// Re-routing alone (indices in, indices out): grid 1, 1024 threads.
__global__ __launch_bounds__(kRouteThreads) void route_kernel(RouteArgs p) {
  __shared__ RouteShared s;
  SimPrefetch<16> pf;  // any M up to 256
  prefetch_sim(p, pf);
  route_phase<false>(p, s, pf);
}

// Top-K + gate (1024 / LP tokens per workgroup), then the batch-wide step by
// the workgroup that takes the last ticket.  With a single workgroup there is
// no ticket and the ids go from the top-K to the batch-wide step through LDS.
// grid ceil(T*LP/1024), 1024 threads; *ticket must be 0 at launch.
// LP = lanes per token >= number of lists (4, 8, 16); K <= KS*LP; KEEP >= min(K, 16).
template <int LP, int KS, int KEEP>
__global__ __launch_bounds__(kRouteThreads) void topk_route_kernel(const uint64_t* __restrict__ list_key,
                                                                   const uint8_t* __restrict__ list_id,
                                                                   int32_t* __restrict__ topk_ids,
                                                                   float* __restrict__ topk_w, int32_t* ticket,
                                                                   RouteArgs p) {
  __shared__ RouteShared s;
  constexpr int NC = LP;  // the similarity scan uses the same bound M <= 16*LP
  // tokens per workgroup: the first p.topk_threads threads merge lists (the host's choice: all 1024,
  // or 256 -- one wavefront per SIMD, the merge being bound by the vector ALU -- so that a batch
  // shared by several workgroups spreads over more compute units)
  const int group_tokens = p.topk_threads / LP;
  // The similarity rows are requested before the top-K so that their latency hides behind it.
  // Only the workgroup that runs the batch-wide step uses them, and which one that is is not
  // known yet: with a handful of workgroups every one of them asks (the lines come from L2), with
  // many the step is long anyway and the rows are loaded where they are needed instead.
  SimPrefetch<NC> pf;
  prefetch_sim(p, pf, gridDim.x <= kSimPrefetchMaxGroups);
  const int nlists = (p.M + 15) >> 4;
  const int t = blockIdx.x * group_tokens + threadIdx.x / LP;
  const bool lone = gridDim.x == 1 && p.T * p.K <= kIdsInLds;
  const bool in_group = static_cast<int>(threadIdx.x) < group_tokens * LP;
  const bool has = in_group && t < p.T;
  const int first_of_wave = blockIdx.x * group_tokens + (threadIdx.x >> 6) * (kWave / LP);
  if (static_cast<int>(threadIdx.x & ~63u) < group_tokens * LP && first_of_wave < p.T) {  // wave-uniform: the wavefront has a token
    const size_t tt = has ? t : 0;
    topk_merge<LP, KS, KEEP>(list_key + tt * nlists * 16, list_id + tt * nlists * 16, has, nlists, topk_ids + tt * p.K,
                       topk_w + tt * p.K, lone ? s.ids8 + tt * p.K : nullptr, p.K);
  }
  if (lone) {
    __syncthreads();
    route_phase<true>(p, s, pf);
    return;
  }
  if (gridDim.x > 1) {
#if SERE_FORMAL_HANDOFF
    // Ordered by the memory model: the barrier orders every thread's id stores before thread 0's
    // ticket, the ticket is a device-scope release (this workgroup's stores become visible) and
    // acquire (the last taker sees every earlier taker's), the second barrier hands that on to
    // the other threads.  On this multi-die part the release writes the L2 back and the acquire
    // invalidates it, which is what the default path avoids.
    __syncthreads();
    if (threadIdx.x == 0)
      s.flag = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == static_cast<int>(gridDim.x) - 1;
    __syncthreads();
    if (!s.flag) return;
#else
    // Fence-free hand-off.  What it rests on (gfx950, not the HIP memory model):
    //  - the ids were written with device-scope atomic stores, which the compiler emits as
    //    global stores with the sc1 bit: they write through this die's L2 to memory instead of
    //    staying dirty in it, and no compiler transformation may drop or merge them;
    //  - s_waitcnt vmcnt(0) (s_waitcnt(0) below waits on every counter) returns only after those
    //    stores have been acknowledged, i.e. have reached the point of coherence; gfx950 counts
    //    stores in vmcnt like loads (there is no separate store counter), and the builtin is a
    //    scheduling barrier for memory operations;
    //  - the ticket is a device-scope atomic add, performed at the point of coherence, so the
    //    workgroup that reads gridDim.x - 1 runs after every other workgroup's acknowledgement;
    //  - that workgroup reads the ids with device-scope atomic loads (sc1: they bypass its own
    //    die's L2, which may hold stale lines), and ONLY the ids: route_phase<false> must not
    //    read any other data written by this launch's other workgroups (it does not: the gate
    //    weights, for one, are never read back).
    // Two device-scope fences here cost this kernel several microseconds (an L2 write-back and
    // an invalidate on a part with one L2 per die).
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0)
      s.flag = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == static_cast<int>(gridDim.x) - 1;
    __syncthreads();
    if (!s.flag) return;
#endif
  } else {
    __syncthreads();
  }
  route_phase<false>(p, s, pf, gridDim.x <= kSimPrefetchMaxGroups);
}

}  // namespace sere
