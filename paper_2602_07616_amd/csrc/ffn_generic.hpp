// Grouped expert FFN on the vector ALU (any dtype, any tokens-per-expert) and
// the weighted combine.  Expert equations: appendix "Preliminaries on MoEs"
// (E(x) = (silu(x W_gate) * (x W_up)) W_down, y = sum_i P_i E_i(x)).
//
// A "work item" is one surviving expert (or one shared expert) together with
// the rows [off, off+cnt) of the expert-sorted slot list that it must serve.
// The number of items is only known on the device, so every grid is sized for
// the worst case and blocks beyond n_work leave at once.
#pragma once

#include "common.hpp"

namespace sere {

struct FfnArgs {
  const void* hidden;          // [T, dh]
  const void* w_gate_up;       // [M, 2*dm, dh]
  const void* w_down;          // [M, dh, dm]
  const void* shared_gate_up;  // [n_sh, 2*dm, dh]
  const void* shared_down;     // [n_sh, dh, dm]
  const int32_t* sorted_token; // [R] token of each sorted row (R = A + n_sh*T)
  const int32_t* work_expert;
  const int32_t* work_off;
  const int32_t* work_cnt;
  const int32_t* n_work;
  float* h;                    // silu(gate) * up: [R, dm] fp32, or bf16 plane(s) [R, dm] on the bf16 path
  float* y;                    // [ksplit, R, dh] fp32 partial down projections
  int T, dh, dm, M, K, n_sh;
  int ksplit;                  // slices of dm in the down projection
  int rows;                    // R
  int split_h;                 // bf16 path: h carried as a high and a low bf16 plane
};

template <int DT>
__device__ __forceinline__ const void* expert_base(const void* routed, const void* shared, int e,
                                                   int M, size_t per_expert_elems) {
  const char* b = static_cast<const char*>(e < M ? routed : shared);
  return b + static_cast<size_t>(e < M ? e : e - M) * per_expert_elems * Store<DT>::bytes;
}

constexpr int kGenTok = 8;   // tokens served per pass over a weight row
constexpr int kGenJB = 16;   // intermediate indices per block (gate/up)
constexpr int kGenRB = 16;   // output rows per block (down)

constexpr int kGenPerWave = kGenJB / 4;  // weight rows a wavefront serves at a time (gate/up: pairs of rows)
static_assert(kGenJB == kGenRB && kGenJB % 4 == 0, "four wavefronts share a block's rows evenly");

// h[row, j] = silu(<Wg_j, x>) * <Wu_j, x>.  grid (ceil(dm/kGenJB), max items), 256 threads.
// A wavefront serves kGenPerWave intermediate indices and kGenTok token rows per pass; all loads
// of a pass are issued together and unconditionally (token slots beyond the item's rows repeat
// its first row and are never stored, indices beyond d_m repeat the last one): a load under a
// condition is waited for on its own, and on a layer this small the kernel is nothing but
// load latencies.
template <int DT>
__global__ __launch_bounds__(256) void ffn_gateup_generic(FfnArgs p) {
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const int dh = p.dh, dm = p.dm;
  const void* W = expert_base<DT>(p.w_gate_up, p.shared_gate_up, e, p.M, static_cast<size_t>(2) * dm * dh);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j0 = blockIdx.x * kGenJB + wave * kGenPerWave;
  if (j0 >= dm) return;
  for (int tc = 0; tc < cnt; tc += kGenTok) {
    const int nt = min(kGenTok, cnt - tc);
    int tok[kGenTok];
#pragma unroll
    for (int q = 0; q < kGenTok; ++q) tok[q] = p.sorted_token[off + tc + (q < nt ? q : 0)];
    float ag[kGenPerWave][kGenTok], au[kGenPerWave][kGenTok];
#pragma unroll
    for (int jj = 0; jj < kGenPerWave; ++jj)
#pragma unroll
      for (int q = 0; q < kGenTok; ++q) ag[jj][q] = au[jj][q] = 0.0f;
    for (int i = lane * 8; i < dh; i += 512) {
      float xv[kGenTok][8], wg[kGenPerWave][8], wu[kGenPerWave][8];
#pragma unroll
      for (int jj = 0; jj < kGenPerWave; ++jj) {
        const int j = min(j0 + jj, dm - 1);
        load8<DT>(W, static_cast<size_t>(j) * dh + i, wg[jj]);
        load8<DT>(W, static_cast<size_t>(dm + j) * dh + i, wu[jj]);
      }
#pragma unroll
      for (int q = 0; q < kGenTok; ++q) load8<DT>(p.hidden, static_cast<size_t>(tok[q]) * dh + i, xv[q]);
#pragma unroll
      for (int jj = 0; jj < kGenPerWave; ++jj)
#pragma unroll
        for (int q = 0; q < kGenTok; ++q)
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            ag[jj][q] = fmaf(wg[jj][c], xv[q][c], ag[jj][q]);
            au[jj][q] = fmaf(wu[jj][c], xv[q][c], au[jj][q]);
          }
    }
#pragma unroll
    for (int jj = 0; jj < kGenPerWave; ++jj)
#pragma unroll
      for (int q = 0; q < kGenTok; ++q) {
        const float g = wave_sum(ag[jj][q]), u = wave_sum(au[jj][q]);
        if (lane == 0 && q < nt && j0 + jj < dm) p.h[static_cast<size_t>(off + tc + q) * dm + j0 + jj] = silu(g) * u;
      }
  }
}

// y[row, r] = <Wd_r, h[row]>.  grid (ceil(dh/kGenRB), max items), 256 threads; built like the
// gate/up kernel.
template <int DT>
__global__ __launch_bounds__(256) void ffn_down_generic(FfnArgs p) {
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const int dh = p.dh, dm = p.dm;
  const void* W = expert_base<DT>(p.w_down, p.shared_down, e, p.M, static_cast<size_t>(dh) * dm);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r0 = blockIdx.x * kGenRB + wave * kGenPerWave;
  if (r0 >= dh) return;
  for (int tc = 0; tc < cnt; tc += kGenTok) {
    const int nt = min(kGenTok, cnt - tc);
    float acc[kGenPerWave][kGenTok];
#pragma unroll
    for (int rr = 0; rr < kGenPerWave; ++rr)
#pragma unroll
      for (int q = 0; q < kGenTok; ++q) acc[rr][q] = 0.0f;
    for (int j = lane * 8; j < dm; j += 512) {
      float hv[kGenTok][8], wd[kGenPerWave][8];
#pragma unroll
      for (int rr = 0; rr < kGenPerWave; ++rr)
        load8<DT>(W, static_cast<size_t>(min(r0 + rr, dh - 1)) * dm + j, wd[rr]);
#pragma unroll
      for (int q = 0; q < kGenTok; ++q)
        load8<SERE_F32>(p.h, static_cast<size_t>(off + tc + (q < nt ? q : 0)) * dm + j, hv[q]);
#pragma unroll
      for (int rr = 0; rr < kGenPerWave; ++rr)
#pragma unroll
        for (int q = 0; q < kGenTok; ++q)
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[rr][q] = fmaf(wd[rr][c], hv[q][c], acc[rr][q]);
    }
#pragma unroll
    for (int rr = 0; rr < kGenPerWave; ++rr)
#pragma unroll
      for (int q = 0; q < kGenTok; ++q) {
        const float v = wave_sum(acc[rr][q]);
        if (lane == 0 && q < nt && r0 + rr < dh) p.y[static_cast<size_t>(off + tc + q) * dh + r0 + rr] = v;
      }
  }
}

struct CombineArgs {
  const float* y;            // [ksplit, R, dh]
  const float* topk_w;       // [T, K]
  const int32_t* slot_pos;   // [T*K]
  const void* residual;      // [T, dh] added to the sum (the layer's input), or NULL
  void* out;                 // [T, dh]
  int T, dh, K, n_sh, ksplit, rows;
};

// out[t, r] = sum_k W[t,k] * y[pos(t,k), r] + sum_s y[A + s*T + t, r] (+ residual[t, r]); slots
// in ascending k, then shared experts, then the residual; fp32, one rounding to the output dtype.
// grid ceil(dh/256) * T (a token's column blocks are neighbours), 256 threads.
template <int DT>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs p) {
  const int col_blocks = (p.dh + 255) / 256;
  const int r = static_cast<int>(blockIdx.x % col_blocks) * 256 + threadIdx.x;
  const int t = blockIdx.x / col_blocks;
  if (r >= p.dh) return;
  const size_t slice = static_cast<size_t>(p.rows) * p.dh;
  float acc = 0.0f;
  // Contributions are added in ascending order, eight at a time: the eight positions, then the
  // eight rows of y are requested together (one memory round trip each instead of one per
  // contribution), then the eight fused multiply-adds run in order.
  constexpr int kBatch = 8;
  auto add = [&](int count, auto&& pos_of, auto&& weight_of) {
    for (int k0 = 0; k0 < count; k0 += kBatch) {
      int pos[kBatch];
      float w[kBatch], v[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int k = min(k0 + j, count - 1);
        pos[j] = pos_of(k);
        w[j] = weight_of(k);
        v[j] = 0.0f;
      }
      for (int s = 0; s < p.ksplit; ++s) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) v[j] += p.y[s * slice + static_cast<size_t>(pos[j]) * p.dh + r];
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j)
        if (k0 + j < count) acc = fmaf(w[j], v[j], acc);
    }
  };
  add(p.K, [&](int k) { return p.slot_pos[t * p.K + k]; }, [&](int k) { return p.topk_w[t * p.K + k]; });
  const int A = p.T * p.K;
  add(p.n_sh, [&](int sh) { return A + sh * p.T + t; }, [](int) { return 1.0f; });
  if (p.residual != nullptr) {
    if (DT == SERE_F32)
      acc += static_cast<const float*>(p.residual)[static_cast<size_t>(t) * p.dh + r];
    else
      acc += bf16_to_f32(static_cast<const uint16_t*>(p.residual)[static_cast<size_t>(t) * p.dh + r]);
  }
  store1<DT>(p.out, static_cast<size_t>(t) * p.dh + r, acc);
}

}  // namespace sere
