// Grouped expert FFN for bf16 on the gfx950 matrix cores.
//
// The decode FFN is bound by streaming each surviving expert's weights from
// HBM once; v_mfma_f32_16x16x32_bf16 is used so that the arithmetic for up to
// 16 tokens per weight fragment costs one instruction and never competes with
// the loads.  Weights are the MFMA "A" operand straight from global memory:
// lane l supplies row (l % 16) of a 16-row tile, 8 consecutive bf16 (one
// 128-bit load) at column 8*(l / 16) of a 32-wide k-step.  Token data are the
// "B" operand with the same (row = token, 8 consecutive k) shape.  The
// accumulator of lane l holds D[4*(l/16) + r][l % 16], r = 0..3, i.e. four
// consecutive weight rows for token (l % 16).
//
// Expert equations: appendix "Preliminaries on MoEs",
// E(x) = (silu(x W_gate) * (x W_up)) W_down.
#pragma once

#include "common.hpp"
#include "ffn_generic.hpp"

namespace sere {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}

// streamed once: keep it out of the caches' way
__device__ __forceinline__ u32x4 load_weight(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ u32x4 load_reused(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

constexpr int kMfmaJB = 16;      // intermediate indices per gate/up block
constexpr int kMfmaRows = 64;    // output rows per down block (one 16-row tile per wave)
constexpr int kTile = 16;        // tokens per MFMA tile

// ---------------------------------------------------------------------------
// gate/up: one block = 16 intermediate indices (16 gate rows + 16 up rows) of
// one work item; its four waves split d_h.  Partial 16x16 tiles are summed
// through LDS, then h = silu(g) * u is stored as a bf16 high plane and a bf16
// low plane (h_hi + h_lo carries 16 mantissa bits).
// ---------------------------------------------------------------------------
template <int NT, int U>
__device__ __forceinline__ void gateup_accumulate(const uint16_t* wg, const uint16_t* wu,
                                                  const uint16_t* const (&xrow)[NT], int kbeg, int kend,
                                                  f32x4 (&accg)[NT], f32x4 (&accu)[NT]) {
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int k = kbeg; k < kend; k += 32 * U) {
    u32x4 ag[U], au[U], b[NT][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = k + 32 * u;
      if (kk < kend) {  // wave-uniform
        ag[u] = load_weight(wg + kk);
        au[u] = load_weight(wu + kk);
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t][u] = xrow[t] != nullptr ? load_reused(xrow[t] + kk) : zero;
      } else {
        ag[u] = au[u] = zero;
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t][u] = zero;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        accg[t] = mfma_bf16(ag[u], b[t][u], accg[t]);
        accu[t] = mfma_bf16(au[u], b[t][u], accu[t]);
      }
    }
  }
}

template <int NT, int U>
__device__ __forceinline__ void gateup_group(const FfnArgs& p, const uint16_t* W, int j0, int row0, int nrows,
                                             float* red) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  // this wave's share of d_h, in 32-wide steps
  const int steps = dh >> 5, per = (steps + 3) >> 2;
  const int kbeg = min(wave * per, steps) << 5, kend = min((wave + 1) * per, steps) << 5;

  const uint16_t* wg = W + static_cast<size_t>(j0 + i) * dh + 8 * g;
  const uint16_t* wu = W + static_cast<size_t>(dm + j0 + i) * dh + 8 * g;
  const uint16_t* xrow[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * kTile + i;
    xrow[t] = n < nrows ? static_cast<const uint16_t*>(p.hidden) +
                              static_cast<size_t>(p.sorted_token[row0 + n]) * dh + 8 * g
                        : nullptr;
  }
  f32x4 accg[NT], accu[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) accg[t] = accu[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  gateup_accumulate<NT, U>(wg, wu, xrow, kbeg, kend, accg, accu);

  // red[wave][m][t][lane] as float4, m = 0 gate, 1 up
  f32x4* red4 = reinterpret_cast<f32x4*>(red);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    red4[((wave * 2 + 0) * NT + t) * 64 + lane] = accg[t];
    red4[((wave * 2 + 1) * NT + t) * 64 + lane] = accu[t];
  }
  __syncthreads();
  uint16_t* h_hi = reinterpret_cast<uint16_t*>(p.h);
  uint16_t* h_lo = h_hi + static_cast<size_t>(p.rows) * dm;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    // thread -> element (lane l = tid / 4, r = tid % 4) of tile t
    const int l = threadIdx.x >> 2, r = threadIdx.x & 3;
    float gsum = 0.f, usum = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      gsum += red[(((q * 2 + 0) * NT + t) * 64 + l) * 4 + r];
      usum += red[(((q * 2 + 1) * NT + t) * 64 + l) * 4 + r];
    }
    const int n = t * kTile + (l & 15);
    const int j = j0 + 4 * (l >> 4) + r;
    if (n < nrows) {
      const float hv = silu(gsum) * usum;
      const uint16_t hi = f32_to_bf16(hv);
      const uint16_t lo = f32_to_bf16(hv - bf16_to_f32(hi));
      const size_t at = static_cast<size_t>(row0 + n) * dm + j;
      h_hi[at] = hi;
      h_lo[at] = lo;
    }
  }
  __syncthreads();  // red is reused by the next group
}

// grid (dm / 16, M + n_sh), 256 threads
__global__ __launch_bounds__(256) void ffn_gateup_mfma(FfnArgs p) {
  __shared__ float red[4 * 2 * 4 * 64 * 4];  // 4 waves x {gate,up} x up to 4 tiles x 64 lanes x 4
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_gate_up, p.shared_gate_up, e, p.M, static_cast<size_t>(2) * p.dm * p.dh));
  const int j0 = blockIdx.x * kMfmaJB;
  if (cnt <= kTile) {
    gateup_group<1, 8>(p, W, j0, off, cnt, red);
  } else if (cnt <= 2 * kTile) {
    gateup_group<2, 4>(p, W, j0, off, cnt, red);
  } else {
    for (int r0 = 0; r0 < cnt; r0 += 4 * kTile) gateup_group<4, 4>(p, W, j0, off + r0, min(4 * kTile, cnt - r0), red);
  }
}

// ---------------------------------------------------------------------------
// down: one block = 64 output rows x one slice of d_m of one work item; each
// wave owns a 16-row tile.  B = h (high and low plane, two MFMAs per weight
// fragment).  Partial results go to y[slice][row][r].
// ---------------------------------------------------------------------------
template <int NT, int U>
__device__ __forceinline__ void down_group(const FfnArgs& p, const uint16_t* W, int r0, int kbeg, int kend,
                                           int slice, int row0, int nrows) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  const uint16_t* wd = W + static_cast<size_t>(r0 + i) * dm + 8 * g;
  const uint16_t* h_hi = reinterpret_cast<const uint16_t*>(p.h);
  const size_t plane = static_cast<size_t>(p.rows) * dm;
  const uint16_t* hrow[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * kTile + i;
    hrow[t] = n < nrows ? h_hi + static_cast<size_t>(row0 + n) * dm + 8 * g : nullptr;
  }
  const u32x4 zero = {0u, 0u, 0u, 0u};
  f32x4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int k = kbeg; k < kend; k += 32 * U) {
    u32x4 a[U], bh[NT][U], bl[NT][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = k + 32 * u;
      if (kk < kend) {
        a[u] = load_weight(wd + kk);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          bh[t][u] = hrow[t] != nullptr ? load_reused(hrow[t] + kk) : zero;
          bl[t][u] = hrow[t] != nullptr ? load_reused(hrow[t] + plane + kk) : zero;
        }
      } else {
        a[u] = zero;
#pragma unroll
        for (int t = 0; t < NT; ++t) bh[t][u] = bl[t][u] = zero;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        acc[t] = mfma_bf16(a[u], bh[t][u], acc[t]);
        acc[t] = mfma_bf16(a[u], bl[t][u], acc[t]);
      }
    }
  }
  float* y = p.y + static_cast<size_t>(slice) * p.rows * dh;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * kTile + i;
    if (n < nrows) *reinterpret_cast<f32x4*>(y + static_cast<size_t>(row0 + n) * dh + r0 + 4 * g) = acc[t];
  }
}

// grid ((dh / 64) * ksplit, M + n_sh), 256 threads
__global__ __launch_bounds__(256) void ffn_down_mfma(FfnArgs p) {
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_down, p.shared_down, e, p.M, static_cast<size_t>(p.dh) * p.dm));
  const int slab = blockIdx.x / p.ksplit, slice = blockIdx.x % p.ksplit;
  const int wave = threadIdx.x >> 6;
  const int r0 = slab * kMfmaRows + wave * 16;
  const int steps = p.dm >> 5, per = (steps + p.ksplit - 1) / p.ksplit;
  const int kbeg = min(slice * per, steps) << 5, kend = min((slice + 1) * per, steps) << 5;
  if (cnt <= kTile) {
    down_group<1, 8>(p, W, r0, kbeg, kend, slice, off, cnt);
  } else if (cnt <= 2 * kTile) {
    down_group<2, 4>(p, W, r0, kbeg, kend, slice, off, cnt);
  } else {
    for (int q = 0; q < cnt; q += 4 * kTile)
      down_group<4, 2>(p, W, r0, kbeg, kend, slice, off + q, min(4 * kTile, cnt - q));
  }
}

}  // namespace sere
