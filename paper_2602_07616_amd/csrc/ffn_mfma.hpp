// Grouped expert FFN for bf16 on the gfx950 matrix cores.
//
// The decode FFN is bound by streaming each surviving expert's weights from
// HBM once.  Two things decide how close a kernel gets to the HBM rate here:
// every load instruction must cover whole 128-byte lines, and the weight
// loads must be non-temporal (measured on the MI355X: 16 rows x 64 B per
// instruction tops out near 5.8 TB/s, 8 rows x 128 B non-temporal near
// 6.8 TB/s).  v_mfma_f32_16x16x32_bf16 wants, from lane l = 16*g + i, row i of
// a 16-row tile and 8 consecutive k (16 bytes): 64 B per row per instruction.
// So the weights are loaded as 8-row HALF tiles instead:
//
//   lane (g, i) loads row (i & 7), 16-byte chunk 2*g + (i >> 3) of a 64-wide
//   k block: 8 rows x one full 128-byte line each per instruction.
//
// Two half tiles X (tile rows 0-7) and Y (tile rows 8-15) then give two full
// MFMA operands with one DPP row rotation by 8 lanes each:
//
//   A_even = lanes i<8 of X | lanes i<8 of Y moved to i+8   (chunks 2g)
//   A_odd  = lanes i>=8 of X moved to i-8 | lanes i>=8 of Y (chunks 2g+1)
//
// and the token operand of lane (g, n) is 32 contiguous bytes of token n:
// chunk 2g for A_even, chunk 2g+1 for A_odd.  Both MFMAs accumulate into the
// same 16x16 tile (the order of k inside a dot product is free as long as both
// operands agree).  The accumulator of lane (g, n) holds D[4*g + r][n],
// r = 0..3.  No LDS, no barrier: a wavefront owns its tile from first load to
// store.
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

// streamed exactly once: non-temporal
__device__ __forceinline__ u32x4 load_weight(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ u32x4 load_reused(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

// lanes 8-15 of every 16-lane row take `other` from 8 lanes below; lanes 0-7 keep `keep`
__device__ __forceinline__ u32x4 upper_from(u32x4 keep, u32x4 other) {
  u32x4 r;
#pragma unroll
  for (int c = 0; c < 4; ++c)
    r[c] = __builtin_amdgcn_update_dpp(static_cast<int>(keep[c]), static_cast<int>(other[c]), 0x128 /*row_ror:8*/,
                                       0xF, 0xC, false);
  return r;
}
// lanes 0-7 of every 16-lane row take `other` from 8 lanes above; lanes 8-15 keep `keep`
__device__ __forceinline__ u32x4 lower_from(u32x4 keep, u32x4 other) {
  u32x4 r;
#pragma unroll
  for (int c = 0; c < 4; ++c)
    r[c] = __builtin_amdgcn_update_dpp(static_cast<int>(keep[c]), static_cast<int>(other[c]), 0x128 /*row_ror:8*/,
                                       0xF, 0x3, false);
  return r;
}

constexpr int kTile = 16;      // tokens per MFMA tile
constexpr int kGateUpJ = 8;    // intermediate indices per wavefront (8 gate rows + 8 up rows = one tile)
constexpr int kDownRows = 32;  // output rows per wavefront (two tiles)
constexpr int kWavesPerBlock = 4;

// The token operand is loaded the same way: half tile BX = tokens 0-7 of the
// tile, BY = tokens 8-15, lane (g, i) -> token (i & 7), chunk 2g + (i >> 3), so a
// load instruction again covers whole lines (8 tokens x 128 B); BY is skipped
// when the tile has at most 8 tokens.
struct TokenRows {
  const uint16_t* x;  // lane's address in half tile BX at k = 0, or NULL
  const uint16_t* y;  // same for BY
};

// acc[a][t] += W_tile_a[16 x (kend-kbeg)] * tokens_t, for NA weight tiles that
// share the token operand and NT token tiles.
//   wx[a], wy[a] : this lane's address in half tile X / Y of weight tile a at k = 0
//                  (row (i&7), chunk 2g + (i>>3))
//   lo_plane     : with LO, a second token operand `lo_plane` elements after the
//                  first is multiplied too (token = high + low bf16 parts)
//   rot          : multiple of 64 below kend-kbeg; the 64-wide k blocks are visited
//                  starting there and wrapping around, so that concurrently running
//                  wavefronts do not all hit the same offset inside their rows
template <int NA, int NT, int U, bool LO>
__device__ __forceinline__ void stream_tile(const uint16_t* const (&wx)[NA], const uint16_t* const (&wy)[NA],
                                            const TokenRows (&b)[NT], const bool (&need_y)[NT], size_t lo_plane,
                                            int kbeg, int kend, int rot, f32x4 (&acc)[NA][NT]) {
  const u32x4 zero = {0u, 0u, 0u, 0u};
  const int len = kend - kbeg;
  constexpr int NP = LO ? 2 : 1;  // planes of the token operand (high [, low])
  for (int k0 = 0; k0 < len; k0 += 64 * U) {
    u32x4 x[NA][U], y[NA][U], bx[NP][NT][U], by[NP][NT][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int off = k0 + 64 * u;
      if (off < len) {  // wave-uniform
        int kk = off + rot;
        if (kk >= len) kk -= len;
        kk += kbeg;
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          x[a][u] = load_weight(wx[a] + kk);
          y[a][u] = load_weight(wy[a] + kk);
        }
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            bx[pl][t][u] = b[t].x != nullptr ? load_reused(b[t].x + pl * lo_plane + kk) : zero;
            by[pl][t][u] = (need_y[t] && b[t].y != nullptr) ? load_reused(b[t].y + pl * lo_plane + kk) : zero;
          }
        }
      } else {
#pragma unroll
        for (int a = 0; a < NA; ++a) x[a][u] = y[a][u] = zero;
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
          for (int t = 0; t < NT; ++t) bx[pl][t][u] = by[pl][t][u] = zero;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      u32x4 b_even[NP][NT], b_odd[NP][NT];
#pragma unroll
      for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          b_even[pl][t] = upper_from(bx[pl][t][u], by[pl][t][u]);
          b_odd[pl][t] = lower_from(by[pl][t][u], bx[pl][t][u]);
        }
      }
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        const u32x4 a_even = upper_from(x[a][u], y[a][u]);
        const u32x4 a_odd = lower_from(y[a][u], x[a][u]);
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            acc[a][t] = mfma_bf16(a_even, b_even[pl][t], acc[a][t]);
            acc[a][t] = mfma_bf16(a_odd, b_odd[pl][t], acc[a][t]);
          }
        }
      }
    }
  }
}

// rows of the token operand for NT tiles starting at `first`; `nrows` valid rows, row stride `ld`
template <int NT>
__device__ __forceinline__ void token_rows(const uint16_t* base, const int32_t* index, int first, int nrows,
                                           int ld, TokenRows (&b)[NT], bool (&need_y)[NT]) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int chunk = 2 * g + (i >> 3);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int nx = t * kTile + (i & 7), ny = nx + 8;
    const int rx = nx < nrows ? (index != nullptr ? index[first + nx] : first + nx) : -1;
    const int ry = ny < nrows ? (index != nullptr ? index[first + ny] : first + ny) : -1;
    b[t].x = rx >= 0 ? base + static_cast<size_t>(rx) * ld + 8 * chunk : nullptr;
    b[t].y = ry >= 0 ? base + static_cast<size_t>(ry) * ld + 8 * chunk : nullptr;
    need_y[t] = nrows > t * kTile + 8;  // wave-uniform
  }
}

// starting k block of a wavefront: spread over the row so that the chip's
// wavefronts touch different offsets (and thus HBM channels) at any moment
__device__ __forceinline__ int start_rotation(int len) {
  const int n = len >> 6;
  if (n <= 1) return 0;
  const unsigned id = (blockIdx.y * gridDim.x + blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
  return static_cast<int>((id * 5u) % static_cast<unsigned>(n)) << 6;
}

// ---------------------------------------------------------------------------
// gate/up: a wavefront owns 8 intermediate indices j0..j0+7 of one work item
// over the full d_h, as ONE weight tile: rows 0-7 = the gate rows (half tile
// X), rows 8-15 = the matching up rows (half tile Y).  Lanes with g < 2 end
// with gate values, lanes g + 2 with the up values of the same (j, token);
// h = silu(gate) * up is stored as bf16 (plus, if split_h, the bf16 rounding
// residual in a second plane).  (Measured against a variant with a
// 16-row gate tile and a 16-row up tile per wavefront: this one keeps twice
// as many wavefronts in flight and is faster when few experts survive.)
// ---------------------------------------------------------------------------
template <int NT, int U>
__device__ __forceinline__ void gateup_group(const FfnArgs& p, const uint16_t* W, int j0, int row0, int nrows) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  const int chunk = 2 * g + (i >> 3);
  const uint16_t* wx[1] = {W + static_cast<size_t>(j0 + (i & 7)) * dh + 8 * chunk};
  const uint16_t* wy[1] = {W + static_cast<size_t>(dm + j0 + (i & 7)) * dh + 8 * chunk};
  TokenRows b[NT];
  bool need_y[NT];
  token_rows<NT>(static_cast<const uint16_t*>(p.hidden), p.sorted_token, row0, nrows, dh, b, need_y);
  f32x4 acc[1][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[0][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_tile<1, NT, U, false>(wx, wy, b, need_y, 0, 0, dh, start_rotation(dh), acc);

  uint16_t* h = reinterpret_cast<uint16_t*>(p.h);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    f32x4 up;
#pragma unroll
    for (int r = 0; r < 4; ++r) up[r] = __shfl(acc[0][t][r], (lane + 32) & 63, kWave);
    const int n = t * kTile + i;
    if (g < 2 && n < nrows) {
      uint16_t hi[4], lo[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float hv = silu(acc[0][t][r]) * up[r];
        hi[r] = f32_to_bf16(hv);
        lo[r] = f32_to_bf16(hv - bf16_to_f32(hi[r]));
      }
      const size_t at = static_cast<size_t>(row0 + n) * dm + j0 + 4 * g;
      uint2 packed;
      packed.x = static_cast<uint32_t>(hi[0]) | (static_cast<uint32_t>(hi[1]) << 16);
      packed.y = static_cast<uint32_t>(hi[2]) | (static_cast<uint32_t>(hi[3]) << 16);
      *reinterpret_cast<uint2*>(h + at) = packed;
      if (p.split_h) {
        packed.x = static_cast<uint32_t>(lo[0]) | (static_cast<uint32_t>(lo[1]) << 16);
        packed.y = static_cast<uint32_t>(lo[2]) | (static_cast<uint32_t>(lo[3]) << 16);
        *reinterpret_cast<uint2*>(h + static_cast<size_t>(p.rows) * dm + at) = packed;
      }
    }
  }
}

// grid (dm / 32, M + n_sh), 256 threads: 4 wavefronts x 8 intermediate indices
__global__ __launch_bounds__(256) void ffn_gateup_mfma(FfnArgs p) {
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_gate_up, p.shared_gate_up, e, p.M, static_cast<size_t>(2) * p.dm * p.dh));
  const int j0 = (blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * kGateUpJ;
  if (cnt <= kTile) {
    gateup_group<1, 4>(p, W, j0, off, cnt);
  } else if (cnt <= 2 * kTile) {
    gateup_group<2, 2>(p, W, j0, off, cnt);
  } else {
    for (int q = 0; q < cnt; q += 4 * kTile) gateup_group<4, 2>(p, W, j0, off + q, min(4 * kTile, cnt - q));
  }
}

// ---------------------------------------------------------------------------
// down: a wavefront owns 32 output rows (two weight tiles sharing the token
// operand h) x one slice of d_m of one work item.  With split_h the token
// operand is h_hi + h_lo (two MFMAs per weight fragment).  Partial results go
// to y[slice][row][r] (fp32).
// ---------------------------------------------------------------------------
template <int NT, int U, bool LO>
__device__ __forceinline__ void down_group(const FfnArgs& p, const uint16_t* W, int r0, int kbeg, int kend,
                                           int slice, int row0, int nrows) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  const int chunk = 2 * g + (i >> 3);
  const uint16_t* base = W + static_cast<size_t>(r0 + (i & 7)) * dm + 8 * chunk;
  const uint16_t* wx[2] = {base, base + static_cast<size_t>(16) * dm};
  const uint16_t* wy[2] = {base + static_cast<size_t>(8) * dm, base + static_cast<size_t>(24) * dm};
  TokenRows b[NT];
  bool need_y[NT];
  token_rows<NT>(reinterpret_cast<const uint16_t*>(p.h), nullptr, row0, nrows, dm, b, need_y);
  f32x4 acc[2][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[0][t] = acc[1][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_tile<2, NT, U, LO>(wx, wy, b, need_y, static_cast<size_t>(p.rows) * dm, kbeg, kend,
                            start_rotation(kend - kbeg), acc);
  float* y = p.y + static_cast<size_t>(slice) * p.rows * dh;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * kTile + i;
    if (n < nrows) {
      float* dst = y + static_cast<size_t>(row0 + n) * dh + r0 + 4 * g;
      *reinterpret_cast<f32x4*>(dst) = acc[0][t];
      *reinterpret_cast<f32x4*>(dst + 16) = acc[1][t];
    }
  }
}

// grid ((dh / 128) * ksplit, M + n_sh), 256 threads: 4 wavefronts x 32 output rows
__global__ __launch_bounds__(256) void ffn_down_mfma(FfnArgs p) {
  const int w = blockIdx.y;
  if (w >= *p.n_work) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_down, p.shared_down, e, p.M, static_cast<size_t>(p.dh) * p.dm));
  const int slab = blockIdx.x / p.ksplit, slice = blockIdx.x % p.ksplit;
  const int r0 = (slab * kWavesPerBlock + (threadIdx.x >> 6)) * kDownRows;
  if (r0 >= p.dh) return;  // d_h is a multiple of 64, not necessarily of 128
  // this slice of d_m, in 64-wide blocks
  const int blocks = p.dm >> 6, per = (blocks + p.ksplit - 1) / p.ksplit;
  const int kbeg = min(slice * per, blocks) << 6, kend = min((slice + 1) * per, blocks) << 6;
  if (p.split_h) {
    if (cnt <= kTile) {
      down_group<1, 4, true>(p, W, r0, kbeg, kend, slice, off, cnt);
    } else {
      for (int q = 0; q < cnt; q += 2 * kTile)
        down_group<2, 2, true>(p, W, r0, kbeg, kend, slice, off + q, min(2 * kTile, cnt - q));
    }
  } else if (cnt <= kTile) {
    down_group<1, 4, false>(p, W, r0, kbeg, kend, slice, off, cnt);
  } else if (cnt <= 2 * kTile) {
    down_group<2, 2, false>(p, W, r0, kbeg, kend, slice, off, cnt);
  } else {
    for (int q = 0; q < cnt; q += 4 * kTile)
      down_group<4, 2, false>(p, W, r0, kbeg, kend, slice, off + q, min(4 * kTile, cnt - q));
  }
}

}  // namespace sere
