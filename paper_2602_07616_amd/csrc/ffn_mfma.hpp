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
// r = 0..3.  The weights go from HBM to registers to the matrix cores and
// nowhere else; the token operand, which the four wavefronts of a workgroup
// share, is staged through LDS (below).
//
// Expert equations: appendix "Preliminaries on MoEs",
// E(x) = (silu(x W_gate) * (x W_up)) W_down.
#pragma once

#include <type_traits>

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
// every lane takes the value of the lane 8 places further round its 16-lane row
__device__ __forceinline__ u32x4 rotate8(u32x4 v) {
  u32x4 r;
#pragma unroll
  for (int c = 0; c < 4; ++c)
    r[c] = __builtin_amdgcn_update_dpp(0, static_cast<int>(v[c]), 0x128 /*row_ror:8*/, 0xF, 0xF, true);
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
// Work per workgroup: two cuts.  With few work items the grid is only a few workgroups per
// compute unit and one workgroup more on some compute units decides the kernel time, so the
// items are cut fine (half the weight rows per workgroup, twice the workgroups).  With many
// items the coarse cut wins: the token tile is staged into LDS once per workgroup, which per
// weight byte costs half as much there.  The routing step chooses per call (n_work[1]); the
// grid is sized for the fine cut; under the coarse cut the workgroups are renumbered along
// their linear id, so that those with work come first and the idle ones (about half) sit
// at the end of the grid, where they cost nothing but their launch.
constexpr int kGateUpJ = 4;    // intermediate indices per wavefront, fine cut: 4 gate + 4 up rows = the
                               // upper half of one tile (coarse: 8 + 8 = one tile)
constexpr int kDownRows = 16;  // output rows per wavefront, fine cut: one tile (coarse: two tiles)
constexpr int kFineCutBlocks = 2560;  // fine cut while the coarse gate/up grid would hold at most this many
                                      // working workgroups (ten per compute unit)
constexpr int kWavesPerBlock = 4;

// The token operand (hidden states for gate/up, h for down) is shared by the
// wavefronts of a workgroup (four; eight in the kernels for prefill-sized
// batches) and staged through LDS in k chunks, double buffered: all threads of
// the workgroup copy a chunk of all token rows with 128-bit loads while
// the previous chunk is being multiplied; lane (g, n) then reads its MFMA
// operand straight from LDS (row n, k offset 16g: chunk 2g for A_even, 2g+1
// for A_odd).  A row of the LDS tile is padded by 16 bytes, which spreads the
// rows over the banks but does not make these reads conflict-free: measured, a
// 128-bit LDS read on gfx950 serves lanes {0-3, 12-15, 20-23, 24-27} of each half
// of the wavefront together and {4-7, 8-11, 16-19, 28-31} together (64 banks), and
// under that grouping every operand read keeps a two-way conflict whatever the
// padding.  A layout without conflicts (unpadded rows, 16-byte pieces stored at
// position p ^ F(row & 15) with a suitable F) was built and verified with the
// conflict counter, and made no kernel faster: the LDS is not what these
// kernels wait for.

// geometry of one staging configuration
template <int NT, int KC, int BT = 256>
struct Stage {
  static constexpr int kRows = NT * kTile;           // token rows held
  static constexpr int kRowBytes = KC * 2 + 16;      // padded LDS row
  static constexpr int kBufBytes = kRows * kRowBytes;
  static constexpr int kPiecesPerRow = KC / 8;       // 16-byte pieces
  static constexpr int kPerThread = kRows * kPiecesPerRow / BT;
  static_assert(kPerThread >= 1 && kRows * kPiecesPerRow % BT == 0, "chunk must split over the workgroup's threads");
};
// the largest configuration (eight token tiles, 64-wide chunks), two buffers
constexpr int kStageLdsBytes = 2 * Stage<8, 64>::kBufBytes;
// the kernels for prefill-sized batches stage 128-wide chunks of up to eight token tiles, or
// 64-wide chunks of sixteen
constexpr int kWideLdsBytes = 2 * Stage<16, 64>::kBufBytes;
static_assert(kWideLdsBytes >= 2 * Stage<8, 128>::kBufBytes, "LDS budget");
static_assert(Stage<8, 64>::kBufBytes >= Stage<4, 128>::kBufBytes && Stage<8, 64>::kBufBytes >= Stage<2, 256>::kBufBytes,
              "LDS budget");

// Token rows of a group: row r (< nrows) of the group is row index[first + r]
// (or first + r if index is NULL) of a matrix with leading dimension ld.
struct TokenSource {
  const uint16_t* base;
  const int32_t* index;
  int first, nrows, ld;
};

// acc[a][t] += W_tile_a[16 x (kend-kbeg)] * tokens_t, for NA weight tiles and
// NT token tiles.
//   wx[a], wy[a] : this lane's address in half tile X / Y of weight tile a at k = 0
//                  (row (i&7), chunk 2g + (i>>3))
//   rot          : chunk the workgroup starts with (the chunks are visited cyclically), so
//                  that concurrently running workgroups do not all hit the same offset
//                  inside their rows (and thus the same HBM channels)
//   lo_plane     : with LO, a second token operand `lo_plane` elements after the
//                  first is multiplied too (token = high + low bf16 parts)
// All BT threads of the workgroup must call this together (it has barriers).
// LDS_BYTES: size of the caller's LDS array (the staging configuration must fit it)
// BT       : threads of the workgroup (all of them stage, every wavefront multiplies every staged tile)
template <int NA, int NT, int KC, bool LO, bool HALF = false, int LDS_BYTES = kStageLdsBytes, int BT = 256>
__device__ __forceinline__ void stream_tiles(const uint16_t* const (&wx)[NA], const uint16_t* const (&wy)[NA],
                                             const TokenSource& tok, size_t lo_plane, int kbeg, int kend, int rot,
                                             unsigned char* lds, f32x4 (&acc)[NA][NT]) {
  using St = Stage<NT, KC, BT>;
  constexpr int KB = KC / 64;          // 64-wide k blocks per chunk
  constexpr int NP = LO ? 2 : 1;
  static_assert(NP * 2 * St::kBufBytes <= LDS_BYTES, "LDS budget");
  const int tid = threadIdx.x, lane = tid & 63;
  const int i = lane & 15, g = lane >> 4;
  const int len = kend - kbeg;
  const int nch = (len + KC - 1) / KC;

  // This thread's pieces of a chunk, the same for every chunk: ONE token row (256 / rows
  // threads share a row) and every kThreadsPerRow-th 16-byte piece of it, so that one row
  // address and compile-time strides describe them all.
  // Every load below is unconditional (rows beyond nrows re-read row 0, columns beyond kend
  // re-read the last valid ones; what they deliver is finite and never used): with loads
  // under branches the compiler can no longer count outstanding loads and waits for ALL of
  // them before every use, which would serialise the prefetch.
  constexpr int kThreadsPerRow = BT / St::kRows;
  static_assert(St::kPiecesPerRow % kThreadsPerRow == 0 && St::kPiecesPerRow / kThreadsPerRow == St::kPerThread,
                "a row's pieces must split evenly over its threads");
  const int srow = tid / kThreadsPerRow;
  const int col0 = (tid % kThreadsPerRow) * 8;  // elements; piece j sits kThreadsPerRow * 8 * j further
  const int dst0 = srow * St::kRowBytes + col0 * 2;
  const int srow_ok = srow < tok.nrows ? srow : 0;
  const uint16_t* src =
      tok.base + static_cast<size_t>(tok.index != nullptr ? tok.index[tok.first + srow_ok] : tok.first + srow_ok) * tok.ld;
  auto chunk_start = [&](int c) {
    int cc = c + rot;
    if (cc >= nch) cc -= nch;
    return kbeg + cc * KC;
  };
  u32x4 stage[NP][St::kPerThread];
  auto fetch_tokens = [&](int k0) {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int j = 0; j < St::kPerThread; ++j)
        stage[pl][j] = load_reused(src + pl * lo_plane + min(k0 + col0 + kThreadsPerRow * 8 * j, kend - 8));
  };
  auto store_tokens = [&](int buf) {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int j = 0; j < St::kPerThread; ++j)
        *reinterpret_cast<u32x4*>(lds + (buf * NP + pl) * St::kBufBytes + dst0 + kThreadsPerRow * 16 * j) = stage[pl][j];
  };
  // Weights: one register slot per 64-wide block of a chunk.  A block's next load (the same
  // block of the next chunk) is issued right after the block has been multiplied, so that a
  // wavefront always has a chunk's worth of weight loads in flight, each wait is for the one
  // oldest load, and nothing is loaded during the last chunk.
  u32x4 rx[NA][KB], ry[NA][KB];
  auto load_block = [&](int k0, int b) {
    const int kk = min(k0 + 64 * b, kend - 64);
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      rx[a][b] = load_weight(wx[a] + kk);
      if (!HALF) ry[a][b] = load_weight(wy[a] + kk);
    }
  };
  // token tiles whose operands are held at a time: all of them, or four when there are sixteen
  // (the accumulators alone are then 128 registers)
  constexpr int TG = NT > 8 ? 4 : NT;
  static_assert(NT % TG == 0, "token tiles are multiplied in equal groups");
  // (Issuing a slot's next load as soon as its weights have been merged into the MFMA operands,
  // i.e. before the block's MFMAs instead of after them, was measured slower: 1-2 % on the decode
  // layers, 5 % at 1024 tokens.)
  auto multiply_block = [&](int k0, int b, int buf) {
    if (k0 + 64 * b < kend) {  // wave-uniform; a block beyond kend holds a duplicate of the last one
      u32x4 a_even[NA], a_odd[NA];
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        // HALF: the tile's rows 8-15 are not used; they multiply whatever the lanes hold
        a_even[a] = HALF ? rx[a][b] : upper_from(rx[a][b], ry[a][b]);
        a_odd[a] = HALF ? rotate8(rx[a][b]) : lower_from(ry[a][b], rx[a][b]);
      }
#pragma unroll
      for (int t0 = 0; t0 < NT; t0 += TG) {
        u32x4 b_even[NP][TG], b_odd[NP][TG];
#pragma unroll
        for (int pl = 0; pl < NP; ++pl)
#pragma unroll
          for (int t = 0; t < TG; ++t) {
            const unsigned char* src = lds + (buf * NP + pl) * St::kBufBytes + ((t0 + t) * kTile + i) * St::kRowBytes +
                                       (64 * b + 16 * g) * 2;
            b_even[pl][t] = *reinterpret_cast<const u32x4*>(src);
            b_odd[pl][t] = *reinterpret_cast<const u32x4*>(src + 16);
          }
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int pl = 0; pl < NP; ++pl)
#pragma unroll
            for (int t = 0; t < TG; ++t) {
              acc[a][t0 + t] = mfma_bf16(a_even[a], b_even[pl][t], acc[a][t0 + t]);
              acc[a][t0 + t] = mfma_bf16(a_odd[a], b_odd[pl][t], acc[a][t0 + t]);
            }
      }
    }
  };

  if (nch > 0) {
    int k0 = chunk_start(0);
    fetch_tokens(k0);
#pragma unroll
    for (int b = 0; b < KB; ++b) load_block(k0, b);
    store_tokens(0);
    for (int c = 0; c + 1 < nch; ++c) {  // every pass of this loop has a next chunk to fetch
      __syncthreads();  // chunk c is in LDS; nobody still reads the other buffer
      const int k1 = chunk_start(c + 1);
      fetch_tokens(k1);
#pragma unroll
      for (int b = 0; b < KB; ++b) {
        multiply_block(k0, b, c & 1);
        load_block(k1, b);
      }
      store_tokens((c + 1) & 1);
      k0 = k1;
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < KB; ++b) multiply_block(k0, b, (nch - 1) & 1);
  }
  __syncthreads();  // the LDS buffers may be refilled by the caller's next group
}

// Which (work item, part of the item) this workgroup serves.  Fine cut: (blockIdx.y,
// blockIdx.x).  Coarse cut: an item has coarse_parts parts, numbered along the linear
// workgroup id.
struct BlockMap {
  int item, part;
};
__device__ __forceinline__ BlockMap map_block(bool fine, int coarse_parts) {
  if (fine) return BlockMap{static_cast<int>(blockIdx.y), static_cast<int>(blockIdx.x)};
  const unsigned id = blockIdx.y * gridDim.x + blockIdx.x;
  return BlockMap{static_cast<int>(id / coarse_parts), static_cast<int>(id % coarse_parts)};
}

// first chunk of a workgroup: spread over the row
// seed < 0: the workgroup's linear id
__device__ __forceinline__ int start_rotation(int len, int chunk, int seed = -1) {
  const int n = (len + chunk - 1) / chunk;
  if (n <= 1) return 0;
  const unsigned id = seed < 0 ? blockIdx.y * gridDim.x + blockIdx.x : static_cast<unsigned>(seed);
  return static_cast<int>((id * 5u) % static_cast<unsigned>(n));
}

// ---------------------------------------------------------------------------
// gate/up: a wavefront owns 8 intermediate indices j0..j0+7 of one work item
// over the full d_h, as ONE weight tile: rows 0-7 = the gate rows (half tile
// X), rows 8-15 = the matching up rows (half tile Y).  Lanes with g < 2 end
// with gate values, lanes g + 2 with the up values of the same (j, token);
// h = silu(gate) * up is stored as bf16 (plus, if split_h, the bf16 rounding
// residual in a second plane).
// ---------------------------------------------------------------------------
// j0 >= d_m (a wavefront beyond the last intermediate index of a wide workgroup): the wavefront
// still takes part in the staging, streams the last rows again and stores nothing.
template <int NT, int KC, bool HALF, int NA = 1, int LDS_BYTES = kStageLdsBytes, int BT = 256>
__device__ __forceinline__ void gateup_group(const FfnArgs& p, const uint16_t* W, int j0, int row0, int nrows,
                                             unsigned char* lds, int rot_seed = -1) {
  static_assert(!HALF || NA == 1, "the half-tile layout has one tile per wavefront");
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  const int chunk = 2 * g + (i >> 3);
  const bool live = j0 < dm;
  if (!live) j0 = dm - 8 * NA;
  // HALF: the one half tile holds gate rows j0..j0+3 (tile rows 0-3) and up rows (tile rows 4-7);
  // otherwise tile a holds gate rows j0 + 8a .. +7 (half tile X) and the matching up rows (Y)
  const uint16_t* wx[NA];
  const uint16_t* wy[NA];
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const int xrow = HALF ? ((i & 4) ? dm + j0 + (i & 3) : j0 + (i & 3)) : j0 + 8 * a + (i & 7);
    wx[a] = W + static_cast<size_t>(xrow) * dh + 8 * chunk;
    wy[a] = W + static_cast<size_t>(dm + j0 + 8 * a + (i & 7)) * dh + 8 * chunk;
  }
  const TokenSource tok{static_cast<const uint16_t*>(p.hidden), p.sorted_token, row0, nrows, dh};
  f32x4 acc[NA][NT];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[a][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_tiles<NA, NT, KC, false, HALF, LDS_BYTES, BT>(wx, wy, tok, 0, 0, dh, start_rotation(dh, KC, rot_seed), lds, acc);
  if (!live) return;

  // gate values sit in lanes g < GL, the up values of the same (j, token) GL * 16 lanes higher
  constexpr int GL = HALF ? 1 : 2;
  uint16_t* h = reinterpret_cast<uint16_t*>(p.h);
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x4 up;
#pragma unroll
      for (int r = 0; r < 4; ++r) up[r] = __shfl(acc[a][t][r], (lane + 16 * GL) & 63, kWave);
      const int n = t * kTile + i;
      if (g < GL && n < nrows) {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float hv = silu(acc[a][t][r]) * up[r];
          hi[r] = f32_to_bf16(hv);
          lo[r] = f32_to_bf16(hv - bf16_to_f32(hi[r]));
        }
        const size_t at = static_cast<size_t>(row0 + n) * dm + j0 + 8 * a + 4 * g;
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

// grid (dm / (4 WAVES), max items), 64 WAVES threads: WAVES wavefronts x 4 (fine) or 8 (coarse)
// intermediate indices.  WAVES = 4, or 8 for batches with a dozen rows per expert and more: the
// staged token tile then serves twice the weight rows (measured with 8: 4 % faster at 16 rows per
// expert on average, 3 % slower at 8).
template <int WAVES>
__global__ __launch_bounds__(64 * WAVES, 16 / WAVES) void ffn_gateup_mfma(FfnArgs p) {
  constexpr int BT = 64 * WAVES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[kStageLdsBytes];
  const int2 nw = *reinterpret_cast<const int2*>(p.n_work);  // items, fine cut?
  const bool fine = nw.y != 0;
  const BlockMap at = map_block(fine, gridDim.x / 2);
  const int w = at.item;
  if (w >= nw.x) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_gate_up, p.shared_gate_up, e, p.M, static_cast<size_t>(2) * p.dm * p.dh));
  const int wave = threadIdx.x >> 6;
  // the routing step cuts experts into items of at most 32 rows; longer items (the
  // similarity estimation's) are served 32 rows at a time, streaming the weights again
  if (fine) {
    const int j0 = (at.part * WAVES + wave) * kGateUpJ;
    if (cnt <= kTile) {
      gateup_group<1, 512, true, 1, kStageLdsBytes, BT>(p, W, j0, off, cnt, lds);
    } else {
      for (int q = 0; q < cnt; q += 2 * kTile) gateup_group<2, 256, true, 1, kStageLdsBytes, BT>(p, W, j0, off + q, min(2 * kTile, cnt - q), lds);
    }
  } else {
    const int j0 = (at.part * WAVES + wave) * (2 * kGateUpJ);
    if (cnt <= kTile) {
      gateup_group<1, 256, false, 1, kStageLdsBytes, BT>(p, W, j0, off, cnt, lds);
    } else {
      // long items (many tokens per expert): 128, 64 or 32 rows per pass over the weights
      int q = 0;
      for (; cnt - q > 4 * kTile; q += 8 * kTile) gateup_group<8, 64, false, 1, kStageLdsBytes, BT>(p, W, j0, off + q, min(8 * kTile, cnt - q), lds);
      if (cnt - q > 2 * kTile) {
        gateup_group<4, 128, false, 1, kStageLdsBytes, BT>(p, W, j0, off + q, cnt - q, lds);
      } else if (q < cnt) {
        gateup_group<2, 256, false, 1, kStageLdsBytes, BT>(p, W, j0, off + q, cnt - q, lds);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// down: a wavefront owns 32 output rows (two weight tiles sharing the token
// operand h) x one slice of d_m of one work item.  With split_h the token
// operand is h_hi + h_lo (two MFMAs per weight fragment).  Partial results go
// to y[slice][row][r] (fp32).
// ---------------------------------------------------------------------------
template <int NA, int NT, int KC, bool LO, int LDS_BYTES = kStageLdsBytes, int BT = 256>
__device__ __forceinline__ void down_group(const FfnArgs& p, const uint16_t* W, int r0, int kbeg, int kend,
                                           int slice, int row0, int nrows, unsigned char* lds, int rot_seed = -1) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int dh = p.dh, dm = p.dm;
  const int chunk = 2 * g + (i >> 3);
  // a workgroup whose last wavefronts fall beyond d_h (d_h is a multiple of 64, not of 128)
  // still takes part in the staging; those wavefronts stream row block 0 again and store nothing
  const bool live = r0 < dh;
  const uint16_t* base = W + static_cast<size_t>((live ? r0 : 0) + (i & 7)) * dm + 8 * chunk;
  const uint16_t* wx[NA];
  const uint16_t* wy[NA];
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    wx[a] = base + static_cast<size_t>(16 * a) * dm;
    wy[a] = base + static_cast<size_t>(16 * a + 8) * dm;
  }
  const TokenSource tok{reinterpret_cast<const uint16_t*>(p.h), nullptr, row0, nrows, dm};
  f32x4 acc[NA][NT];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[a][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_tiles<NA, NT, KC, LO, false, LDS_BYTES, BT>(wx, wy, tok, static_cast<size_t>(p.rows) * dm, kbeg, kend,
                                                     start_rotation(kend - kbeg, KC, rot_seed), lds, acc);
  if (!live) return;
  float* y = p.y + static_cast<size_t>(slice) * p.rows * dh;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * kTile + i;
    if (n < nrows) {
      float* dst = y + static_cast<size_t>(row0 + n) * dh + r0 + 4 * g;
#pragma unroll
      for (int a = 0; a < NA; ++a) *reinterpret_cast<f32x4*>(dst + 16 * a) = acc[a][t];
    }
  }
}

// grid (ceil(dh / 64) * ksplit, max items), 256 threads: 4 wavefronts x 16 (fine) or 32 (coarse) output rows
__global__ __launch_bounds__(256, 4) void ffn_down_mfma(FfnArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kStageLdsBytes];
  const int2 nw = *reinterpret_cast<const int2*>(p.n_work);  // items, fine cut?
  const bool fine = nw.y != 0;
  const int coarse_slabs = (p.dh + 2 * kDownRows * kWavesPerBlock - 1) / (2 * kDownRows * kWavesPerBlock);
  const BlockMap at = map_block(fine, coarse_slabs * p.ksplit);
  const int w = at.item;
  if (w >= nw.x) return;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_down, p.shared_down, e, p.M, static_cast<size_t>(p.dh) * p.dm));
  const int slab = at.part / p.ksplit, slice = at.part % p.ksplit;
  const int wave = threadIdx.x >> 6;
  // this slice of d_m, in 64-wide blocks
  const int blocks = p.dm >> 6, per = (blocks + p.ksplit - 1) / p.ksplit;
  const int kbeg = min(slice * per, blocks) << 6, kend = min((slice + 1) * per, blocks) << 6;
  if (fine) {
    const int r0 = (slab * kWavesPerBlock + wave) * kDownRows;
    // a slice of d_m that ends half way through a 256-wide chunk (d_m = 1408: 5.5 chunks) is
    // streamed in 128-wide chunks instead: the partial chunk's loads cost as much as a full one's
    const bool half_tail = ((kend - kbeg) & 255) == 128;
    if (cnt <= kTile) {
      if (p.split_h) {
        down_group<1, 1, 256, true>(p, W, r0, kbeg, kend, slice, off, cnt, lds);
      } else if (half_tail) {
        down_group<1, 1, 128, false>(p, W, r0, kbeg, kend, slice, off, cnt, lds);
      } else {
        down_group<1, 1, 256, false>(p, W, r0, kbeg, kend, slice, off, cnt, lds);
      }
    } else {
      for (int q = 0; q < cnt; q += 2 * kTile) {
        if (p.split_h) {
          down_group<1, 2, 64, true>(p, W, r0, kbeg, kend, slice, off + q, min(2 * kTile, cnt - q), lds);
        } else if (half_tail) {
          down_group<1, 2, 128, false>(p, W, r0, kbeg, kend, slice, off + q, min(2 * kTile, cnt - q), lds);
        } else {
          down_group<1, 2, 256, false>(p, W, r0, kbeg, kend, slice, off + q, min(2 * kTile, cnt - q), lds);
        }
      }
    }
  } else {
    const int r0 = (slab * kWavesPerBlock + wave) * (2 * kDownRows);
    if (cnt <= kTile) {
      if (p.split_h) {
        down_group<2, 1, 128, true>(p, W, r0, kbeg, kend, slice, off, cnt, lds);
      } else {
        down_group<2, 1, 128, false>(p, W, r0, kbeg, kend, slice, off, cnt, lds);
      }
    } else {
      if (p.split_h) {
        for (int q = 0; q < cnt; q += 2 * kTile)
          down_group<2, 2, 64, true>(p, W, r0, kbeg, kend, slice, off + q, min(2 * kTile, cnt - q), lds);
      } else {
        // 64 rows per pass over the weights while more than 32 remain (128 rows per pass, one
        // weight tile per wavefront, measured slower here: 237 vs 211 us at 2048 tokens)
        int q = 0;
        for (; cnt - q > 4 * kTile; q += 4 * kTile)
          down_group<2, 4, 64, false>(p, W, r0, kbeg, kend, slice, off + q, 4 * kTile, lds);
        if (cnt - q > 2 * kTile) {
          down_group<2, 4, 64, false>(p, W, r0, kbeg, kend, slice, off + q, cnt - q, lds);
        } else if (q < cnt) {
          down_group<2, 2, 128, false>(p, W, r0, kbeg, kend, slice, off + q, cnt - q, lds);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Prefill-sized batches (every expert has many token rows): the same building
// blocks with squarer workgroup tiles.  Staging the token tile costs as much
// traffic from L2 as the weights themselves once the tile holds 128 rows, so a
// workgroup should cover as many weight rows per staged tile as it can hold
// accumulators for: two weight tiles per wavefront and eight (items of up to
// 128 rows) or sixteen (up to 256 rows) token tiles per pass.  The host launches
// these kernels instead of the ones above when the routing kernel cuts items
// of 64 rows or more; bf16 without the split h only.
// ---------------------------------------------------------------------------
constexpr int kWideGateUpJ = 16;  // intermediate indices per wavefront: two tiles of 8 gate + 8 up rows
constexpr int kWideDownRows = 32; // output rows per wavefront: two tiles

// k chunk per number of token tiles: the staged chunk must give each thread of the workgroup a piece,
// and two buffers of it must fit the LDS budget
constexpr int wide_chunk(int nt) { return nt == 1 ? 256 : (nt <= 8 ? 128 : 64); }

template <int NA, bool GATEUP, typename Fn>
__device__ __forceinline__ void wide_rows(int cnt, Fn&& pass) {
  // rows of the item: up to 256 in one pass (more than 128: sixteen token tiles); beyond that, passes
  // of 128 while more than 64 remain; then one pass of <= 64, <= 32 or <= 16
  if (cnt > 8 * kTile && cnt <= 16 * kTile) {
    pass(std::integral_constant<int, 16>{}, 0, cnt);
    return;
  }
  int q = 0;
  for (; cnt - q > 4 * kTile; q += 8 * kTile) pass(std::integral_constant<int, 8>{}, q, min(8 * kTile, cnt - q));
  const int rem = cnt - q;
  if (rem > 2 * kTile) {
    pass(std::integral_constant<int, 4>{}, q, rem);
  } else if (rem > kTile) {
    pass(std::integral_constant<int, 2>{}, q, rem);
  } else if (rem > 0) {
    pass(std::integral_constant<int, 1>{}, q, rem);
  }
}

// The hardware hands workgroups to the chip's 8 XCDs round-robin by linear workgroup id, and each
// XCD has an L2 of its own.  With the parts of a work item numbered along that id, the item's token
// rows (512 KB for 128 rows of d_h = 2048) are fetched into all eight L2s, and a batch of thousands
// of tokens does not fit any of them: measured at T = 2048, the gate/up kernel then moves twice the
// weights' bytes across the fabric.  This renumbering gives every XCD a contiguous range of the
// `total` working (item, part) pairs, so the parts of an item meet in one L2.  Ids >= total idle.
constexpr unsigned kXcds = 8;
__device__ __forceinline__ BlockMap map_block_per_xcd(unsigned items, unsigned parts, bool* idle) {
  const unsigned id = blockIdx.y * gridDim.x + blockIdx.x, total = items * parts;
  *idle = id >= total;
  const unsigned x = id % kXcds, q = total / kXcds, r = total % kXcds;
  const unsigned v = x * q + min(x, r) + id / kXcds;
  return BlockMap{static_cast<int>(v / parts), static_cast<int>(v % parts)};
}

// Workgroups of the wide kernels: 8 wavefronts, one workgroup per compute unit.  What bounds these
// kernels is the bytes a compute unit takes in per flop (weights from HBM plus staged token rows
// from L2, measured at about 30 GB/s per compute unit whatever the mix), so all eight wavefronts
// multiply the same staged token tiles, each with two weight tiles of its own: 256 weight rows per
// staged tile (four wavefronts: 128), and a work item holds up to 256 rows (sixteen token tiles, 128
// accumulator registers), so that an expert with that many rows streams its weights once.
constexpr int kWideItemRows = 16 * kTile;
constexpr int kWideThreads = 512;
constexpr int kWideWaves = kWideThreads / kWave;

// grid (ceil(dm / 128), max items), 512 threads
__global__ __launch_bounds__(kWideThreads, 1) void ffn_gateup_mfma_wide(FfnArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWideLdsBytes];
  bool idle;
  const BlockMap at = map_block_per_xcd(*p.n_work, gridDim.x, &idle);
  if (idle) return;
  const int w = at.item;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_gate_up, p.shared_gate_up, e, p.M, static_cast<size_t>(2) * p.dm * p.dh));
  const int j0 = (at.part * kWideWaves + (threadIdx.x >> 6)) * kWideGateUpJ;  // may lie beyond d_m
  wide_rows<2, true>(cnt, [&](auto nt, int q, int n) {
    constexpr int NT = decltype(nt)::value;
    gateup_group<NT, wide_chunk(NT), false, 2, kWideLdsBytes, kWideThreads>(p, W, j0, off + q, n, lds, at.part);
  });
}

// grid (ceil(dh / 256) * ksplit, max items), 512 threads
__global__ __launch_bounds__(kWideThreads, 1) void ffn_down_mfma_wide(FfnArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWideLdsBytes];
  bool idle;
  const BlockMap at = map_block_per_xcd(*p.n_work, gridDim.x, &idle);
  if (idle) return;
  const int w = at.item;
  const int e = p.work_expert[w], off = p.work_off[w], cnt = p.work_cnt[w];
  const uint16_t* W = static_cast<const uint16_t*>(
      expert_base<SERE_BF16>(p.w_down, p.shared_down, e, p.M, static_cast<size_t>(p.dh) * p.dm));
  const int slab = at.part / p.ksplit, slice = at.part % p.ksplit;
  const int r0 = (slab * kWideWaves + (threadIdx.x >> 6)) * kWideDownRows;  // may lie beyond d_h
  const int blocks = p.dm >> 6, per = (blocks + p.ksplit - 1) / p.ksplit;
  const int kbeg = min(slice * per, blocks) << 6, kend = min((slice + 1) * per, blocks) << 6;
  wide_rows<2, false>(cnt, [&](auto nt, int q, int n) {
    constexpr int NT = decltype(nt)::value;
    down_group<2, NT, wide_chunk(NT), false, kWideLdsBytes, kWideThreads>(p, W, r0, kbeg, kend, slice, off + q, n, lds,
                                                                           at.part);
  });
}

}  // namespace sere
