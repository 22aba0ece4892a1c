// Shared device helpers for the SERE decode library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sere.h"

// The kernels rest on gfx950 facts (wave64, the 16x16x32 bf16 MFMA and its lane layout, DPP row
// operations, and the cache behaviour of device-scope stores that the routing kernels' hand-off
// between workgroups uses): no other target may be built.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "this library is written for gfx950 (MI355X) only"
#endif

// 1: the hand-off of top-K ids between workgroups of one launch is ordered by the memory model
// itself (release on the ticket, acquire by the workgroup that takes the last one, both at device
// scope).  0 (default): the fence-free hand-off described at topk_route_kernel, which rests on
// gfx950's behaviour and is several microseconds faster.  Both give the same results; a second
// copy of the library is built with 1 and the tests compare the two.
#ifndef SERE_FORMAL_HANDOFF
#define SERE_FORMAL_HANDOFF 0
#endif

namespace sere {

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Element storage selected by the ABI dtype.
template <int DT>
struct Store;
template <>
struct Store<SERE_F32> {
  using type = float;
  static constexpr int bytes = 4;
};
template <>
struct Store<SERE_BF16> {
  using type = uint16_t;
  static constexpr int bytes = 2;
};

// Eight consecutive elements starting at element index idx (idx % 8 == 0,
// base 16-byte aligned) widened to fp32.
template <int DT>
__device__ __forceinline__ void load8(const void* base, size_t idx, float (&v)[8]);

template <>
__device__ __forceinline__ void load8<SERE_F32>(const void* base, size_t idx, float (&v)[8]) {
  const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
  float4 a = p[0], b = p[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

template <>
__device__ __forceinline__ void load8<SERE_BF16>(const void* base, size_t idx, float (&v)[8]) {
  const uint4 q = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
  v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
  v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
  v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
  v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
}

// The same eight elements kept as loaded (bf16: one 128-bit register group),
// to be widened later: lets many loads be in flight in few registers.
template <int DT>
struct Raw8;
template <>
struct Raw8<SERE_F32> {
  float4 a, b;
  __device__ __forceinline__ void load(const void* base, size_t idx) {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
    a = p[0];
    b = p[1];
  }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <>
struct Raw8<SERE_BF16> {
  uint4 q;
  __device__ __forceinline__ void load(const void* base, size_t idx) {
    q = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
  }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
  }
};

template <int DT>
__device__ __forceinline__ void store1(void* base, size_t idx, float v);
template <>
__device__ __forceinline__ void store1<SERE_F32>(void* base, size_t idx, float v) {
  static_cast<float*>(base)[idx] = v;
}
template <>
__device__ __forceinline__ void store1<SERE_BF16>(void* base, size_t idx, float v) {
  static_cast<uint16_t*>(base)[idx] = f32_to_bf16(v);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }

}  // namespace sere
