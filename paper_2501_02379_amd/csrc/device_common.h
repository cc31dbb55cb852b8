// Device helpers shared by the kernel files: element loads for the two gradient
// storage types and the float32 selection key.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tgrad_internal.h"

namespace tgrad {

constexpr int kWave = 64;

// One complex element as (re, im) float32.  DT = TGRAD_C64: interleaved float32 pairs.
// DT = TGRAD_CBF16: interleaved bfloat16 pairs; a bf16 is the upper half of a float32, so
// widening is exact (re sits in the low 16 bits of the little-endian 32-bit word).
template <int DT>
__device__ __forceinline__ float2 load_elem(const void* g, int64_t i) {
  if constexpr (DT == TGRAD_C64) {
    return reinterpret_cast<const float2*>(g)[i];
  } else {
    uint32_t raw = reinterpret_cast<const uint32_t*>(g)[i];
    return make_float2(__uint_as_float(raw << 16), __uint_as_float(raw & 0xFFFF0000u));
  }
}

// Elements 2p and 2p+1 with one vector load (the pair is 16-byte / 8-byte aligned because
// the tensor base is).  The caller guarantees 2p + 1 < I.
template <int DT>
__device__ __forceinline__ void load_pair(const void* g, int64_t p, float2& e0, float2& e1) {
  if constexpr (DT == TGRAD_C64) {
    float4 v = reinterpret_cast<const float4*>(g)[p];
    e0 = make_float2(v.x, v.y);
    e1 = make_float2(v.z, v.w);
  } else {
    uint2 v = reinterpret_cast<const uint2*>(g)[p];
    e0 = make_float2(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u));
    e1 = make_float2(__uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u));
  }
}

// Selection key |g|^2 = fl(fl(re*re) + fl(im*im)) in float32, one rounding per operation (the
// _rn intrinsics are never contracted into a fused multiply-add).  Non-negative floats order
// like their bit patterns, so the key is compared as an unsigned integer.
__device__ __forceinline__ uint32_t select_key(float2 e) {
  return __float_as_uint(__fadd_rn(__fmul_rn(e.x, e.x), __fmul_rn(e.y, e.y)));
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Number of set bits of `b` strictly below this lane.
__device__ __forceinline__ int popc_below(uint64_t b, int lane) {
  return __popcll(b & ((1ull << lane) - 1ull));
}

}  // namespace tgrad
