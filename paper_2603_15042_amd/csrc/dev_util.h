// Device helpers: bf16 conversion, bf16 pair dot product, fixed-order reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN (quiet, payload kept); denormals kept.
// One v_cvt_pk_bf16_f32 per pair.  The instruction was checked on the device against the integer
// formulation ((u + 0x7fff + ((u >> 16) & 1)) >> 16, NaN: (u >> 16) | 0x40) for every 16-bit upper half
// with lower halves on both sides of the tie: no difference, NaN and denormal inputs included.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16(f, 0.f) & 0xffffu; }

// acc + w.lo*x.lo + w.hi*x.hi on two packed bf16 pairs (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w),
                                         __builtin_bit_cast(bf16x2_t, x), acc, false);
}
__device__ __forceinline__ float dot8_bf16(u32x4 w, u32x4 x, float acc) {
  acc = dot2_bf16(w.x, x.x, acc);
  acc = dot2_bf16(w.y, x.y, acc);
  acc = dot2_bf16(w.z, x.z, acc);
  acc = dot2_bf16(w.w, x.w, acc);
  return acc;
}

// Sum over the 64 lanes of a wave in one fixed butterfly (partner distance 32,
// 16, 8, 4, 2, 1).  fp32 addition is commutative, so every lane ends with the
// same bits, and those bits depend on nothing but the 64 inputs.
__device__ __forceinline__ float wave_sum(float v) {
  v += __shfl_xor(v, 32, 64);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 8, 64);
  v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 2, 64);
  v += __shfl_xor(v, 1, 64);
  return v;
}

// 128-bit global load / store of 8 bf16.
__device__ __forceinline__ u32x4 ld16(const uint16_t* p) {
  return *reinterpret_cast<const u32x4*>(p);
}
// Streaming variant for data read exactly once (weights): keeps it out of the
// way of the activations that are reused from cache.
__device__ __forceinline__ u32x4 ld16_stream(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void st16(uint16_t* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }

// (value, index) order used by the greedy token: larger value wins, equal values
// go to the lower index, NaN never wins.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
  return (v > bv) || (v == bv && i < bi);
}
