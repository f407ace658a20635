// Small device helpers shared by the WIND kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wind {

typedef uint16_t bf16_t;  // raw bf16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // 16 bytes = 8 bf16
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;

// fp32 -> bf16, round to nearest even, two values per instruction: gfx950 converts in hardware
// (v_cvt_pk_bf16_f32), with the same result as the usual integer sequence u + 0x7FFF + ((u >> 16) & 1)
// on every finite input, ties and denormals included (checked on the device over 2 M values).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// c + a.lo * b.lo + a.hi * b.hi on two packed bf16 pairs, fp32 result (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) { return pack_bf16x2(x, 0.f) & 0xFFFFu; }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// load one weight element as fp32
__device__ __forceinline__ float ldw(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldw(const bf16_t *p, size_t i) { return bf16_bits_to_f32(p[i]); }

// two consecutive weights (i even) as fp32
__device__ __forceinline__ float2 ldw2(const float *p, size_t i) {
  return *reinterpret_cast<const float2 *>(p + i);
}
__device__ __forceinline__ float2 ldw2(const bf16_t *p, size_t i) {
  uint32_t u = *reinterpret_cast<const uint32_t *>(p + i);
  return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xFFFF0000u));
}

// Wave-wide reductions.  Inside a row of 16 lanes the partners come from DPP permutations, which cost
// no more than a move (row mirror i <-> 15-i, half mirror i <-> 7-i, then i ^ 2 and i ^ 1: after the
// four steps every lane of the row holds the row's result); the four row results are then read
// with v_readlane.  No step goes through the LDS crossbar, whose latency dominated the shuffle
// version in the latency-bound kernels.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int x) {
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, false);
}
constexpr int kDppRowMirror = 0x140, kDppRowHalfMirror = 0x141, kDppQuadXor2 = 0x4E, kDppQuadXor1 = 0xB1;
__device__ __forceinline__ float readlane_f32(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// the same four steps alone: reductions over each row of 16 lanes, four independent results per wave
__device__ __forceinline__ float row16_max_f32(float v) {
  v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
  v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
  return fmaxf(v, dpp_f32<kDppQuadXor1>(v));
}
__device__ __forceinline__ int row16_max_i32(int v) {
  v = max(v, dpp_i32<kDppRowMirror>(v));
  v = max(v, dpp_i32<kDppRowHalfMirror>(v));
  v = max(v, dpp_i32<kDppQuadXor2>(v));
  return max(v, dpp_i32<kDppQuadXor1>(v));
}
__device__ __forceinline__ int row16_sum_i32(int v) {
  v += dpp_i32<kDppRowMirror>(v);
  v += dpp_i32<kDppRowHalfMirror>(v);
  v += dpp_i32<kDppQuadXor2>(v);
  return v + dpp_i32<kDppQuadXor1>(v);
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppRowMirror>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  v += dpp_f32<kDppQuadXor2>(v);
  v += dpp_f32<kDppQuadXor1>(v);
  return (readlane_f32(v, 0) + readlane_f32(v, 16)) + (readlane_f32(v, 32) + readlane_f32(v, 48));
}
__device__ __forceinline__ int wave_sum_i32(int v) {
  v += dpp_i32<kDppRowMirror>(v);
  v += dpp_i32<kDppRowHalfMirror>(v);
  v += dpp_i32<kDppQuadXor2>(v);
  v += dpp_i32<kDppQuadXor1>(v);
  return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
         (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}
__device__ __forceinline__ int wave_max_i32(int v) {
  v = max(v, dpp_i32<kDppRowMirror>(v));
  v = max(v, dpp_i32<kDppRowHalfMirror>(v));
  v = max(v, dpp_i32<kDppQuadXor2>(v));
  v = max(v, dpp_i32<kDppQuadXor1>(v));
  return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// (logit, column) carried in one fp32 word: the low 7 mantissa bits of the logit give way to
// 127 - column (column within a part of at most 128), which costs 2^-16 of relative precision and
// keeps ordinary float ordering, so top-2 selection is v_max_f32 / v_med3_f32 on the packed words.
// Among equal truncated positive values the lower column compares larger.
constexpr uint32_t kKeyColMask = 127u;
constexpr float kKeyNone = -3.0e38f;   // below every real logit; finite, so packing never makes a NaN

__device__ __forceinline__ float make_key(float v, int col_in_part) {
  return __uint_as_float((__float_as_uint(v) & ~kKeyColMask) | (kKeyColMask - (uint32_t)col_in_part));
}
__device__ __forceinline__ int key_col(float k) { return (int)(kKeyColMask - (__float_as_uint(k) & kKeyColMask)); }
__device__ __forceinline__ float key_val(float k) { return __uint_as_float(__float_as_uint(k) & ~kKeyColMask); }

// A tag bit in a key: the lowest bit of the value field (one more bit of truncation, 2^-15 relative in all).
// The resident loop kernel marks the second key of every (first, second) pair it exchanges with the
// iteration's parity, so that a reader can tell this iteration's pair from the one two iterations old
// without a separate flag.
constexpr uint32_t kKeyTagBit = 128u;
__device__ __forceinline__ float key_with_tag(float k, int tag) {
  return __uint_as_float((__float_as_uint(k) & ~kKeyTagBit) | (tag ? kKeyTagBit : 0u));
}
__device__ __forceinline__ int key_tag(float k) { return (int)((__float_as_uint(k) >> 7) & 1u); }

// top-2 of the union of two sorted pairs (a1 >= a2), (b1 >= b2)
__device__ __forceinline__ void merge_top2(float &a1, float &a2, float b1, float b2) {
  const float m = fmaxf(a2, b2);
  a2 = __builtin_amdgcn_fmed3f(a1, b1, m);
  a1 = fmaxf(a1, b1);
}
__device__ __forceinline__ void push_top2(float &a1, float &a2, float k) {
  a2 = __builtin_amdgcn_fmed3f(k, a1, a2);
  a1 = fmaxf(a1, k);
}
// the same for the three largest (a1 >= a2 >= a3)
// (the maximum as the median with +infinity: fmaxf would first quieten a possible NaN, one more
// instruction per element of the joint kernels' epilogues, whose keys are never NaN)
__device__ __forceinline__ float key_inf() {
  float inf = __builtin_inff();
  asm volatile("" : "+v"(inf));   // opaque, so that the median is not folded back into a maximum
  return inf;
}
__device__ __forceinline__ void push_top3(float &a1, float &a2, float &a3, float k, float inf) {
  a3 = __builtin_amdgcn_fmed3f(k, a2, a3);
  a2 = __builtin_amdgcn_fmed3f(k, a1, a2);
  a1 = __builtin_amdgcn_fmed3f(a1, k, inf);
}
__device__ __forceinline__ void push_top3(float &a1, float &a2, float &a3, float k) {
  a3 = __builtin_amdgcn_fmed3f(k, a2, a3);
  a2 = __builtin_amdgcn_fmed3f(k, a1, a2);
  a1 = fmaxf(a1, k);
}
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
  v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
  v = fmaxf(v, dpp_f32<kDppQuadXor1>(v));
  return fmaxf(fmaxf(readlane_f32(v, 0), readlane_f32(v, 16)), fmaxf(readlane_f32(v, 32), readlane_f32(v, 48)));
}

}  // namespace wind
