// Small device helpers: bf16 conversion, wave64 reductions, (value, index) arg-max merge.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;
typedef uint16_t f16_t;    // IEEE half bit pattern in memory

// Pointers that reach a kernel through a descriptor in memory are generic to the compiler and
// would be accessed with FLAT instructions, whose completion is tied to the LDS counter; casting
// them to the global address space keeps vector memory and LDS waits independent.
#define TS_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ float bf16_to_f32(bf16_t u) { return __uint_as_float((uint32_t)u << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  b += 0x7fffu + ((b >> 16) & 1u);
  return (bf16_t)(b >> 16);
}

// two floats -> packed bf16 pair (low half = a), round to nearest even, one v_cvt_pk_bf16_f32
typedef __bf16 ts_bf16x2 __attribute__((ext_vector_type(2)));
typedef float ts_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const ts_f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ts_bf16x2));
}

// two floats -> packed IEEE half pair (low half = a), round to nearest even
typedef _Float16 ts_f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_f16x2(float a, float b) {
  const ts_f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ts_f16x2));
}
// packed bf16 pair -> packed half pair (exact in the normal range of half)
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
  return pack_f16x2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}
// activation -> IEEE half, round to nearest even, saturating at the largest finite half (NaN stays NaN)
__device__ __forceinline__ float sat_f16_range(float f) { return f == f ? fminf(fmaxf(f, -65504.f), 65504.f) : f; }
__device__ __forceinline__ uint16_t f32_to_f16_sat(float f) { return f32_to_f16_bits(sat_f16_range(f)); }
__device__ __forceinline__ uint32_t pack_f16x2_sat(float a, float b) { return pack_f16x2(sat_f16_range(a), sat_f16_range(b)); }

// An activation that enters a weight projection of a bf16 model is carried as TWO halves,
// x = hi + lo with hi = half(x) (saturating) and lo = half(x - hi): about 22 significant bits, so
// that the projection inputs add no rounding of their own beyond fp32's.  The planes are separate
// arrays `plane` elements apart; both feed the same MFMA accumulator.
constexpr int TS_ACT_PLANES = 2;
__device__ __forceinline__ void split_f16_planes(float x, _Float16& hi, _Float16& lo) {
  const float xs = sat_f16_range(x);
  hi = (_Float16)xs;
  lo = (_Float16)(xs - (float)hi);
}
// `sat` counts the activations whose magnitude exceeded the largest finite half and were clamped
// (a model whose activations leave half's range is computed wrongly from there on: the caller can
// see that it happened instead of getting silently clipped values)
__device__ __forceinline__ void count_saturated(float x, unsigned long long* sat) {
  if (fabsf(x) > 65504.f) atomicAdd(sat, 1ull);
}
__device__ __forceinline__ void st_act_planes(f16_t* p, size_t plane, float x, unsigned long long* sat) {
  _Float16 hi, lo;
  count_saturated(x, sat);
  split_f16_planes(x, hi, lo);
  p[0] = __builtin_bit_cast(uint16_t, hi);
  p[plane] = __builtin_bit_cast(uint16_t, lo);
}
// four consecutive activations (p 8-byte aligned): one vector store per plane
__device__ __forceinline__ void st_act_planes4(f16_t* p, size_t plane, float x0, float x1, float x2, float x3,
                                               unsigned long long* sat) {
  if (fmaxf(fmaxf(fabsf(x0), fabsf(x1)), fmaxf(fabsf(x2), fabsf(x3))) > 65504.f) {
    count_saturated(x0, sat); count_saturated(x1, sat); count_saturated(x2, sat); count_saturated(x3, sat);
  }
  _Float16 h[4], l[4];
  split_f16_planes(x0, h[0], l[0]);
  split_f16_planes(x1, h[1], l[1]);
  split_f16_planes(x2, h[2], l[2]);
  split_f16_planes(x3, h[3], l[3]);
  const ts_f16x2 h01 = {h[0], h[1]}, h23 = {h[2], h[3]}, l01 = {l[0], l[1]}, l23 = {l[2], l[3]};
  *reinterpret_cast<uint2*>(p) = make_uint2(__builtin_bit_cast(uint32_t, h01), __builtin_bit_cast(uint32_t, h23));
  *reinterpret_cast<uint2*>(p + plane) = make_uint2(__builtin_bit_cast(uint32_t, l01), __builtin_bit_cast(uint32_t, l23));
}

__device__ __forceinline__ float ld_f32(const float* p) { return *p; }
__device__ __forceinline__ float ld_f32(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st_from_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_from_f32(bf16_t* p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// maximum over the four lanes l, l^16, l^32, l^48 of a wave, through the lane-swap instructions
// of gfx950 (v_permlane16_swap / v_permlane32_swap): each leaves a lane with its own value and
// its partner's, so two swaps and two maxima replace two LDS-routed shuffles and their waits
__device__ __forceinline__ float max_over_lane_groups(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t v = __float_as_uint(fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// keep the larger value; among equal values the lower index
__device__ __forceinline__ void amax_take(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}
__device__ __forceinline__ void wave_amax(float& bv, int& bi) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    amax_take(bv, bi, ov, oi);
  }
}
