// Storage types and 16-byte vector helpers for the device code.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace hgnn {

struct bf16 {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
// Round to nearest, ties to even; NaN stays (quiet) NaN.  gfx950 converts in hardware, two values per
// instruction; the result equals the integer recipe (add 0x7fff + lsb, shift) bit for bit.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2(float a, float b) {  // a in the low half
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) { return pack2(f, 0.f) & 0xffffu; }

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16 v) { return bf16_bits_to_float(v.bits); }
template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_float<bf16>(float v) {
  bf16 r;
  r.bits = (uint16_t)float_to_bf16_bits(v);
  return r;
}

// A 16-byte piece of a feature row: N scalars of T.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void add(float *acc, const uint4 &v) {
    acc[0] += __uint_as_float(v.x);
    acc[1] += __uint_as_float(v.y);
    acc[2] += __uint_as_float(v.z);
    acc[3] += __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float *a) {
    return make_uint4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3]));
  }
  static __device__ __forceinline__ uint4 pack_remainder(const float *, const uint4 &) { return make_uint4(0, 0, 0, 0); }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void add(float *acc, const uint4 &v) {
    acc[0] += __uint_as_float(v.x << 16);
    acc[1] += __uint_as_float(v.x & 0xffff0000u);
    acc[2] += __uint_as_float(v.y << 16);
    acc[3] += __uint_as_float(v.y & 0xffff0000u);
    acc[4] += __uint_as_float(v.z << 16);
    acc[5] += __uint_as_float(v.z & 0xffff0000u);
    acc[6] += __uint_as_float(v.w << 16);
    acc[7] += __uint_as_float(v.w & 0xffff0000u);
  }
  static __device__ __forceinline__ uint4 pack(const float *a) {
    uint4 r;
    r.x = pack2(a[0], a[1]);
    r.y = pack2(a[2], a[3]);
    r.z = pack2(a[4], a[5]);
    r.w = pack2(a[6], a[7]);
    return r;
  }
  // What `hi` = pack(a) dropped, rounded to the storage type in turn: hi + remainder carries 16 significant
  // bits of a (the difference of an fp32 value and its bf16 rounding is exact in fp32).
  static __device__ __forceinline__ uint4 pack_remainder(const float *a, const uint4 &hi) {
    float back[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) back[i] = 0.f;
    add(back, hi);
#pragma unroll
    for (int i = 0; i < 8; ++i) back[i] = a[i] - back[i];
    return pack(back);
  }
};

}  // namespace hgnn
