// Device-side helpers shared by the libmtla kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mtla {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kBlock = 256;        // threads per workgroup in the VALU kernels (4 waves)
constexpr int kHeaderBytes = 256;  // workspace header; int32[0] is the sticky device status

// Storage element types.  bf16 is carried as its 16-bit pattern.
struct bf16 {
  uint16_t bits;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return __uint_as_float(uint32_t(v.bits) << 16); }

// fp32 -> bf16, round to nearest, ties to even: gfx950's v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
// Two fp32 values to a packed bf16 pair (lo in bits 0..15), one instruction.
// One int32 at a wavefront-uniform address, from memory that nothing writes while the kernel runs (a page
// table): read through the constant address space, so that it is a scalar load and has a wait counter of its
// own.  As an ordinary load it is a vector load, and waiting for it means waiting for every tile load in flight.
__device__ __forceinline__ int32_t load_uniform_i32(const int32_t* p, int idx) {
  typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
  return reinterpret_cast<const_i32_ptr>(reinterpret_cast<uintptr_t>(p))[idx];
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// Two fp32 values to a packed IEEE-half pair (lo in bits 0..15), round to nearest even.
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}
// ... and back.
__device__ __forceinline__ float f16_lo_to_f32(uint32_t v) {
  return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v & 0xffffu)));
}
__device__ __forceinline__ float f16_hi_to_f32(uint32_t v) {
  return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v >> 16)));
}

// 8 consecutive stored elements as fp32.
__device__ __forceinline__ void load8(const bf16* p, float (&o)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __uint_as_float(w[i] << 16);
    o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void load8(const float* p, float (&o)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
  o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// fp32 pair -> bf16 pair hi plus bf16 pair lo with hi + lo ~ value to about 16 mantissa bits.
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16x2(a, b);
  lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ bf16 from_f32<bf16>(float v) {
  return bf16{f32_to_bf16_bits(v)};
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

// The pair (a, b) = elements (2k, 2k+1) of a d-wide vector, turned by pos * freq, freq = base^(-2k/d)
// (a double, from the host: positions reach tens of thousands of radians, so the product and its
// reduction to [-pi, pi] are done in double; sine and cosine of the reduced angle in float).
__device__ __forceinline__ void rope_pair(float& a, float& b, int pos, double freq) {
  double ang = (double)pos * freq;
  ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
  float sn, cs;
  sincosf((float)ang, &sn, &cs);
  const float ra = a * cs - b * sn, rb = a * sn + b * cs;
  a = ra;
  b = rb;
}

}  // namespace mtla
