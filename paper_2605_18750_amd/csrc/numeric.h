// Storage-type helpers shared by the device kernels: bf16 <-> fp32 and IEEE half <-> fp32 conversion
// (round-to-nearest-even) and 16-byte vector loads/stores converted to fp32.
//
// bf16 is the storage type of the stage's interface tensors, of its parameters and of every gradient
// tensor (range of fp32).  IEEE half (f16_t: 11-bit significand) holds the forward activations on the
// path into the attention scores (first norm output, q, k, v, and the attention-internal copy of dO),
// where bf16's 8-bit significand is amplified by the softmax; those tensors are O(1..100), far inside
// half's range, and conversions saturate at +-65504 instead of producing infinities.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rrfp {

struct bf16_t { uint16_t bits; };

__device__ __host__ inline float bf16_bits_to_float(uint32_t b) {
  union { uint32_t u; float f; } v;
  v.u = b << 16;
  return v.f;
}

__device__ __host__ inline uint16_t float_to_bf16_bits(float f) {
  union { uint32_t u; float f; } v;
  v.f = f;
  if ((v.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((v.u >> 16) | 0x40u);  // NaN stays NaN
  return (uint16_t)((v.u + 0x7fffu + ((v.u >> 16) & 1u)) >> 16);
}

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(bf16_t v) { return bf16_bits_to_float(v.bits); }

template <typename T> __device__ inline T from_float(float f);
template <> __device__ inline float from_float<float>(float f) { return f; }
// On the device the conversion is the hardware one (v_cvt_pk_bf16_f32: round-to-nearest-even).
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef float floatx2_native __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  const floatx2_native v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native));
}
template <> __device__ inline bf16_t from_float<bf16_t>(float f) { return bf16_t{(uint16_t)(pack_bf16x2(f, 0.f) & 0xffffu)}; }

struct f16_t { uint16_t bits; };

typedef _Float16 halfx2_native __attribute__((ext_vector_type(2)));
__device__ inline float f16_sat(float f) { return __builtin_fminf(__builtin_fmaxf(f, -65504.0f), 65504.0f); }   // NaN passes through
// Two floats -> packed IEEE halves, round-to-nearest-even, saturating.
__device__ inline uint32_t pack_f16x2(float lo, float hi) {
  const floatx2_native v = {f16_sat(lo), f16_sat(hi)};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, halfx2_native));
}
// The same with truncation toward zero in ONE instruction (v_cvt_pkrtz_f16_f32), for values known to be in
// range that are produced inside the attention inner loops (probabilities, dS).
__device__ inline uint32_t pack_f16x2_rtz(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
__device__ inline float to_float(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.bits); }
template <> __device__ inline f16_t from_float<f16_t>(float f) { return f16_t{(uint16_t)(pack_f16x2(f, 0.f) & 0xffffu)}; }

template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<bf16_t> { static constexpr int N = 8; };
template <> struct Vec<f16_t> { static constexpr int N = 8; };

// 16-byte aligned vector load of Vec<T>::N elements, widened to fp32.
template <typename T> __device__ inline void load_vec(const T* p, float* out);
template <> __device__ inline void load_vec<float>(const float* p, float* out) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <> __device__ inline void load_vec<bf16_t>(const bf16_t* p, float* out) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

template <> __device__ inline void load_vec<f16_t>(const f16_t* p, float* out) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const halfx2_native h = __builtin_bit_cast(halfx2_native, w[i]);
    out[2 * i] = (float)h[0];
    out[2 * i + 1] = (float)h[1];
  }
}

template <typename T> __device__ inline void store_vec(T* p, const float* in);
template <> __device__ inline void store_vec<float>(float* p, const float* in) {
  *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
}
template <> __device__ inline void store_vec<bf16_t>(bf16_t* p, const float* in) {
  uint4 v;
  v.x = pack_bf16x2(in[0], in[1]);
  v.y = pack_bf16x2(in[2], in[3]);
  v.z = pack_bf16x2(in[4], in[5]);
  v.w = pack_bf16x2(in[6], in[7]);
  *reinterpret_cast<uint4*>(p) = v;
}

template <> __device__ inline void store_vec<f16_t>(f16_t* p, const float* in) {
  uint4 v;
  v.x = pack_f16x2(in[0], in[1]);
  v.y = pack_f16x2(in[2], in[3]);
  v.z = pack_f16x2(in[4], in[5]);
  v.w = pack_f16x2(in[6], in[7]);
  *reinterpret_cast<uint4*>(p) = v;
}

}  // namespace rrfp
