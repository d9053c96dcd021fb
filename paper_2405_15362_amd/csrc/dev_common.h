// Device-side helpers shared by the kernels: vector types, bf16 packing, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pmc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef uint16_t bf16_t;  // storage type of a bfloat16 value

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// Round to nearest even.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Storage-type traits: T = float or bf16_t; loads/stores of VEC consecutive elements (16 bytes).
template <typename T>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const float* p, float* out) {
    f32x4 v = *reinterpret_cast<const f32x4*>(p);
    out[0] = v[0]; out[1] = v[1]; out[2] = v[2]; out[3] = v[3];
  }
  __device__ static __forceinline__ void store(float* p, const float* in) {
    f32x4 v = {in[0], in[1], in[2], in[3]};
    *reinterpret_cast<f32x4*>(p) = v;
  }
  // the 16 bytes as they are in memory (a row kept this way costs 4 registers per chunk whatever the type)
  __device__ static __forceinline__ u32x4 load_raw(const float* p) { return *reinterpret_cast<const u32x4*>(p); }
  __device__ static __forceinline__ void store_raw(float* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }
  __device__ static __forceinline__ void unpack(u32x4 v, float* out) {
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(v[i]);
  }
};
template <>
struct Vec<bf16_t> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float* out) {
    u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = bf16lo_to_f32(v[i]);
      out[2 * i + 1] = bf16hi_to_f32(v[i]);
    }
  }
  __device__ static __forceinline__ void store(bf16_t* p, const float* in) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = pack_bf16x2(in[2 * i], in[2 * i + 1]);
    *reinterpret_cast<u32x4*>(p) = v;
  }
  __device__ static __forceinline__ u32x4 load_raw(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
  __device__ static __forceinline__ void store_raw(bf16_t* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }
  __device__ static __forceinline__ void unpack(u32x4 v, float* out) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = bf16lo_to_f32(v[i]);
      out[2 * i + 1] = bf16hi_to_f32(v[i]);
    }
  }
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// tanh-form GeLU and its derivative.
__device__ __forceinline__ float gelu_f(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float t = tanhf(k0 * (u + k1 * u * u * u));
  return 0.5f * u * (1.0f + t);
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float t = tanhf(k0 * (u + k1 * u * u * u));
  return 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * k0 * (1.0f + 3.0f * k1 * u * u);
}

// The same two maps with tanh built from the hardware exp2 and reciprocal (absolute error of
// tanh about 1e-7): used where the result is rounded to bf16 anyway.
__device__ __forceinline__ float tanh_fast(float z) {
  const float e = __builtin_amdgcn_exp2f(z * 2.885390081777927f);  // exp(2z)
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}
__device__ __forceinline__ float gelu_fast(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  return 0.5f * u * (1.0f + tanh_fast(k0 * (u + k1 * u * u * u)));
}
// gelu(u) and gelu'(u) from one exp2 and one reciprocal: with r = 1 / (exp(2z) + 1), tanh z = 1 - 2r,
// so gelu = u (1 - r) and gelu' = (1 - r) (1 + 2 u r z'),  z = k0 (u + k1 u^3),  z' = k0 (1 + 3 k1 u^2).
__device__ __forceinline__ void gelu_both_fast(float u, float& g, float& dg) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  const float u2 = u * u;
  const float z = k0 * u * __builtin_fmaf(k1, u2, 1.0f);
  const float r = __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(z * 2.885390081777927f) + 1.0f);
  const float s = 1.0f - r;
  g = u * s;
  dg = s * __builtin_fmaf(2.0f * k0 * u * r, __builtin_fmaf(3.0f * k1, u2, 1.0f), 1.0f);
}
__device__ __forceinline__ float gelu_grad_fast(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  const float t = tanh_fast(k0 * (u + k1 * u * u * u));
  return 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * k0 * (1.0f + 3.0f * k1 * u * u);
}

}  // namespace pmc
