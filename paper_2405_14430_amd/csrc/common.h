// Shared device helpers for the gfx950 kernels: storage types, bf16 conversion, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace pf {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// Raises a kernel's dynamic-LDS limit to Bytes, once per kernel instance and process, safely from any number of host
// threads (stages on different threads share the kernels).  Every later call returns the first call's status.
template <auto Kernel, int Bytes>
inline hipError_t allow_dynamic_lds() {
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, Bytes);
  });
  return status;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t *p) { return static_cast<float>(*p); }
  static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = static_cast<bf16_t>(v); }  // RNE
};

template <typename T> __device__ __forceinline__ float to_f32(T v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return static_cast<T>(v); }

// Sum / max over the 64 lanes of a wavefront; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

__device__ __forceinline__ float gelu_f(float x, int tanh_form) {
  if (tanh_form) {
    // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3): one exponential and one reciprocal of
    // the hardware (about 1 ulp each) instead of the library tanh (a few dozen instructions per element in a GEMM epilogue)
    const float k0 = 0.7978845608028654f;  // sqrt(2/pi)
    const float u = k0 * x * fmaf(0.044715f * x, x, 1.0f);
    const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);   // exp(-2u); +inf for very negative u
    return x * __builtin_amdgcn_rcpf(1.0f + e);                                // x * 0 = -0 there, as it should be
  }
  return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

}  // namespace pf

namespace pf {
// 16-byte vector access: 4 floats or 8 bf16, widened to float.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float *p, float *o) {
    float4 v = *reinterpret_cast<const float4 *>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  static __device__ __forceinline__ void store(float *p, const float *o) {
    *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t *p, float *o) {
    bf16x8 v = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = static_cast<float>(v[i]);
  }
  static __device__ __forceinline__ void store(bf16_t *p, const float *o) {
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = static_cast<bf16_t>(o[i]);
    *reinterpret_cast<bf16x8 *>(p) = v;
  }
};
}  // namespace pf
