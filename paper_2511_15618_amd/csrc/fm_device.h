// Device-side helpers shared by the kernels: storage-type traits and reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Storage / MFMA operand type of the "bf16" configurations.  Their weights are bf16-valued, which
// convert to IEEE half exactly (8-bit significand into 11 bits; only magnitudes below 2^-14 go
// subnormal), and half keeps 3 more significand bits for activations and K/V at the same byte
// and MFMA cost, which is what holds the logits inside the stated tolerance.
typedef _Float16 f16_t;

#define FM_HD 64          // head width the single-launch verify kernel and the fused q,k,v epilogue are written for
#define FM_WAVE 64

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void ld8(const float* p, float* o) {
    float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
};
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
template <> struct Store<f16_t> {
  static __device__ __forceinline__ float ld(const f16_t* p) { return (float)*p; }
  static __device__ __forceinline__ void st(f16_t* p, float v) { *p = (f16_t)v; }   // round-to-nearest-even
  static __device__ __forceinline__ void ld8(const f16_t* p, float* o) {
    const f16x8 a = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (float)a[i];
  }
};

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

__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float k = 0.7978845608028654f;  // sqrt(2/pi)
  float u = k * (x + 0.044715f * x * x * x);
  return 0.5f * x * (1.0f + tanhf(u));
}
