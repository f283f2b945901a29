// Shared device helpers for the gfx950 low-rank linear kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace deinfer {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// ---- bf16 <-> fp32 (storage type is a raw 16-bit pattern) -------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest, ties to even; NaN stays NaN (the device's packed conversion instruction)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return static_cast<uint16_t>(pack_bf16x2(f, 0.0f) & 0xffffu);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {  // bf16
  static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(uint16_t *p, float v) { *p = f32_to_bf16(v); }
};

// SiLU in fp32: z * sigmoid(z) = z / (1 + exp(-z))
__device__ __forceinline__ float silu_f32(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// Activation of the non-GLU MLP sub-layer (Table 2 lists both kinds of model), applied in fp32
// to the sum of product and bias: 0 identity, 1 ReLU, 2 GELU z Phi(z) (erf form).
constexpr int ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2;
__device__ __forceinline__ float act_f32(float z, int act) {
  if (act == ACT_RELU) return fmaxf(z, 0.0f);
  if (act == ACT_GELU) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
  return z;
}

__device__ __forceinline__ bf16x8_t as_bf16x8(const u32x4_t &v) {
  return __builtin_bit_cast(bf16x8_t, v);
}

}  // namespace deinfer
