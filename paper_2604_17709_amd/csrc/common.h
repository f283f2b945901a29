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

// ---- the two 16-bit storage types of the packed path, selected by a template integer that equals
// the dtype code of the boundary (1 = bf16, 2 = fp16).  Storage is a raw 16-bit pattern; sums are
// fp32; results are rounded once, to nearest even, by the device's packed conversion instructions.
constexpr int DT_BF16 = 1, DT_F16 = 2;
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
template <int DT> __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  if constexpr (DT == DT_F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, f16x2_t));
  else return pack_bf16x2(lo, hi);
}
template <int DT> __device__ __forceinline__ float lo_f32(uint32_t w) {      // element in the low half of a word
  if constexpr (DT == DT_F16) return (float)__builtin_bit_cast(f16x2_t, w)[0];
  else return __uint_as_float(w << 16);
}
template <int DT> __device__ __forceinline__ float hi_f32(uint32_t w) {
  if constexpr (DT == DT_F16) return (float)__builtin_bit_cast(f16x2_t, w)[1];
  else return __uint_as_float(w & 0xffff0000u);
}
template <int DT> __device__ __forceinline__ float cvt_in(uint16_t b) { return lo_f32<DT>(b); }
template <int DT> __device__ __forceinline__ uint16_t cvt_out(float f) { return static_cast<uint16_t>(pack2<DT>(f, 0.0f) & 0xffffu); }

struct f16_bits { uint16_t v; };          // element type of fp16 tensors in the generic kernels

template <typename T> struct Elem;
template <> struct Elem<f16_bits> {
  static __device__ __forceinline__ float load(const f16_bits *p) { return cvt_in<DT_F16>(p->v); }
  static __device__ __forceinline__ void store(f16_bits *p, float v) { p->v = cvt_out<DT_F16>(v); }
};
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {  // bf16
  static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(uint16_t *p, float v) { *p = f32_to_bf16(v); }
};
template <typename T> struct DtOf { static constexpr int value = 0; };          // storage-type code of an element type
template <> struct DtOf<uint16_t> { static constexpr int value = DT_BF16; };
template <> struct DtOf<f16_bits> { static constexpr int value = DT_F16; };

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

// value of the lane 8 further round the same row of 16 lanes (lane ^ 8); every lane of the row must be active
__device__ __forceinline__ uint32_t across8(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128 /* row_ror:8 */, 0xf, 0xf, false);
#else
  return v;
#endif
}
__device__ __forceinline__ float across8(float v) { return __uint_as_float(across8(__float_as_uint(v))); }

__device__ __forceinline__ bf16x8_t as_bf16x8(const u32x4_t &v) {
  return __builtin_bit_cast(bf16x8_t, v);
}

// The two matrix instructions of the kernels, on 8 packed 16-bit values per lane and operand.
template <int DT> __device__ __forceinline__ f32x16_t mfma32(const u32x4_t &a, const u32x4_t &b, const f32x16_t &c) {
#if defined(__HIP_DEVICE_COMPILE__)
  if constexpr (DT == DT_F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
#else
  (void)a; (void)b;                      // (the host pass only needs the stub)
  return c;
#endif
}
template <int DT> __device__ __forceinline__ f32x4_t mfma16(const u32x4_t &a, const u32x4_t &b, const f32x4_t &c) {
#if defined(__HIP_DEVICE_COMPILE__)
  if constexpr (DT == DT_F16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
#else
  (void)a; (void)b;                      // (the host pass only needs the stub)
  return c;
#endif
}

// The activation operand is read in 16-byte chunks of 8 columns.  Where the valid columns K of a row are
// no multiple of 8 (the caller's rank-space rows of an upward projection alone), the chunk that holds
// column K - 1 also holds columns that are not the kernel's to use (the weights there are zero, but
// 0 x NaN is NaN): once that chunk has landed in LDS its elements K % 8 .. 7 are set to zero.  Chunks
// that lie wholly beyond K fetch the row's first chunk instead (any finite values: zero weights).
__device__ __forceinline__ void lds_zero_chunk_tail(unsigned char *chunk, int n_keep) {      // n_keep = K % 8 in 1 .. 7
  u32x4_t v = *reinterpret_cast<u32x4_t *>(chunk);
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const int keep = n_keep - 2 * d;
    v[d] &= keep >= 2 ? 0xffffffffu : keep == 1 ? 0x0000ffffu : 0u;
  }
  *reinterpret_cast<u32x4_t *>(chunk) = v;
}

}  // namespace deinfer
