// Measurement aids: what the device itself delivers on the two rooflines the kernels are priced
// against, so that a benchmark can print a measured denominator beside the published one.
//   probe_stream_read_kernel   plain coalesced read of a buffer (16 bytes per lane, eight loads in
//                              flight per lane, nontemporal), nothing done with the data
//   probe_mfma_bf16_kernel     back-to-back 32x32x16 bf16 products on register operands (one
//                              wavefront per SIMD, eight independent accumulator blocks), no memory
//                              traffic inside the loop; the operands come from a caller buffer, so
//                              the switching activity is that of real values
#pragma once
#include "common.h"

namespace deinfer {

constexpr int PROBE_READ_THREADS = 512;
constexpr int PROBE_READ_UNROLL = 8;
constexpr int PROBE_MFMA_THREADS = 256;
constexpr int PROBE_MFMA_ACC = 8;

// n_kb: 1 KiB pieces (64 lanes x 16 bytes).  Workgroup g takes pieces [g n_kb / G, (g + 1) n_kb / G).
__global__ __launch_bounds__(PROBE_READ_THREADS) void probe_stream_read_kernel(const u32x4_t *src, size_t n_kb, u32x4_t *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = PROBE_READ_THREADS / 64;
  const size_t a = (size_t)blockIdx.x * n_kb / gridDim.x, b = (size_t)(blockIdx.x + 1) * n_kb / gridDim.x;
  u32x4_t acc = {0u, 0u, 0u, 0u};
  for (size_t k0 = a + wave; k0 < b; k0 += (size_t)W * PROBE_READ_UNROLL) {
    u32x4_t v[PROBE_READ_UNROLL];
#pragma unroll
    for (int i = 0; i < PROBE_READ_UNROLL; ++i) {
      size_t k = k0 + (size_t)i * W;
      k = k < b ? k : k0;                  // past the end: read a piece of this workgroup again
      v[i] = __builtin_nontemporal_load(src + k * 64 + lane);
    }
#pragma unroll
    for (int i = 0; i < PROBE_READ_UNROLL; ++i) acc ^= v[i];
  }
  // keeps the loads alive; the condition practically never holds
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u) sink[threadIdx.x] = acc;
}

// Every wavefront issues n_rounds * PROBE_MFMA_ACC products.  operands: 256 x 32 bytes of bf16.
__global__ __launch_bounds__(PROBE_MFMA_THREADS) void probe_mfma_bf16_kernel(const u32x4_t *operands, int n_rounds, float *sink) {
#if defined(__HIP_DEVICE_COMPILE__)
  f32x16_t acc[PROBE_MFMA_ACC];
#pragma unroll
  for (int i = 0; i < PROBE_MFMA_ACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  const u32x4_t a = operands[2 * threadIdx.x], b = operands[2 * threadIdx.x + 1];
  for (int it = 0; it < n_rounds; ++it) {
#pragma unroll
    for (int i = 0; i < PROBE_MFMA_ACC; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PROBE_MFMA_ACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[(size_t)blockIdx.x * PROBE_MFMA_THREADS + threadIdx.x] = s;
#else
  (void)operands; (void)n_rounds; (void)sink;
#endif
}

}  // namespace deinfer
