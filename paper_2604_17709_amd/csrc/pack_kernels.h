// Re-layout of a RAW bf16 factor into MFMA-fragment order (see deinfer.h, "Packed
// weight format").  Source S[K x F] row-major (pitch ld): for U, K = d_in and F = r;
// for V, K = r and F = d_out.  Destination: fragments of 16 features x 32 k, 64 lanes
// x 8 bf16, lane = (f % 16) + 16 * ((k % 32) / 8), element = k % 8, fragment index
// (f / 16) * KB + (k / 32).  Out-of-range features and k are zero.
#pragma once
#include "common.h"

namespace deinfer {

__global__ void pack_fragments_kernel(const uint16_t *__restrict__ S, int64_t ld, int K, int F,
                                      int n_ftiles, int KB, uint4 *__restrict__ dst) {
  const int64_t n = (int64_t)n_ftiles * KB * 64;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(i & 63);
    const int64_t frag = i >> 6;
    const int kb = (int)(frag % KB);
    const int tile = (int)(frag / KB);
    const int f = tile * 16 + (lane & 15);
    const int k0 = kb * 32 + (lane >> 4) * 8;
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = k0 + j;
      e[j] = (f < F && k < K) ? S[(int64_t)k * ld + f] : (uint16_t)0;
    }
    uint4 v;
    v.x = e[0] | ((uint32_t)e[1] << 16);
    v.y = e[2] | ((uint32_t)e[3] << 16);
    v.z = e[4] | ((uint32_t)e[5] << 16);
    v.w = e[6] | ((uint32_t)e[7] << 16);
    dst[i] = v;
  }
}

}  // namespace deinfer
