// Generic (any size, any alignment) kernels for RAW-layout factor pairs, fp32 or bf16
// storage with fp32 accumulation.  Plain LDS-tiled FMA GEMM on row-major operands:
//   C[M x N] = A[M x K] . B[K x N]            (one stage of y = (x U) V, Sec. 4.1)
// and, for the GLU sub-layer, C = silu(A1 . B1) * (A2 . B2) in one pass.
// These kernels are the correctness baseline of the library (small fp32 case, odd
// shapes); the packed MFMA kernels are the fast path.
#pragma once
#include "common.h"

namespace deinfer {

constexpr int GT = 64;   // output tile edge
constexpr int GK = 16;   // k step
constexpr int GTHREADS = 256;

// Accumulate a 64x64 tile of A.B into acc (4x4 per thread).
template <typename TA, typename TB>
__device__ __forceinline__ void tile_gemm_rr(const TA *__restrict__ A, int64_t lda,
                                             const TB *__restrict__ B, int64_t ldb,
                                             int M, int N, int K, int m0, int n0,
                                             float (&acc)[4][4], float (*sA)[GT + 1], float (*sB)[GT]) {
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  for (int k0 = 0; k0 < K; k0 += GK) {
    // A tile: 64 rows x 16 k  -> sA[k][row]
#pragma unroll
    for (int i = 0; i < (GT * GK) / GTHREADS; ++i) {
      int idx = tid + i * GTHREADS;
      int r = idx / GK, c = idx % GK;
      int gr = m0 + r, gc = k0 + c;
      sA[c][r] = (gr < M && gc < K) ? Elem<TA>::load(A + (int64_t)gr * lda + gc) : 0.0f;
    }
    // B tile: 16 k x 64 cols -> sB[k][col]
#pragma unroll
    for (int i = 0; i < (GT * GK) / GTHREADS; ++i) {
      int idx = tid + i * GTHREADS;
      int r = idx / GT, c = idx % GT;
      int gr = k0 + r, gc = n0 + c;
      sB[r][c] = (gr < K && gc < N) ? Elem<TB>::load(B + (int64_t)gr * ldb + gc) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = sB[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
}

// C = act(A.B + bias), or (DUAL) C = silu(A.B) * (A2.B2).  Grid: (ceil(N/64), ceil(M/64)).
// bias: one value per column of C (may be null), act: see act_f32.
template <typename TA, typename TB, typename TC, bool DUAL>
__global__ __launch_bounds__(GTHREADS) void gemm_generic_kernel(
    const TA *__restrict__ A, int64_t lda, const TB *__restrict__ B, int64_t ldb, int K,
    const TA *__restrict__ A2, int64_t lda2, const TB *__restrict__ B2, int64_t ldb2, int K2,
    TC *__restrict__ C, int64_t ldc, int M, int N, const TC *__restrict__ bias = nullptr, int act = ACT_NONE) {
  __shared__ float sA[GK][GT + 1];
  __shared__ float sB[GK][GT];
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  tile_gemm_rr<TA, TB>(A, lda, B, ldb, M, N, K, m0, n0, acc, sA, sB);
  float acc2[4][4] = {};
  if (DUAL) tile_gemm_rr<TA, TB>(A2, lda2, B2, ldb2, M, N, K2, m0, n0, acc2, sA, sB);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int r = m0 + ty * 4 + i;
    if (r >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = n0 + tx * 4 + j;
      if (c >= N) continue;
      float v = acc[i][j];
      if (DUAL) v = (v / (1.0f + expf(-v))) * acc2[i][j];
      else v = act_f32(v + (bias ? Elem<TC>::load(bias + c) : 0.0f), act);
      Elem<TC>::store(C + (int64_t)r * ldc + c, v);
    }
  }
}

// C[r][c] = act(bias[c]): the non-GLU sub-layer of a pair of rank 0 (empty product).
template <typename TC>
__global__ void bias_act_fill_kernel(TC *C, int64_t ldc, int M, int N, const TC *bias, int act) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)M * N) {
    const int64_t r = i / N, c = i % N;
    Elem<TC>::store(C + r * ldc + c, act_f32(bias ? Elem<TC>::load(bias + c) : 0.0f, act));
  }
}

// Zero-fill of a strided 2-D region (r == 0 outputs) and of raw words (workspace init).
template <typename TC>
__global__ void zero2d_kernel(TC *C, int64_t ldc, int M, int N) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)M * N) C[(i / N) * ldc + (i % N)] = TC{};
}
__global__ void fill_words_kernel(uint32_t *p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Copy a column block of a row-major matrix (used to hand out the rank-space
// intermediates of k and v, the low-rank KV cache of Sec. 2.1).
template <typename TS, typename TD>
__global__ void copy2d_kernel(const TS *S, int64_t lds, TD *D, int64_t ldd, int M, int N) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)M * N) {
    int64_t r = i / N, c = i % N;
    Elem<TD>::store(D + r * ldd + c, Elem<TS>::load(S + r * lds + c));
  }
}

// Rows of 16-bit elements copied with zero padding: D[row][c] = c < n_valid ? S[row][c] : 0 for
// c < N (the caller's rank-space rows brought to the 16-byte row layout the packed kernels read,
// with exact zeros where the zero-padded weights are met).  One thread = one 16-byte chunk of 8
// columns of D (D 16-byte aligned, ldd % 8 == 0, N % 8 == 0); a chunk that lies wholly inside the
// valid columns of a 16-byte aligned source row is one 16-byte load, any other chunk is read
// element by element, and never beyond column n_valid - 1.
__global__ void pad_rows16_kernel(const uint16_t *S, int64_t lds, uint16_t *D, int64_t ldd, int M, int n_valid, int N, int vec) {
  const int c8 = N / 8;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)M * c8) return;
  const int64_t r = i / c8;
  const int c = (int)(i % c8) * 8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  const uint16_t *src = S + r * lds + c;
  if (vec && c + 8 <= n_valid) {
    v = *reinterpret_cast<const uint4 *>(src);
  } else if (c < n_valid) {
    uint16_t e[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) e[k] = c + k < n_valid ? src[k] : (uint16_t)0;
    v = make_uint4((unsigned)e[0] | ((unsigned)e[1] << 16), (unsigned)e[2] | ((unsigned)e[3] << 16),
                   (unsigned)e[4] | ((unsigned)e[5] << 16), (unsigned)e[6] | ((unsigned)e[7] << 16));
  }
  *reinterpret_cast<uint4 *>(D + r * ldd + c) = v;
}

}  // namespace deinfer
