// Paged low-rank cache -> compact buffer, and the in-place rotary embedding of the rebuilt keys
// (Sec. 4.2: "graph replay stage").  Both kernels take everything that changes from step to step
// (the run list, the token positions) from device memory and have a grid that depends only on
// capacities, so a captured launch stays valid when the cache contents change.
#pragma once
#include "common.h"

namespace deinfer {

constexpr int KV_PLAN_HEADER = 4;            // int32 words before the (src, dst, length) triples
constexpr int KV_COPY_THREADS = 256;
constexpr int KV_PIECE = KV_COPY_THREADS * 4 * 16;   // bytes one workgroup moves per step (16 KiB)
constexpr int KV_LDS_RUNS = 2048;            // run destinations a workgroup keeps in LDS (8 KiB)

// plan: [0] number of runs, [1] number of blocks (sum of the lengths), then the runs in the order
// of their destinations, which tile [0, plan[1]) without gaps.  A piece p = (destination block,
// 16 KiB slice of it) finds its run by bisection over the destinations.  Entries that point
// outside the pool or the buffer are skipped, so a damaged plan cannot cause an access fault.
__global__ __launch_bounds__(KV_COPY_THREADS) void kv_compact_copy_kernel(
    const unsigned char *pool, long long n_pool_blocks, long long block_bytes, const int *plan, int plan_capacity,
    unsigned char *buffer, long long buffer_blocks) {
  int n_runs = plan[0];
  n_runs = n_runs < plan_capacity ? n_runs : plan_capacity;
  long long nb = plan[1];
  nb = nb < buffer_blocks ? nb : buffer_blocks;
  if (n_runs <= 0 || nb <= 0) return;
  const int *runs = plan + KV_PLAN_HEADER;
  const long long ppb = (block_bytes + KV_PIECE - 1) / KV_PIECE;
  if ((long long)blockIdx.x >= nb * ppb) return;
  // The destinations of the runs go to LDS first (one round trip to memory), so that the bisection
  // of every piece is a handful of LDS reads and not a chain of dependent global loads; run lists
  // too long for that are bisected in global memory.
  __shared__ int dst_of[KV_LDS_RUNS];
  const bool in_lds = n_runs <= KV_LDS_RUNS;
  if (in_lds) {
    for (int i = threadIdx.x; i < n_runs; i += KV_COPY_THREADS) dst_of[i] = runs[3 * i + 1];
    __syncthreads();
  }
  for (long long p = blockIdx.x; p < nb * ppb; p += gridDim.x) {
    const long long d = p / ppb, c = p - d * ppb;
    int lo = 0, hi = n_runs - 1;               // last run whose destination is <= d
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((in_lds ? dst_of[mid] : runs[3 * mid + 1]) <= d) lo = mid; else hi = mid - 1;
    }
    const long long src0 = runs[3 * lo], dst0 = runs[3 * lo + 1], len = runs[3 * lo + 2];
    const long long off = d - dst0, src = src0 + off;
    if (off < 0 || off >= len || src < 0 || src >= n_pool_blocks) continue;
    const long long lo_b = c * KV_PIECE;
    const long long n16 = ((block_bytes - lo_b < KV_PIECE ? block_bytes - lo_b : KV_PIECE)) / 16;
    const u32x4_t *s = reinterpret_cast<const u32x4_t *>(pool + src * block_bytes + lo_b);
    u32x4_t *t = reinterpret_cast<u32x4_t *>(buffer + d * block_bytes + lo_b);
    u32x4_t v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long long k = threadIdx.x + i * KV_COPY_THREADS;
      v[i] = u32x4_t{0u, 0u, 0u, 0u};
      if (k < n16) v[i] = __builtin_nontemporal_load(s + k);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long long k = threadIdx.x + i * KV_COPY_THREADS;
      if (k < n16) t[k] = v[i];
    }
  }
}

// Rotary embedding in place.  One thread = one token and one group of 8 pair indices i (angles
// depend on the token position and i only), looping over the heads.  Angles in double precision
// (a position of several thousand times a frequency near 1 leaves too few bits in single).
//   x[t, h D + i]       <- a cos - b sin
//   x[t, h D + i + D/2] <- b cos + a sin        a, b = the old values, angle = pos theta^(-2 i / D)
template <typename TE>
__global__ __launch_bounds__(256) void rope_inplace_kernel(TE *x, long long T, long long ldx, int n_heads, int head_dim,
                                                           const int *positions, double log2_theta) {
  const int half = head_dim / 2;
  const int chunks = (half + 7) / 8;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long tok = idx / chunks;
  const int i0 = (int)(idx % chunks) * 8;
  if (tok >= T) return;
  const double pos = (double)positions[tok];
  float cs[8], sn[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double ang = pos * exp2(-2.0 * (double)(i0 + e) / (double)head_dim * log2_theta);
    double s, c;
    sincos(ang, &s, &c);
    cs[e] = (float)c; sn[e] = (float)s;
  }
  TE *row = x + tok * ldx;
  const int n = half - i0 < 8 ? half - i0 : 8;
  const bool vec = n == 8 && sizeof(TE) == 2 && ((reinterpret_cast<uintptr_t>(row) & 15u) == 0) && (head_dim % 16 == 0);
  for (int h = 0; h < n_heads; ++h) {
    TE *pa = row + (long long)h * head_dim + i0, *pb = pa + half;
    if (vec) {
      const u32x4_t va = *reinterpret_cast<const u32x4_t *>(pa), vb = *reinterpret_cast<const u32x4_t *>(pb);
      u32x4_t ra, rb;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        constexpr int DT = DtOf<TE>::value == DT_F16 ? DT_F16 : DT_BF16;
        const float a0 = lo_f32<DT>(va[w]), a1 = hi_f32<DT>(va[w]);
        const float b0 = lo_f32<DT>(vb[w]), b1 = hi_f32<DT>(vb[w]);
        ra[w] = pack2<DT>(a0 * cs[2 * w] - b0 * sn[2 * w], a1 * cs[2 * w + 1] - b1 * sn[2 * w + 1]);
        rb[w] = pack2<DT>(b0 * cs[2 * w] + a0 * sn[2 * w], b1 * cs[2 * w + 1] + a1 * sn[2 * w + 1]);
      }
      *reinterpret_cast<u32x4_t *>(pa) = ra;
      *reinterpret_cast<u32x4_t *>(pb) = rb;
    } else {
      for (int e = 0; e < n; ++e) {
        const float a = Elem<TE>::load(pa + e), b = Elem<TE>::load(pb + e);
        Elem<TE>::store(pa + e, a * cs[e] - b * sn[e]);
        Elem<TE>::store(pb + e, b * cs[e] + a * sn[e]);
      }
    }
  }
}

// cos / sin of the rotary angles of every token: table[t][i] = cos(pos_t theta^(-2 i / D)),
// table[t][D / 2 + i] = sin(...), i < D / 2 (fp32, angles in double precision).  One thread per
// (token, i).  The upward projection with a rotary epilogue reads it.
__global__ __launch_bounds__(256) void rope_table_kernel(const int *positions, long long T, int head_dim, double log2_theta, float *table) {
  const int half = head_dim / 2;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * half) return;
  const long long tok = idx / half;
  const int i = (int)(idx - tok * half);
  const double ang = (double)positions[tok] * exp2(-2.0 * (double)i / (double)head_dim * log2_theta);
  double s, c;
  sincos(ang, &s, &c);
  table[tok * head_dim + i] = (float)c;
  table[tok * head_dim + half + i] = (float)s;
}

// Rotary embedding in place from the table (the path of deinfer_lowrank_up_rope where the
// epilogue of the large-T kernel does not apply).  One thread per (token, head, pair index).
template <typename TE>
__global__ __launch_bounds__(256) void rope_from_table_kernel(TE *x, long long T, long long ldx, int n_heads, int head_dim, const float *table) {
  const int half = head_dim / 2;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * n_heads * half) return;
  const int i = (int)(idx % half);
  const long long th = idx / half;
  const int h = (int)(th % n_heads);
  const long long tok = th / n_heads;
  const float c = table[tok * head_dim + i], sn = table[tok * head_dim + half + i];
  TE *pa = x + tok * ldx + (long long)h * head_dim + i, *pb = pa + half;
  const float a = Elem<TE>::load(pa), b = Elem<TE>::load(pb);
  Elem<TE>::store(pa, a * c - b * sn);
  Elem<TE>::store(pb, b * c + a * sn);
}

}  // namespace deinfer
