// Memory-bound ("decode", T <= 128 tokens) kernel for PACKED bf16 factor pairs.
//
// One persistent launch per entry-point call, one 512-thread workgroup per compute
// unit, two phases separated by a single grid barrier:
//
//   phase 1  t = x . [U_a | U_b | U_c]   downward projections of up to three pairs as
//            one concatenated product (Sec. 4.1).  The fragment stream of the packed
//            U image is cut into equal contiguous ranges, one per workgroup, so every
//            compute unit pulls the same number of bytes whatever the ranks are.  A
//            16-wide rank tile that straddles a range boundary is completed by the
//            workgroup where the tile starts: the others leave their partial sums in
//            a slot and raise a flag (fixed summation order -> deterministic).
//            t is kept as bf16 (one nearest-even rounding) in the workspace, which is
//            small enough (<= 1.3 MB) to live in L2 / Infinity Cache.
//   phase 2  y = t . V per pair (upward projections), 16 output features per work item,
//            the 8 wavefronts of a workgroup split the rank dimension and reduce
//            through LDS ("split-r"); optional SiLU-GLU epilogue for the gate/up call.
//
// Operands: weights are the MFMA A operand (16 features x 32 k fragments, one coalesced
// 1 KiB load per wavefront), activations the B operand (16 tokens x 32 k), so the
// accumulator holds [feature][token]; T is padded to a multiple of 16 tokens.
#pragma once
#include "common.h"

namespace deinfer {

constexpr int DEC_THREADS = 512;
constexpr int DEC_WAVES = DEC_THREADS / kWave;
constexpr int DEC_MAX_GRID = 1024;          // flag words reserved in the workspace header
constexpr unsigned long long DEC_SPIN_LIMIT = 200000000ull;  // 2 s of the 100 MHz wall clock

struct DecPair {
  const uint4 *Up;      // packed U fragments [r_pad/16][KB1][64]
  const uint4 *Vp;      // packed V fragments [n_otiles][r_pad/32][64]
  uint16_t *y;          // output (bf16); for the GLU call only pair 0 carries the output
  long long ldy;
  uint16_t *t_out;      // optional copy of this pair's rank-space result (may be null)
  long long ldt_out;
  int r;                // true rank
  int r_pad;            // multiple of 32
  int d_out;
  int n_otiles;         // ceil(d_out / 16)
  int tile0;            // first 16-wide rank tile of this pair in the concatenated t
};

struct DecParams {
  const uint16_t *x;
  long long ldx;
  int T, d_in, KB1;     // KB1 = ceil(d_in / 32)
  int n_pairs;
  DecPair p[3];
  int n_rtiles;         // total rank tiles = Rtot_pad / 16
  int Rtot_pad;         // pitch of t in elements
  uint16_t *t;          // [T16][Rtot_pad]
  float4 *slots;        // [grid][NT][64] partial sums of straddling tiles
  unsigned *flags;      // [grid]
  unsigned *bar;        // [0] arrivals, [1] generation, [2] error
  int n_items2;         // phase-2 work items
  int G1;               // workgroups that take a phase-1 range: min(grid, n_rtiles * KB1)
};

__device__ __forceinline__ bool spin_until_set(unsigned *flag, unsigned *err) {
  const unsigned long long t0 = wall_clock64();
  while (__hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
    __builtin_amdgcn_s_sleep(1);
    if (wall_clock64() - t0 > DEC_SPIN_LIMIT) {
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return false;
    }
  }
  return true;
}

// Self-resetting barrier over all workgroups of the (co-resident) grid.  Returns false
// if the wait was abandoned (error word set); callers then skip their remaining work.
__device__ __forceinline__ bool grid_barrier(unsigned *bar, unsigned nwg) {
  __shared__ int ok_s;
  __syncthreads();
  if (threadIdx.x == 0) {
    int ok = 1;
    const unsigned gen = __hip_atomic_load(bar + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned prev = __hip_atomic_fetch_add(bar, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (prev == nwg - 1) {
      __hip_atomic_store(bar, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(bar + 1, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      const unsigned long long t0 = wall_clock64();
      while (__hip_atomic_load(bar + 1, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == gen) {
        __builtin_amdgcn_s_sleep(1);
        if (wall_clock64() - t0 > DEC_SPIN_LIMIT) {
          __hip_atomic_store(bar + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = 0;
          break;
        }
      }
    }
    ok_s = ok;
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return ok_s != 0;
}

template <int NT>
struct DecUnroll { static constexpr int value = NT == 1 ? 8 : NT == 2 ? 4 : 2; };

// One split-k sweep: acc[nt] += W_frag(kb) x act(kb) for kb = kb_begin + wave, +8, ... < kb_end.
// wfrag points at fragment 0 of the tile (+ lane); act[nt] at the lane's 8 bf16 of k-block 0
// for token tile nt.  k_lim masks activation reads beyond the true reduction length.
template <int NT>
__device__ __forceinline__ void sweep(const uint4 *__restrict__ wfrag, const uint16_t *const (&act)[NT],
                                      int kb_begin, int kb_end, int wave, int k_lane, int k_lim,
                                      const uint16_t *__restrict__ safe, f32x4_t (&acc)[NT]) {
  constexpr int UN = DecUnroll<NT>::value;
  for (int kb0 = kb_begin + wave; kb0 < kb_end; kb0 += DEC_WAVES * UN) {
    u32x4_t a[UN];
    u32x4_t b[UN][NT];
#pragma unroll
    for (int i = 0; i < UN; ++i) {
      const int kb = kb0 + i * DEC_WAVES;
      const bool ok = kb < kb_end;
      const int kbc = ok ? kb : kb0;
      a[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(wfrag + (long long)kbc * 64));
      const bool kok = ok && (kbc * 32 + k_lane < k_lim);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        // lanes beyond the reduction length read a valid dummy address and contribute zero
        const uint16_t *src = kok ? act[nt] + (long long)kbc * 32 : safe;
        const u32x4_t v = *reinterpret_cast<const u32x4_t *>(src);
        b[i][nt] = kok ? v : u32x4_t{0u, 0u, 0u, 0u};
      }
    }
#pragma unroll
    for (int i = 0; i < UN; ++i)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a[i]), as_bf16x8(b[i][nt]), acc[nt], 0, 0, 0);
  }
}

template <int NT, bool DUAL>
__global__ __launch_bounds__(DEC_THREADS) void decode_kernel(const DecParams P) {
  __shared__ float4 red[DUAL ? 2 : 1][DEC_WAVES][NT][kWave];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 15, lkg = lane >> 4;
  const int G = gridDim.x, g = blockIdx.x;

  // ------------------------------------------------------------------ phase 1: t = x . U
  {
    const uint16_t *xact[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int tok = nt * 16 + lrow;
      tok = tok < P.T ? tok : P.T - 1;
      xact[nt] = P.x + (long long)tok * P.ldx + lkg * 8;
    }
    const long long total = (long long)P.n_rtiles * P.KB1;
    // only the first G1 = min(G, total) workgroups take a (non-empty) range
    const int G1 = P.G1;
    const long long ua = g < G1 ? (long long)g * total / G1 : total;
    const long long ub = g < G1 ? (long long)(g + 1) * total / G1 : total;
    long long u = ua;
    while (u < ub) {
      const int tile = (int)(u / P.KB1);
      const long long tbeg = (long long)tile * P.KB1, tend = tbeg + P.KB1;
      const long long se = ub < tend ? ub : tend;
      const bool starts = (u == tbeg), ends = (se == tend);
      int pi = 0;
      if (P.n_pairs > 1 && tile >= P.p[1].tile0) pi = 1;
      if (P.n_pairs > 2 && tile >= P.p[2].tile0) pi = 2;
      const DecPair &pr = P.p[pi];
      const uint4 *wfrag = pr.Up + (long long)(tile - pr.tile0) * P.KB1 * 64 + lane;

      f32x4_t acc[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      sweep<NT>(wfrag, xact, (int)(u - tbeg), (int)(se - tbeg), wave, lkg * 8, P.d_in, P.x, acc);

#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        red[0][wave][nt][lane] = make_float4(acc[nt][0], acc[nt][1], acc[nt][2], acc[nt][3]);
      __syncthreads();

      const bool owner_wait = starts && !ends;
      int g_last = g;
      if (owner_wait) {
        // workgroup that holds the last k-block of this tile
        g_last = (int)((tend * G1 + total - 1) / total) - 1;
        if (tid == 0)
          for (int gg = g + 1; gg <= g_last; ++gg) spin_until_set(P.flags + gg, P.bar + 2);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
      if (tid < NT * kWave) {
        const int nt = wave;
        float4 s = red[0][0][nt][lane];
#pragma unroll
        for (int w = 1; w < DEC_WAVES; ++w) {
          const float4 v = red[0][w][nt][lane];
          s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        if (!starts) {
          P.slots[((long long)g * NT + nt) * kWave + lane] = s;
        } else {
          for (int gg = g + 1; gg <= g_last; ++gg) {
            const float4 v = P.slots[((long long)gg * NT + nt) * kWave + lane];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
          }
          const int tok = nt * 16 + lrow;
          const int col = tile * 16 + lkg * 4;
          uint2 pk;
          pk.x = pack_bf16x2(s.x, s.y);
          pk.y = pack_bf16x2(s.z, s.w);
          *reinterpret_cast<uint2 *>(P.t + (long long)tok * P.Rtot_pad + col) = pk;
          if (pr.t_out != nullptr && tok < P.T) {
            const int c0 = (tile - pr.tile0) * 16 + lkg * 4;
            const float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (c0 + v < pr.r) pr.t_out[(long long)tok * pr.ldt_out + c0 + v] = f32_to_bf16(sv[v]);
          }
        }
      }
      if (!starts) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (tid == 0) __hip_atomic_store(P.flags + g, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
      } else if (owner_wait) {
        __syncthreads();
        if (tid == 0)
          for (int gg = g + 1; gg <= g_last; ++gg)
            __hip_atomic_store(P.flags + gg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();
      u = se;
    }
  }

  if (!grid_barrier(P.bar, (unsigned)G)) return;

  // ------------------------------------------------------------------ phase 2: y = t . V
  for (int it = g; it < P.n_items2; it += G) {
    int pi = 0, otile = it;
    if (!DUAL) {
      if (P.n_pairs > 1 && otile >= P.p[0].n_otiles) { otile -= P.p[0].n_otiles; pi = 1; }
      if (P.n_pairs > 2 && pi == 1 && otile >= P.p[1].n_otiles) { otile -= P.p[1].n_otiles; pi = 2; }
    }
    f32x4_t acc[NT], acc2[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f}; acc2[nt] = acc[nt]; }
    {
      const DecPair &pr = P.p[pi];
      const int KB2 = pr.r_pad >> 5;
      const uint16_t *tact[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        tact[nt] = P.t + (long long)(nt * 16 + lrow) * P.Rtot_pad + pr.tile0 * 16 + lkg * 8;
      sweep<NT>(pr.Vp + (long long)otile * KB2 * 64 + lane, tact, 0, KB2, wave, lkg * 8, pr.r_pad, P.t, acc);
    }
    if (DUAL) {
      const DecPair &pr = P.p[1];
      const int KB2 = pr.r_pad >> 5;
      const uint16_t *tact[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        tact[nt] = P.t + (long long)(nt * 16 + lrow) * P.Rtot_pad + pr.tile0 * 16 + lkg * 8;
      sweep<NT>(pr.Vp + (long long)otile * KB2 * 64 + lane, tact, 0, KB2, wave, lkg * 8, pr.r_pad, P.t, acc2);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      red[0][wave][nt][lane] = make_float4(acc[nt][0], acc[nt][1], acc[nt][2], acc[nt][3]);
      if (DUAL) red[DUAL ? 1 : 0][wave][nt][lane] = make_float4(acc2[nt][0], acc2[nt][1], acc2[nt][2], acc2[nt][3]);
    }
    __syncthreads();
    if (tid < NT * kWave) {
      const int nt = wave;
      float4 s = red[0][0][nt][lane];
#pragma unroll
      for (int w = 1; w < DEC_WAVES; ++w) {
        const float4 v = red[0][w][nt][lane];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      if (DUAL) {
        float4 s2 = red[DUAL ? 1 : 0][0][nt][lane];
#pragma unroll
        for (int w = 1; w < DEC_WAVES; ++w) {
          const float4 v = red[DUAL ? 1 : 0][w][nt][lane];
          s2.x += v.x; s2.y += v.y; s2.z += v.z; s2.w += v.w;
        }
        s.x = silu_f32(s.x) * s2.x; s.y = silu_f32(s.y) * s2.y;
        s.z = silu_f32(s.z) * s2.z; s.w = silu_f32(s.w) * s2.w;
      }
      const DecPair &pr = P.p[pi];
      const int tok = nt * 16 + lrow;
      const int f0 = otile * 16 + lkg * 4;
      if (tok < P.T) {
        uint16_t *dst = pr.y + (long long)tok * pr.ldy + f0;
        if (f0 + 3 < pr.d_out && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
          uint2 pk;
          pk.x = pack_bf16x2(s.x, s.y);
          pk.y = pack_bf16x2(s.z, s.w);
          *reinterpret_cast<uint2 *>(dst) = pk;
        } else {
          const float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (f0 + v < pr.d_out) dst[v] = f32_to_bf16(sv[v]);
        }
      }
    }
    __syncthreads();
  }
}

}  // namespace deinfer
