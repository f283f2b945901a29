// Memory-bound second stage of the GLU call (Sec. 4.1: "activation computation" after the upward
// projections; Table 2: GLU-based MLP) for 16 < T <= 128 tokens, PACKED pairs:
//
//   h[T x F] = silu(t_gate . V_gate) * (t_up . V_up)
//
// in ONE launch without partial sums: a workgroup owns 32 NW output features over the whole rank
// range; half of its wavefronts multiply the gate blocks, the other half the up blocks of the same
// features, and the up sums cross LDS once at the end, so silu and the product are taken on-chip and
// h is stored once.  The full-width gate and up results never reach memory.
//
// Otherwise the scheme of skinny_kernel.h: weights straight into registers with non-temporal 16-byte
// loads (two per k-block and product), the two [T x 64 k] activation slabs of a stage (rank-space
// rows of the gate pair and of the up pair) shared by the wavefronts through LDS (global -> LDS
// loads, 128-byte rows with swizzled 16-byte slots), 32x32x16 MFMA with tokens as columns, four
// register sets / slab pairs so that three stages of loads are in flight, two wavefronts per SIMD.
#pragma once
#include "common.h"
#include "skinny_kernel.h"

namespace deinfer {

constexpr int SG_KBS = 2;                  // k-blocks per stage and product
constexpr int SG_XROW = SG_KBS * 64;       // bytes per token row of a slab
constexpr int SG_SLABS = 4;

struct SkGluParams {
  int T;
  SkProblem gate, up;        // act, lda, frags, K, KB, n_ftiles (the same feature tiles for both)
  uint16_t *out;             // h, row-major, 16-bit storage type
  long long ldo;
  int width;                 // valid output columns (d_ff)
};

constexpr size_t sk_glu_lds_bytes(int NB) { return (size_t)SG_SLABS * 2 * NB * 32 * SG_XROW; }

// NB = 32-token blocks (1, 2 or 4); NW = 32-feature blocks per workgroup (4).  The workgroup has 2 NW
// wavefronts, two per SIMD: wavefront w < NW multiplies the gate block w, wavefront NW + w the up
// block w of the same output features.  (What a compute unit can take in, weights from HBM and slabs
// from L2 together, grows with the wavefronts that issue loads: measured 51 GB/s with four and 65 GB/s
// with eight at equal shares of both, and at 128 tokens the slabs are as many bytes as the weights.)
// TAIL: as in skinny_kernel.h (rank-space rows whose valid columns are no multiple of 8).
template <int DT, int NB, int NW, bool TAIL = false>
__global__ __launch_bounds__(128 * NW, 1) void skinny_glu_kernel(const SkGluParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  constexpr int KBS = SG_KBS, XROW = SG_XROW;
  constexpr int SPR = KBS * 4;            // 16-byte slots per row = lanes per row of a slab load (8)
  constexpr int RPI = 64 / SPR;           // rows per slab load instruction (8)
  constexpr int SLAB = NB * 32 * XROW;    // bytes of one product's slab of one stage
  extern __shared__ __attribute__((aligned(16))) unsigned char sg_lds[];      // [SG_SLABS][2][SLAB]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int prod = wave / NW, fw = wave % NW;            // 0: gate, 1: up; feature block inside the workgroup
  const int fblk = blockIdx.x * NW + fw;                 // this wavefront's 32-feature block
  // a 128-byte row spans half of the banks: the slot is XORed with (row / 2) % 8 (see skinny_kernel.h)
  auto swz = [](int row) { return (row >> 1) & (SPR - 1); };

  constexpr unsigned OOB = 0x7ffffff0u;
  const SkProblem &Q = prod == 0 ? P.gate : P.up;
  const int KBq = Q.KB;
  const unsigned wbytes = (unsigned)Q.n_ftiles * (unsigned)Q.KB * 1024u;
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.frags, 0, (int)wbytes, 0x00020000);
  // lane l holds feature l % 32 (tile 2 fblk + (l / 16) % 2, row l % 16) and k-group 2 s + l / 32
  const unsigned wtile = (unsigned)(2 * fblk + ((lane >> 4) & 1));
  const unsigned wlane = (int)wtile < Q.n_ftiles ? wtile * (unsigned)Q.KB * 1024u + (unsigned)(((lane & 15) + 16 * (lane >> 5)) * 16) : OOB;
  const unsigned xbytes = (unsigned)(((long long)(P.T - 1) * Q.lda + ((Q.K + 7) & ~7)) * 2);
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)xbytes, 0x00020000);
  const unsigned xkend = (unsigned)(((Q.K + 7) >> 3) * 16);      // bytes of a row up to the end of the chunk that holds column K - 1
  const unsigned xklim = (unsigned)(Q.K * 2 - 16);               // (K a multiple of 8: the last chunk)
  // the chunk with columns that are not to be used (lds_zero_chunk_tail in common.h): its stage and slot,
  // per product; the barrier that follows the fix is taken by every wavefront when either product has one there
  const int krem = Q.K & 7;
  const int st_fix = (TAIL && krem != 0) ? (Q.K >> 5) / KBS : -1;
  const int slot_fix = ((Q.K >> 5) % KBS) * 4 + ((Q.K >> 3) & 3);
  const int st_fix_gate = (TAIL && (P.gate.K & 7) != 0) ? (P.gate.K >> 5) / KBS : -1;
  const int st_fix_up = (TAIL && (P.up.K & 7) != 0) ? (P.up.K >> 5) / KBS : -1;
  constexpr int NI = NB * 32 / RPI;                     // slab load instructions per stage and product
  constexpr int NX = NI / NW;                           // ... per wavefront of the product
  static_assert(NI % NW == 0, "every wavefront issues the same number of slab loads");
  unsigned xrow[NX], xchunk[NX];
  int xm[NX];
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const int m = i * NW + fw;                          // instruction m covers rows RPI m .. RPI m + RPI - 1
    xm[i] = m;
    const int row = RPI * m + lane / SPR;
    xchunk[i] = (unsigned)(((lane & (SPR - 1)) ^ swz(row)) * 16);
    xrow[i] = row < P.T ? (unsigned)row * (unsigned)(Q.lda * 2) : OOB;
  }
  const int kb_max = P.gate.KB > P.up.KB ? P.gate.KB : P.up.KB;
  const int n_stages = (kb_max + KBS - 1) / KBS;        // the same for both products: the stage barriers are shared
  unsigned char *const slabs = sg_lds + prod * SLAB;    // this product's slab of stage buffer b: slabs + b * 2 * SLAB

  // One load of stage `fst` into register set wn / stage buffer fbuf: the weights, then this wavefront's slab rows.
  constexpr int NWL = KBS * 2;                          // weight loads per stage
  constexpr int NLOAD = NWL + NX;
  auto fetch_one = [&](u32x4_t (&wn)[NWL], int fst, int fbuf, int idx) {
    if (idx < NWL) {
      const int kb = fst * KBS + (idx >> 1);
      const unsigned off = kb < KBq ? wlane : OOB;                // k-blocks past the product's range read zeros
      wn[idx] = __builtin_amdgcn_raw_buffer_load_b128(wres, off, kb * 1024 + (idx & 1) * 512, 2);
    } else {
      const int i = idx - NWL;
      const unsigned dead = fst * KBS < KBq ? 0u : OOB;
      // chunks beyond K re-read a chunk of valid columns (the last one; TAIL: the first one), which meets zero weights
      unsigned kb = (unsigned)(fst * KBS) * 64u + xchunk[i];
      kb = TAIL ? (kb < xkend ? kb : 0u) : (kb < xklim ? kb : xklim);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LDS_PTR void *)(slabs + fbuf * 2 * SLAB + xm[i] * RPI * XROW), 16,
                                               (xrow[i] + kb) | dead, 0, 0, 0);
    }
  };

  f32x16_t acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  const int b_row = lane & 31;
  // A stage is 4 steps (k-block, half) of NB matrix products; the token operands are read from LDS
  // DEPTH steps ahead of their use into rotating registers, one read after each product
  constexpr int STEPS = NWL;
  constexpr int DEPTH = NB >= 4 ? 2 : 3;
  auto read_b = [&](int buf, int step, int j) -> u32x4_t {      // step = 2 * k-block + half: 16-byte slot 2 * step + lane / 32
    const int slot = (step * 2 + (lane >> 5)) ^ swz(b_row);
    return *reinterpret_cast<const u32x4_t *>(slabs + buf * 2 * SLAB + (32 * j + b_row) * XROW + slot * 16);
  };
  auto compute = [&](const u32x4_t (&w)[NWL], int buf, u32x4_t (&wn)[NWL], int fst, int fbuf) {
    constexpr int NPOS = STEPS * NB;
    u32x4_t b[DEPTH + 1][NB];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
#pragma unroll
      for (int j = 0; j < NB; ++j) b[d][j] = read_b(buf, d, j);
#pragma unroll
    for (int step = 0; step < STEPS; ++step) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        __builtin_amdgcn_sched_barrier(0);
        acc[j] = mfma32<DT>(w[step], b[step % (DEPTH + 1)][j], acc[j]);
        __builtin_amdgcn_sched_barrier(0);
        if (step + DEPTH < STEPS) b[(step + DEPTH) % (DEPTH + 1)][j] = read_b(buf, step + DEPTH, j);
        const int pos = step * NB + j;
#pragma unroll
        for (int idx = pos * NLOAD / NPOS; idx < (pos + 1) * NLOAD / NPOS; ++idx) fetch_one(wn, fst, fbuf, idx);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Stage s uses register set / stage buffer s % 4.  Every stage issues exactly NLOAD loads (those past
  // the k-range read zeros through an out-of-range offset and cost no traffic), so "all but the
  // loads of the next two stages have arrived" is one constant wait.
  static_assert((SG_SLABS - 1) * NLOAD < 64, "the load counter has 6 bits");
  if (n_stages > 0) {
    u32x4_t w0[NWL], w1[NWL], w2[NWL], w3[NWL];
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w0, 0, 0, idx);
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w1, 1, 1, idx);
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w2, 2, 2, idx);
    auto stage = [&](const u32x4_t (&w)[NWL], u32x4_t (&wn)[NWL], int st, int slab) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((SG_SLABS - 2) * NLOAD) : "memory");
      __builtin_amdgcn_s_barrier();                     // stage st has arrived everywhere; nobody reads stage buffer (st - 1) % 4 any more
      asm volatile("" ::: "memory");
      if constexpr (TAIL) {
        if (st == st_fix_gate || st == st_fix_up) {     // (uniform over the workgroup)
          const int row = fw * 64 + lane;               // the product's wavefronts share out its slab's rows
          if (st == st_fix && row < NB * 32)
            lds_zero_chunk_tail(slabs + slab * 2 * SLAB + row * XROW + ((slot_fix ^ swz(row)) * 16), krem);
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
      }
      compute(w, slab, wn, st + SG_SLABS - 1, slab == 0 ? SG_SLABS - 1 : slab - 1);
    };
    for (int st = 0; st < n_stages; st += 4) {
      stage(w0, w3, st, 0);
      if (st + 1 >= n_stages) break;
      stage(w1, w0, st + 1, 1);
      if (st + 2 >= n_stages) break;
      stage(w2, w1, st + 2, 2);
      if (st + 3 >= n_stages) break;
      stage(w3, w2, st + 3, 3);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // drain the out-of-range tail loads before LDS is reused
  }

  // ---- the up wavefronts hand their sums to the gate wavefronts of the same features through LDS
  // (element 4 q + e of block j is feature 8 q + 4 (l / 32) + e, token 32 j + l % 32)
  static_assert(sk_glu_lds_bytes(NB) >= (size_t)NW * NB * 4 * 64 * 16, "the exchange buffer fits the slab space");
  __syncthreads();                                        // every wavefront has read its last operands
  float4 *const xch = reinterpret_cast<float4 *>(sg_lds);   // [fw][j][q][lane]
  if (prod == 1) {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        xch[((fw * NB + j) * 4 + q) * 64 + lane] = make_float4(acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]);
  }
  __syncthreads();
  if (prod == 1) return;
  // ---- h = silu(gate) * up
  const int col0 = fblk * 32 + 4 * (lane >> 5);
  uint16_t *o = P.out + (long long)(lane & 31) * P.ldo;
  const bool vec = (reinterpret_cast<uintptr_t>(P.out) & 7u) == 0 && (P.ldo & 3) == 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int col = col0 + 8 * q;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      if (32 * j + (lane & 31) >= P.T) continue;
      const float4 u = xch[((fw * NB + j) * 4 + q) * 64 + lane];
      const float v[4] = {silu_f32(acc[j][4 * q + 0]) * u.x, silu_f32(acc[j][4 * q + 1]) * u.y,
                          silu_f32(acc[j][4 * q + 2]) * u.z, silu_f32(acc[j][4 * q + 3]) * u.w};
      uint16_t *dst = o + (long long)(32 * j) * P.ldo + col;
      if (vec && col + 4 <= P.width) {
        *reinterpret_cast<uint2 *>(dst) = uint2{pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3])};
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (col + e < P.width) dst[e] = cvt_out<DT>(v[e]);
      }
    }
  }
#else
  (void)P;
#endif
}

}  // namespace deinfer
