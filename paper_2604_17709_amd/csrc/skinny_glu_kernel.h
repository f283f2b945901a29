// Memory-bound second stage of the GLU call (Sec. 4.1: "activation computation" after the upward
// projections; Table 2: GLU-based MLP) for 16 < T <= 128 tokens, PACKED pairs:
//
//   h[T x F] = silu(t_gate . V_gate) * (t_up . V_up)
//
// in ONE launch without partial sums: a workgroup owns 32 NW output features over the whole rank
// range, and every wavefront multiplies BOTH products of its 32 features (gate block and up block on
// two accumulator sets), so silu and the product are taken on registers and h is stored once.  The
// full-width gate and up results never reach memory.
//
// Otherwise the scheme of skinny_kernel.h: weights straight into registers with non-temporal 16-byte
// loads (two per k-block and product), the two [T x 64 k] activation slabs of a stage (rank-space
// rows of the gate pair and of the up pair) shared by the wavefronts through LDS (global -> LDS
// loads, 128-byte rows with swizzled 16-byte slots), 32x32x16 MFMA with tokens as columns, four
// register sets / slab pairs so that three stages of loads are in flight, one wavefront per SIMD.
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

// NB = 32-token blocks (1, 2 or 4); NW = wavefronts per workgroup = 32-feature blocks per workgroup (4 is
// what the host launches: 2 was measured slower than the split with partial sums wherever it applied)
template <int DT, int NB, int NW>
__global__ __launch_bounds__(64 * NW, 1) void skinny_glu_kernel(const SkGluParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  constexpr int KBS = SG_KBS, XROW = SG_XROW;
  constexpr int SPR = KBS * 4;            // 16-byte slots per row = lanes per row of a slab load (8)
  constexpr int RPI = 64 / SPR;           // rows per slab load instruction (8)
  constexpr int SLAB = NB * 32 * XROW;    // bytes of one product's slab of one stage
  extern __shared__ __attribute__((aligned(16))) unsigned char sg_lds[];      // [SG_SLABS][2][SLAB]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fblk = blockIdx.x * NW + wave;               // this wavefront's 32-feature block (gate and up)
  // a 128-byte row spans half of the banks: the slot is XORed with (row / 2) % 8 (see skinny_kernel.h)
  auto swz = [](int row) { return (row >> 1) & (SPR - 1); };

  constexpr unsigned OOB = 0x7ffffff0u;
  __amdgpu_buffer_rsrc_t wres[2], xres[2];
  unsigned wlane[2], xklim[2];
  int KBp[2];
  constexpr int NI = NB * 32 / RPI;                     // slab load instructions per stage and product
  constexpr int NX = (NI + NW - 1) / NW;                // ... per wavefront
  static_assert(NI % NW == 0, "every wavefront issues the same number of slab loads");
  unsigned xrow[2][NX], xchunk[NX];
  int xm[NX];
  long long ldap[2];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const SkProblem &Qp = p == 0 ? P.gate : P.up;
    KBp[p] = Qp.KB;
    ldap[p] = Qp.lda;
    const unsigned wbytes = (unsigned)Qp.n_ftiles * (unsigned)Qp.KB * 1024u;
    wres[p] = __builtin_amdgcn_make_buffer_rsrc((void *)Qp.frags, 0, (int)wbytes, 0x00020000);
    // lane l holds feature l % 32 (tile 2 fblk + (l / 16) % 2, row l % 16) and k-group 2 s + l / 32
    const unsigned wtile = (unsigned)(2 * fblk + ((lane >> 4) & 1));
    wlane[p] = (int)wtile < Qp.n_ftiles ? wtile * (unsigned)Qp.KB * 1024u + (unsigned)(((lane & 15) + 16 * (lane >> 5)) * 16) : OOB;
    const unsigned xbytes = (unsigned)(((long long)(P.T - 1) * Qp.lda + Qp.K) * 2);
    xres[p] = __builtin_amdgcn_make_buffer_rsrc((void *)Qp.act, 0, (int)xbytes, 0x00020000);
    xklim[p] = (unsigned)(Qp.K * 2 - 16);
  }
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const int m = i * NW + wave;                        // instruction m covers rows RPI m .. RPI m + RPI - 1
    xm[i] = m;
    const int row = RPI * m + lane / SPR;
    xchunk[i] = (unsigned)(((lane & (SPR - 1)) ^ swz(row)) * 16);
#pragma unroll
    for (int p = 0; p < 2; ++p) xrow[p][i] = row < P.T ? (unsigned)row * (unsigned)(ldap[p] * 2) : OOB;
  }
  const int kb_max = KBp[0] > KBp[1] ? KBp[0] : KBp[1];
  const int n_stages = (kb_max + KBS - 1) / KBS;

  // One load of stage `fst` into register set wn / slab pair fbuf: index 0 .. 8 * KBS / 2 - 1 ... the
  // weights of the gate product, then of the up product, then the slab rows of both.
  constexpr int NWL = KBS * 2;                          // weight loads per product and stage
  constexpr int NLOAD = 2 * NWL + 2 * NX;
  auto fetch_one = [&](u32x4_t (&wn)[2 * NWL], int fst, int fbuf, int idx) {
    if (idx < 2 * NWL) {
      const int p = idx / NWL, li = idx % NWL;
      const int kb = fst * KBS + (li >> 1);
      const unsigned off = kb < KBp[p] ? wlane[p] : OOB;          // k-blocks past the product's range read zeros
      wn[idx] = __builtin_amdgcn_raw_buffer_load_b128(wres[p], off, kb * 1024 + (li & 1) * 512, 2);
    } else {
      const int p = (idx - 2 * NWL) / NX, i = (idx - 2 * NWL) % NX;
      const unsigned dead = fst * KBS < KBp[p] ? 0u : OOB;
      // chunks beyond K re-read valid columns (k clamped to K - 8), which meet zero weights
      unsigned kb = (unsigned)(fst * KBS) * 64u + xchunk[i];
      kb = kb < xklim[p] ? kb : xklim[p];
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xres[p], (DEINFER_LDS_PTR void *)(sg_lds + (fbuf * 2 + p) * SLAB + xm[i] * RPI * XROW), 16,
                                               (xrow[p][i] + kb) | dead, 0, 0, 0);
    }
  };

  f32x16_t acc[2][NB];
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[p][j][e] = 0.f;

  const int b_row = lane & 31;
  // A stage is 2 x 4 steps (product, k-block, half) of NB matrix products; the token operands are read
  // from LDS DEPTH steps ahead of their use into rotating registers, one read after each product
  constexpr int STEPS = 2 * NWL;
  constexpr int DEPTH = NB >= 4 ? 2 : NB == 2 ? 3 : 6;
  auto read_b = [&](int buf, int step, int j) -> u32x4_t {
    const int p = step / NWL, s = step % NWL;          // s = 2 * k-block + half: 16-byte slot 2 * s + lane / 32
    const int slot = (s * 2 + (lane >> 5)) ^ swz(b_row);
    return *reinterpret_cast<const u32x4_t *>(sg_lds + (buf * 2 + p) * SLAB + (32 * j + b_row) * XROW + slot * 16);
  };
  auto compute = [&](const u32x4_t (&w)[2 * NWL], int buf, u32x4_t (&wn)[2 * NWL], int fst, int fbuf) {
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
        acc[step / NWL][j] = mfma32<DT>(w[step], b[step % (DEPTH + 1)][j], acc[step / NWL][j]);
        __builtin_amdgcn_sched_barrier(0);
        if (step + DEPTH < STEPS) b[(step + DEPTH) % (DEPTH + 1)][j] = read_b(buf, step + DEPTH, j);
        const int pos = step * NB + j;
#pragma unroll
        for (int idx = pos * NLOAD / NPOS; idx < (pos + 1) * NLOAD / NPOS; ++idx) fetch_one(wn, fst, fbuf, idx);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Stage s uses register set / slab pair s % 4.  Every stage issues exactly NLOAD loads (those past
  // the k-range read zeros through an out-of-range offset and cost no traffic), so "all but the
  // loads of the next two stages have arrived" is one constant wait.
  static_assert((SG_SLABS - 1) * NLOAD < 64, "the load counter has 6 bits");
  if (n_stages > 0) {
    u32x4_t w0[2 * NWL], w1[2 * NWL], w2[2 * NWL], w3[2 * NWL];
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w0, 0, 0, idx);
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w1, 1, 1, idx);
#pragma unroll
    for (int idx = 0; idx < NLOAD; ++idx) fetch_one(w2, 2, 2, idx);
    auto stage = [&](const u32x4_t (&w)[2 * NWL], u32x4_t (&wn)[2 * NWL], int st, int slab) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((SG_SLABS - 2) * NLOAD) : "memory");
      __builtin_amdgcn_s_barrier();                     // stage st has arrived everywhere; nobody reads slab pair (st - 1) % 4 any more
      asm volatile("" ::: "memory");
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
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // drain the out-of-range tail loads
  }

  // ---- h = silu(gate) * up: element 4 q + e of block j is feature 8 q + 4 (l / 32) + e, token 32 j + l % 32
  const int col0 = fblk * 32 + 4 * (lane >> 5);
  uint16_t *o = P.out + (long long)(lane & 31) * P.ldo;
  const bool vec = (reinterpret_cast<uintptr_t>(P.out) & 7u) == 0 && (P.ldo & 3) == 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int col = col0 + 8 * q;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      if (32 * j + (lane & 31) >= P.T) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = silu_f32(acc[0][j][4 * q + e]) * acc[1][j][4 * q + e];
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
