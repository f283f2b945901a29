// Compute-bound ("prefill", T > 128 tokens) kernel for PACKED bf16 factor pairs.
//
// Both stages of y = (x U) V (Sec. 4.1) are the same "NT" GEMM  out[T x F] = act[T x K] . W^T
// with the weights W[F x K] in packed MFMA-fragment order:
//   stage 1  act = x,  W = [U_a | U_b | U_c]^T (concatenated feature axis), out = t (bf16, one
//            nearest-even rounding, row-major so that it is stage 2's activation operand);
//   stage 2  act = t,  W = V^T of one pair, out = y; for the GLU call two products (gate, up)
//            are accumulated side by side and combined by the SiLU-GLU epilogue in fp32.
// t makes one round trip through HBM / Infinity Cache (<= 75 MB, a few percent of the MFMA
// time); a 256-row t tile does not fit the 160 KB LDS at these ranks.
//
// Tiling: 256 threads = 4 wavefronts (2 x 2), one per SIMD, workgroup tile 256 tokens x
// (32 * MF) features x 64 k; each wavefront owns 128 tokens x (16 * MF) features:
// MF x 8 accumulator fragments of the 16x16x32 bf16 MFMA (features = MFMA rows, tokens =
// MFMA columns, so a lane ends up with 4 consecutive features of one token).  MF = 8 for a
// single product (256 accumulator registers), MF = 4 for the GLU pair (2 x 128).
// Both operands go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
// 1 KiB contiguous in LDS per wavefront instruction, no staging registers): weight fragments
// are already contiguous 1 KiB pieces; an activation tile is kept as 128-byte token rows whose
// eight 16-byte slots are XOR-swizzled with (row >> 1) & 7, applied on the global side of the
// load (lane -> slot is fixed, lane -> k-chunk is permuted), which makes the operand reads
// (16 rows x 16 bytes per quarter-wave) conflict free without padding.
// LDS is double buffered: the loads of k-step s + 1 are in flight while step s is multiplied;
// one barrier per k-step.
#pragma once
#include "common.h"

namespace deinfer {

#if defined(__HIP_DEVICE_COMPILE__)
#define DEINFER_GLOBAL __attribute__((address_space(1)))
#define DEINFER_LOCAL __attribute__((address_space(3)))
#else
#define DEINFER_GLOBAL
#define DEINFER_LOCAL
#endif

constexpr int PF_THREADS = 256;
constexpr int PF_BT = 256;                 // tokens per workgroup tile
constexpr int PF_BK = 64;                  // k per step (two 32-wide k-blocks)
constexpr int PF_XPITCH = PF_BK * 2;       // bytes per token row of the activation tile in LDS

struct PfSeg {             // a run of 16-feature tiles that belongs to one factor
  const uint4 *frags;      // its packed fragments [tiles][KB][64]
  uint16_t *out;           // output rows of this segment (bf16, row-major)
  long long ldo;
  int tile0;               // first tile of the segment on the concatenated feature axis
  int width;               // valid output columns of the segment
};

struct PfProblem {         // one product  act[T x K] . W^T
  const uint16_t *act;     // row-major bf16
  long long lda;
  int K;                   // valid k (columns of act)
  int KB;                  // 32-wide k-blocks of the packed weights (zero padded)
  int n_seg;
  PfSeg seg[3];
  int n_ftiles;            // 16-feature tiles on the (concatenated) feature axis
};

struct PfParams {
  int T;
  int n_tblocks;           // ceil(T / 256)
  PfProblem prob[2];       // [1] only for the GLU call (same feature axis, output through prob[0])
};

template <int MF>
struct PfShared {
  uint4 w[2][2 * MF][2][64];                       // [buffer][feature tile][k-block][lane]
  unsigned char x[2][PF_BT * PF_XPITCH];           // [buffer][token row * pitch]
};

template <int MF, bool DUAL>
__global__ __launch_bounds__(PF_THREADS) void prefill_kernel(const PfParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  PfShared<MF> &S = *reinterpret_cast<PfShared<MF> *>(smem_raw);
  constexpr int BF_TILES = 2 * MF;                 // 16-feature tiles per workgroup
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave & 1, wt = wave >> 1;         // wavefront position: features x tokens
  const int lrow = lane & 15, lkg = lane >> 4;

  // consecutive workgroups share a feature block and differ in the token block: the token
  // blocks of one feature block run at the same time, spread over the XCDs, so each L2
  // streams those weights once
  const int tb = blockIdx.x % P.n_tblocks;
  const int fb = blockIdx.x / P.n_tblocks;
  const int tok0 = tb * PF_BT;

  f32x4_t acc[DUAL ? 2 : 1][MF][8];
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[p][i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
    const PfProblem &Q = P.prob[p];
    // ---- load assignment (every instruction moves 1 KiB: lane l -> LDS base + 16 l).
    // Buffer addressing: a scalar resource descriptor, a scalar byte offset for the k position
    // and one 32-bit per-lane offset, which leaves the registers to the accumulators; reads
    // beyond a descriptor's size (token rows >= T, feature tiles past the last one) return
    // zeros instead of faulting.  (Host guarantees every tensor here is below 2^31 bytes.)
    constexpr int WT = BF_TILES / 4;       // feature tiles fetched per wavefront, x 2 k-blocks
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    __amdgpu_buffer_rsrc_t wres[WT];
    unsigned wtile_off[WT];
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      const int gt = fb * BF_TILES + uwave * WT + i;
      int s = 0;
      if (Q.n_seg > 1 && gt >= Q.seg[1].tile0) s = 1;
      if (Q.n_seg > 2 && gt >= Q.seg[2].tile0) s = 2;
      const int seg_end = s + 1 < Q.n_seg ? Q.seg[s + 1].tile0 : Q.n_ftiles;
      wres[i] = __builtin_amdgcn_make_buffer_rsrc((void *)Q.seg[s].frags, 0,
                                                  (int)((unsigned)(seg_end - Q.seg[s].tile0) * (unsigned)Q.KB * 1024u), 0x00020000);
      wtile_off[i] = (unsigned)(gt - Q.seg[s].tile0) * (unsigned)Q.KB * 1024u;
    }
    const unsigned wlane = lane * 16;
    // activations: instruction i of wavefront w covers tile rows 8 (4 i + w) .. + 7; lane l holds
    // slot l % 8 of row l / 8 and fetches k-chunk slot ^ ((row >> 1) & 7).  With row = 8 m + l / 8,
    // (row >> 1) & 7 is ((l >> 4) & 3) | ((m & 1) << 2), and m & 1 = w & 1.
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)((unsigned)P.T * (unsigned)(Q.lda * 2)), 0x00020000);
    const int chunk = (lane & 7) ^ ((lane >> 4) & 3) ^ ((wave & 1) << 2);
    unsigned xoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      xoff[i] = (unsigned)(tok0 + 8 * (4 * i + wave) + (lane >> 3)) * (unsigned)(Q.lda * 2) + (unsigned)(chunk * 16);
    const int n_steps = (Q.KB + 1) >> 1;

    auto fetch = [&](int step, int buf) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          // a k-block past the end (odd KB) is asked for beyond the descriptor: it arrives as zeros
          const unsigned so = step * 2 + kk < Q.KB ? wtile_off[i] + (unsigned)(step * 2 + kk) * 1024u : 0xffffff00u;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(wres[i], (DEINFER_LOCAL void *)&S.w[buf][uwave * WT + i][kk][0], 16,
                                                   wlane, so, 0, 0);
        }
      if ((step + 1) * PF_BK <= Q.K) {            // uniform: the whole 64-wide slab is inside K
#pragma unroll
        for (int i = 0; i < 8; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LOCAL void *)&S.x[buf][8 * (4 * i + uwave) * PF_XPITCH], 16,
                                                   xoff[i], (unsigned)step * (PF_BK * 2), 0, 0);
      } else {
        // slab reaches beyond K: those chunks re-read valid columns, which meet zero weights
        int k = step * PF_BK + chunk * 8;
        k = k < Q.K - 8 ? k : Q.K - 8;
        const unsigned fix = (unsigned)(k * 2) - (unsigned)(chunk * 16);
#pragma unroll
        for (int i = 0; i < 8; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LOCAL void *)&S.x[buf][8 * (4 * i + uwave) * PF_XPITCH], 16,
                                                   xoff[i] + fix, 0, 0, 0);
      }
    };

    auto read_a = [&](int buf, int kk, int i) -> u32x4_t {
      return *reinterpret_cast<const u32x4_t *>(&S.w[buf][wf * MF + i][kk][lane]);
    };
    auto read_b = [&](int buf, int kk, int j) -> u32x4_t {
      const int r = wt * 128 + j * 16 + lrow;
      const int slot = (kk * 4 + lkg) ^ ((r >> 1) & 7);
      return *reinterpret_cast<const u32x4_t *>(&S.x[buf][r * PF_XPITCH + slot * 16]);
    };

    // One barrier per k-step: when it is passed, step s has landed in buffer s % 2 and nobody
    // reads buffer (s + 1) % 2 any more, so step s + 1 is requested into it right away and has
    // the whole step to arrive.  Inside a step the LDS operand reads run ahead of the MFMAs in
    // registers: the token fragment one product group ahead, and the feature fragments of the
    // second k-block during the last product groups of the first.
    fetch(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int step = 0; step < n_steps; ++step) {
      const int buf = step & 1;
      if (step + 1 < n_steps) fetch(step + 1, buf ^ 1);
      u32x4_t a0[MF], a1[MF], bc, bn;
#pragma unroll
      for (int i = 0; i < MF; ++i) a0[i] = read_a(buf, 0, i);
      bc = read_b(buf, 0, 0);
#ifdef PF_SCHED
      __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        bn = j < 7 ? read_b(buf, 0, j + 1) : read_b(buf, 1, 0);
        if (j >= 8 - MF / 2) {
          const int i0 = 2 * (j - (8 - MF / 2));
          a1[i0] = read_a(buf, 1, i0);
          a1[i0 + 1] = read_a(buf, 1, i0 + 1);
        }
#pragma unroll
        for (int i = 0; i < MF; ++i)
          acc[p][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0[i]), as_bf16x8(bc), acc[p][i][j], 0, 0, 0);
        bc = bn;
#ifdef PF_SCHED
        __builtin_amdgcn_sched_barrier(0);      // keep the hand-written read-ahead distance
#endif
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (j < 7) bn = read_b(buf, 1, j + 1);
#pragma unroll
        for (int i = 0; i < MF; ++i)
          acc[p][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a1[i]), as_bf16x8(bc), acc[p][i][j], 0, 0, 0);
        bc = bn;
#ifdef PF_SCHED
        __builtin_amdgcn_sched_barrier(0);
#endif
      }
      // the loads of the next step have had the whole multiply to land
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
  }

  // ---- epilogue: a lane holds features f .. f + 3 of token (lane % 16) for every fragment
  const PfProblem &Q = P.prob[0];
#pragma unroll
  for (int i = 0; i < MF; ++i) {
    const int gt = fb * BF_TILES + wf * MF + i;
    if (gt >= Q.n_ftiles) continue;
    int s = 0;
    if (Q.n_seg > 1 && gt >= Q.seg[1].tile0) s = 1;
    if (Q.n_seg > 2 && gt >= Q.seg[2].tile0) s = 2;
    const PfSeg &sg = Q.seg[s];
    const int col = (gt - sg.tile0) * 16 + lkg * 4;
    if (col >= sg.width) continue;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = tok0 + wt * 128 + j * 16 + lrow;
      if (tok >= P.T) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = acc[0][i][j][e];
        if (DUAL) v[e] = silu_f32(v[e]) * acc[DUAL ? 1 : 0][i][j][e];
      }
      uint16_t *dst = sg.out + (long long)tok * sg.ldo + col;
      if (col + 3 < sg.width && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
        uint2 pk;
        pk.x = pack_bf16x2(v[0], v[1]);
        pk.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2 *>(dst) = pk;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (col + e < sg.width) dst[e] = f32_to_bf16(v[e]);
      }
      __builtin_amdgcn_sched_barrier(0);    // one fragment at a time: keeps the epilogue's register need small
    }
  }
#else
  (void)P;
#endif
}

}  // namespace deinfer
