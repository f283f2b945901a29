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
    // ---- per-lane load assignment (every instruction moves 1 KiB: lane l -> LDS base + 16 l)
    // weights: wavefront w fetches feature tiles [w * WT, +WT) x 2 k-blocks
    constexpr int WT = BF_TILES / 4;
    const uint4 *wsrc[WT];
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      int gt = fb * BF_TILES + wave * WT + i;
      gt = gt < Q.n_ftiles ? gt : Q.n_ftiles - 1;
      int s = 0;
      if (Q.n_seg > 1 && gt >= Q.seg[1].tile0) s = 1;
      if (Q.n_seg > 2 && gt >= Q.seg[2].tile0) s = 2;
      wsrc[i] = Q.seg[s].frags + (long long)(gt - Q.seg[s].tile0) * Q.KB * 64 + lane;
    }
    // activations: instruction i of wavefront w covers tile rows 8 (4 i + w) .. + 7; lane l holds
    // slot l % 8 of row l / 8 and fetches k-chunk slot ^ ((row >> 1) & 7)
    const uint16_t *xsrc[8];
    int xchunk[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 8 * (4 * i + wave) + (lane >> 3);
      int row = tok0 + r;
      row = row < P.T ? row : P.T - 1;
      xsrc[i] = Q.act + (long long)row * Q.lda;
      xchunk[i] = (lane & 7) ^ ((r >> 1) & 7);
    }
    const int n_steps = (Q.KB + 1) >> 1;

    auto fetch = [&](int step, int buf) {
      const int kb0 = step * 2;
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const int kb = kb0 + kk < Q.KB ? kb0 + kk : Q.KB - 1;   // odd tail: duplicate, skipped below
          __builtin_amdgcn_global_load_lds((const DEINFER_GLOBAL void *)(wsrc[i] + (long long)kb * 64),
                                           (DEINFER_LOCAL void *)&S.w[buf][wave * WT + i][kk][0], 16, 0, 0);
        }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int k = step * PF_BK + xchunk[i] * 8;
        k = k < Q.K - 8 ? k : Q.K - 8;     // beyond K: re-read valid columns, they meet zero weights
        __builtin_amdgcn_global_load_lds((const DEINFER_GLOBAL void *)(xsrc[i] + k),
                                         (DEINFER_LOCAL void *)&S.x[buf][8 * (4 * i + wave) * PF_XPITCH], 16, 0, 0);
      }
    };

    fetch(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int step = 0; step < n_steps; ++step) {
      const int buf = step & 1;
      if (step + 1 < n_steps) fetch(step + 1, buf ^ 1);
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        if (step * 2 + kk < Q.KB) {        // uniform: odd number of k-blocks
          u32x4_t a[MF], b[8];
#pragma unroll
          for (int i = 0; i < MF; ++i)
            a[i] = *reinterpret_cast<const u32x4_t *>(&S.w[buf][wf * MF + i][kk][lane]);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int r = wt * 128 + j * 16 + lrow;
            const int slot = (kk * 4 + lkg) ^ ((r >> 1) & 7);
            b[j] = *reinterpret_cast<const u32x4_t *>(&S.x[buf][r * PF_XPITCH + slot * 16]);
          }
#pragma unroll
          for (int i = 0; i < MF; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
              acc[p][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a[i]), as_bf16x8(b[j]), acc[p][i][j], 0, 0, 0);
        }
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
    }
  }
}

}  // namespace deinfer
