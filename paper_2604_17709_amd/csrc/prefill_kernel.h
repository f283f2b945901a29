// Compute-bound ("prefill", T > 128 tokens) kernel for PACKED bf16 factor pairs.
//
// Both stages of y = (x U) V (Sec. 4.1) are the same "NT" GEMM  out[T x F] = act[T x K] . W^T
// with the weights W[F x K] in packed MFMA-fragment order:
//   stage 1  act = x,  W = [U_a | U_b | U_c]^T (concatenated feature axis), out = t (bf16, one
//            nearest-even rounding, row-major so that it is stage 2's activation operand);
//   stage 2  act = t,  W = V^T of one pair, out = y.  The GLU call computes both products of a
//            tile in one workgroup, one after the other on the same accumulators: the gate product,
//            then silu of it rounded to the storage type into 128 registers that the main loop
//            leaves free, then the up product, whose epilogue multiplies the two: the full-width
//            gate and up results never leave the registers (a side-by-side accumulation, half the
//            tile per product, would need 1.5 x the LDS traffic per flop).
// t makes one round trip through HBM / Infinity Cache (<= 75 MB, a few percent of the MFMA
// time); a 256-row t tile does not fit the 160 KB LDS at these ranks.
//
// Tiling: 256 threads = 4 wavefronts (2 x 2), one per SIMD, workgroup tile 256 tokens x
// (32 * MF) features; each wavefront owns 128 tokens x (16 * MF) features as (MF / 2) x 4
// accumulator blocks of the 32x32x16 bf16 MFMA (features = MFMA rows, tokens = MFMA columns).
// MF = 8 uses all 256 accumulator registers.  (The 16x16x32 form of the instruction issued at
// only about 60 % of the rate of the 32x32x16 form in a bare issue-rate measurement on this
// device, which is why the wider form is used although the packed fragments are 16 features
// tall: a 32-feature operand is gathered from two neighbouring fragments by LDS addressing.)
// Both operands go from global memory straight into LDS (buffer loads with the LDS modifier,
// 16 bytes per lane, 1 KiB contiguous in LDS per wavefront instruction, no staging registers):
// weight fragments are already contiguous 1 KiB pieces; an activation tile is kept as 64-byte
// token rows whose four 16-byte slots are XOR-swizzled with (row >> 2) & 3, applied on the
// global side of the load (lane -> slot is fixed, lane -> k-chunk is permuted), which makes the
// operand reads (16 rows x 16 bytes per quarter-wave) conflict free without padding.
// Pipeline: one stage = one 32-wide k-block; four LDS stage buffers; the loads of stage s + 3
// are requested while stage s is multiplied (about 2.5 stages = 2500 MFMA cycles of cover for
// L2 misses); one barrier per stage, placed in the middle of the stage's products so that the
// feature fragments of stage s + 1 can be read from LDS during the second half of stage s.
#pragma once
#include <type_traits>
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
constexpr int PF_BK = 32;                  // k per pipeline stage (one k-block)
constexpr int PF_STAGES = 4;               // LDS stage buffers of the 256-token tile
constexpr int PF_STAGES_TB2 = 6;           // ... of the 128 x 256 tile (half the products per stage: a deeper queue for the same cover)
constexpr int PF_STAGES_MF4 = 6;           // ... of the 128 x 128 tile (four stages, which would let two workgroups share a
                                           // compute unit, measured 3-7 % slower on launches of 32-128 tiles; eight the same as six)
constexpr int pf_stages(int tb, int mf = 8) { return tb == 4 ? PF_STAGES : mf == 8 ? PF_STAGES_TB2 : PF_STAGES_MF4; }

// s_waitcnt vmcnt(k * LPS + EXTRA) for a run-time k in [C, CMAX] (the instruction takes an immediate)
template <int C, int CMAX, int LPS, int EXTRA>
struct PfVmWait {
  static __device__ __forceinline__ void run(int k) {
    if (k == C) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C * LPS + EXTRA) : "memory");
    else PfVmWait<C + 1, CMAX, LPS, EXTRA>::run(k);
  }
};
template <int CMAX, int LPS, int EXTRA>
struct PfVmWait<CMAX, CMAX, LPS, EXTRA> {
  static __device__ __forceinline__ void run(int) { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CMAX * LPS + EXTRA) : "memory"); }
};
constexpr int PF_XPITCH = PF_BK * 2;       // bytes per token row of the activation tile in LDS

struct PfSeg {             // a run of 16-feature tiles that belongs to one factor
  const uint4 *frags;      // its packed fragments [tiles][KB][64]
  int tile0;               // first tile of the segment on the concatenated feature axis
};

struct PfProblem {         // one product  act[T x K] . W^T
  const uint16_t *act;     // row-major bf16
  long long lda;
  int K;                   // valid k (columns of act)
  int KB;                  // 32-wide k-blocks of the packed weights (zero padded)
  int n_seg;
  PfSeg seg[3];
  int n_ftiles;            // 16-feature tiles on the (concatenated) feature axis
  uint16_t *out;           // output [T x width] bf16 row-major: feature tile g lands at columns 16 g ..
  long long ldo;
  int width;               // valid output columns
  const uint16_t *bias;    // POST kernels only: out = act(product + bias[column]); may be null
  int post_act;            // see act_f32
  const float *rope;       // ROPE kernels only: [T][128] cos | sin of the rotary angles (heads of 128 features)
};

struct PfParams {
  int T;
  int n_tblocks;           // ceil(T / 256)
  // Up to three independent products in one launch (the upward projections of a q/k/v call: a
  // narrow one alone would leave most of the device idle); product i owns the feature blocks
  // [fb0[i], fb0[i + 1]) of the grid.
  int n_prob;
  int fb0[3];
  PfProblem prob[3];
  // SPLIT kernels only (few tiles, long k: the k range is cut into parts, one workgroup per part)
  int n_fblocks;           // feature blocks of 256; grid = n_tblocks * n_fblocks * n_parts
  int kb_per_part;         // k-blocks per part
  float *part;             // [n_parts][n_tblocks * 256][n_fblocks * 256] fp32 partial products
  long long part_stride;   // elements between parts
  // prefill_mixed_kernel only
  int n_big;               // workgroups with 256 x 256 tiles (they come first)
  int n_tblocks2;          // ceil(T / 128): token blocks of the 128 x 256 tiles
  int fb_shift2;           // first feature block (of 256 features) of the 128 x 256 tiles
};

template <int MF, int TB = 4>
struct PfShared {
  uint4 w[pf_stages(TB, MF)][2 * MF][64];                   // [stage][feature tile][lane]
  unsigned char x[pf_stages(TB, MF)][64 * TB * PF_XPITCH];  // [stage][token row * 64 bytes], slots swizzled
};

// GLU = true: two products per tile, P.prob[0] (gate) and P.prob[1] (up, same feature tiles and output):
// out = silu(gate product) * up product.
// POST = PF_POST_BIAS_ACT: bias and activation of the non-GLU MLP sub-layer on the fp32 accumulators;
// PF_POST_TAIL: the activation rows' valid columns K may be no multiple of 8 (the caller's rank-space rows
// of an upward projection alone): what the last chunk holds beyond column K - 1 is set to zero in LDS.
// SPLIT = true: this workgroup multiplies only its part of the k range and stores the fp32
// accumulators to a partial buffer (the sum and the epilogue are a second, small kernel's).
// DT = storage type of weights, activations and outputs (DT_BF16 or DT_F16).
// ROPE = true: rotary embedding of the output (heads of 128 features = one wavefront's features:
// feature i of a head pairs with feature i + 64 of the same token, both in this wavefront's LDS
// tile), on the rounded products, cos / sin from a table; the result is rounded once more.
// TB = 32-token blocks per wavefront: 4 (workgroup tile of 256 tokens) or 2 (128 tokens: twice the
// workgroups, for launches whose 256-token tiles are fewer than the compute units; its loop keeps a
// whole k-step of operands ahead instead of the hand-placed reads of the TB = 4 loop).
// The body of a workgroup: bid = its index among the workgroups of this tile shape, n_tblocks = token
// blocks of this tile shape, fb_shift = first feature block of this tile shape (0 unless the launch
// mixes two shapes, see prefill_mixed_kernel).
constexpr int PF_POST_NONE = 0, PF_POST_BIAS_ACT = 1, PF_POST_TAIL = 2;

template <int DT, int MF, bool GLU, int POSTK, bool SPLIT, bool ROPE, int TB>
__device__ __forceinline__ void prefill_body(const PfParams &P, const int bid, const int n_tblocks, const int fb_shift) {
  constexpr bool POST = POSTK == PF_POST_BIAS_ACT, TAIL = POSTK == PF_POST_TAIL;
  static_assert(!(ROPE && (GLU || POST || SPLIT)), "the rotary epilogue goes with a plain product");
  static_assert(!(TAIL && SPLIT), "only a second stage reads caller rows");
  static_assert(TB == 4 || (TB == 2 && !SPLIT), "token blocks per wavefront");
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  constexpr int WTOK = 32 * TB;                    // tokens per wavefront
  constexpr int BT = 2 * WTOK;                     // tokens per workgroup tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  PfShared<MF, TB> &S = *reinterpret_cast<PfShared<MF, TB> *>(smem_raw);
  constexpr int NST = pf_stages(TB, MF);           // LDS stage buffers; loads run NST - 1 stages ahead
  constexpr int BF_TILES = 2 * MF;                 // 16-feature tiles per workgroup
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave & 1, wt = wave >> 1;         // wavefront position: features x tokens

  // consecutive workgroups share a feature block and differ in the token block: the token
  // blocks of one feature block run at the same time, spread over the XCDs, so each L2
  // streams those weights once
  const int tb = bid % n_tblocks;
  const int fb_all = bid / n_tblocks + fb_shift;
  int fb = SPLIT ? fb_all % P.n_fblocks : fb_all;
  int pi = 0;                                                   // which product (uniform)
  if (!SPLIT && P.n_prob > 1 && fb >= P.fb0[1]) pi = 1;
  if (!SPLIT && P.n_prob > 2 && fb >= P.fb0[2]) pi = 2;
  fb -= P.fb0[pi];
  const int kpart = SPLIT ? fb_all / P.n_fblocks : 0;
  const int kb0 = SPLIT ? kpart * P.kb_per_part : 0;          // first k-block of this workgroup
  const int tok0 = tb * BT;

  constexpr int MB = MF / 2;                       // 32-feature blocks per wavefront
  static_assert(MF == 8 || (MF == 4 && TB == 2 && !ROPE), "the hand-placed loop of the 256-token tile is written for four 32-feature blocks per wavefront");
  f32x16_t acc[MB][TB];                            // [feature block][32-token block]
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // GLU: silu(gate product), rounded once to the storage type, kept in registers (as pairs) while the
  // up product is accumulated: element [i][j][g] holds the four values of accumulator elements 4 g .. 4 g + 3
  uint2 gpk[GLU ? MB : 1][GLU ? TB : 1][4];
  // One product of this workgroup's tile: acc += act . W^T over the whole k range of Q.  between() runs
  // once the first pipeline stages have been requested and before they are waited for.
  auto product = [&](const PfProblem &Q, auto &&between) {
    // ---- load assignment (every instruction moves 1 KiB: lane l -> LDS base + 16 l).
    // Buffer addressing: a scalar resource descriptor, a scalar byte offset for the k position
    // and one 32-bit per-lane offset, which leaves the registers to the accumulators; reads
    // beyond a descriptor's size (token rows >= T, feature tiles past the last one) return
    // zeros instead of faulting.  (Host guarantees every tensor here is below 2^31 bytes.)
    constexpr int WT = BF_TILES / 4;       // feature tiles fetched per wavefront and stage
    constexpr int LPS = WT + TB;           // load instructions per wavefront and stage
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    __amdgpu_buffer_rsrc_t wres[WT];
    unsigned wtile_off[WT];
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      const int gt = fb * BF_TILES + uwave * WT + i;
      int sgi = 0;
      if (Q.n_seg > 1 && gt >= Q.seg[1].tile0) sgi = 1;
      if (Q.n_seg > 2 && gt >= Q.seg[2].tile0) sgi = 2;
      const int seg_end = sgi + 1 < Q.n_seg ? Q.seg[sgi + 1].tile0 : Q.n_ftiles;
      // a feature tile past the last one gets an empty descriptor: every read of it returns zeros
      const bool live = gt < Q.n_ftiles;
      wres[i] = __builtin_amdgcn_make_buffer_rsrc((void *)Q.seg[sgi].frags, 0,
                                                  live ? (int)((unsigned)(seg_end - Q.seg[sgi].tile0) * (unsigned)Q.KB * 1024u) : 0, 0x00020000);
      wtile_off[i] = live ? (unsigned)(gt - Q.seg[sgi].tile0) * (unsigned)Q.KB * 1024u : 0u;
    }
    const unsigned wlane = lane * 16;
    // activations: instruction i of wavefront w covers tile rows 16 (4 i + w) .. + 15; lane l holds
    // slot l % 4 of row l / 4 and fetches k-chunk slot ^ ((row >> 2) & 3) = (l & 3) ^ ((l >> 4) & 3)
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)((unsigned)P.T * (unsigned)(Q.lda * 2)), 0x00020000);
    const int chunk = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned xrow[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) xrow[i] = (unsigned)(tok0 + 16 * (4 * i + wave) + (lane >> 2)) * (unsigned)(Q.lda * 2);
    const int n_stages = SPLIT ? (Q.KB - kb0 < P.kb_per_part ? Q.KB - kb0 : P.kb_per_part) : Q.KB;

    // one load instruction (index 0 .. LPS - 1) of stage st: weight tiles first, then activation rows.
    // Activation chunks beyond K re-read a chunk of valid columns (the last one; PF_POST_TAIL: the first one),
    // which meets zero weights.
    const unsigned xchunk = (unsigned)(chunk * 16);
    const unsigned xkend = (unsigned)(((Q.K + 7) >> 3) * 16);    // bytes of a row up to the end of the chunk that holds column K - 1
    const unsigned xklim = (unsigned)(Q.K * 2 - 16);             // (K a multiple of 8: the last chunk)
    // Valid columns K that are no multiple of 8 (the caller's rank-space rows of an upward projection alone):
    // the stage whose tile holds the chunk with column K - 1; once it has landed, the elements of that chunk
    // beyond K - 1 are set to zero (lds_zero_chunk_tail in common.h).  -1: nothing to do (every other call).
    const int krem = Q.K & 7;
    const int st_fix = (TAIL && krem != 0) ? (Q.K >> 5) - kb0 : -1;
    auto fix_tail = [&](int buf) {
      int row = threadIdx.x;
      asm volatile("" : "+v"(row));
      if (row < 64 * TB) lds_zero_chunk_tail(&S.x[buf][row * PF_XPITCH + ((((Q.K >> 3) & 3) ^ ((row >> 2) & 3)) * 16)], krem);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };
    auto fetch_part = [&](int st, int idx) {
      const int buf = st % NST;
      if (idx < WT) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wres[idx], (DEINFER_LOCAL void *)&S.w[buf][uwave * WT + idx][0], 16,
                                                 wlane, wtile_off[idx] + (unsigned)(st + kb0) * 1024u, 0, 0);
      } else {
        const int i = idx - WT;
        unsigned kb = (unsigned)(st + kb0) * (PF_BK * 2) + xchunk;
        kb = TAIL ? (kb < xkend ? kb : 0u) : (kb < xklim ? kb : xklim);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LOCAL void *)&S.x[buf][16 * (4 * i + uwave) * PF_XPITCH], 16,
                                                 xrow[i] + kb, 0, 0, 0);
      }
    };
    // Operand reads for the 32x32x16 product: lane l works on row (feature or token) l % 32 and on
    // the 8 consecutive k of group 2 s + l / 32 of the stage's four k-groups, s = 0, 1 being the
    // two k-steps of a stage.  In a packed 16-feature fragment that k-group of feature f % 16
    // sits at lane position (f % 16) + 16 * group.
    const int a_off = ((lane >> 4) & 1) * 64 + (lane & 15) + 16 * (lane >> 5);     // in uint4 units
    const int b_row = wt * WTOK + (lane & 31);
    const int b_swz = ((lane & 31) >> 2) & 3;
    auto read_a = [&](int buf, int ib, int ks) -> u32x4_t {
      return *reinterpret_cast<const u32x4_t *>(&S.w[buf][wf * MF + 2 * ib][0] + a_off + 32 * ks);
    };
    auto read_b = [&](int buf, int jb, int ks) -> u32x4_t {
      const int slot = (2 * ks + (lane >> 5)) ^ b_swz;
      return *reinterpret_cast<const u32x4_t *>(&S.x[buf][(b_row + 32 * jb) * PF_XPITCH + slot * 16]);
    };
    constexpr int H1 = LPS / 2;            // loads 0 .. H1 - 1 of stage s + 3 go out during k-step 1 of stage s,
                                           // loads H1 .. LPS - 1 during k-step 0 of stage s + 1: at most one
                                           // load after each group of products, so their issue never holds
                                           // the matrix pipeline up
    static_assert(LPS - H1 <= 4 && H1 <= 4, "one load per token block and k-step");
    if constexpr (TB == 4) {
#pragma unroll
      for (int i = 0; i < LPS; ++i) fetch_part(0, i);
      if (n_stages > 1) {
#pragma unroll
        for (int i = 0; i < LPS; ++i) fetch_part(1, i);
      }
      if (n_stages > 2) {
#pragma unroll
        for (int i = 0; i < H1; ++i) fetch_part(2, i);
      }
      between();
      if (n_stages > 2) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS + H1) : "memory");
      } else if (n_stages > 1) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    } else {
      // stages 0 .. D - 2 whole and the first half of stage D - 1, then wait for stage 0
      constexpr int D = NST - 1;
      static_assert((D - 2) * LPS + H1 < 64, "the load counter has 6 bits");
#pragma unroll
      for (int sg = 0; sg < D - 1; ++sg)
        if (sg < n_stages) {
#pragma unroll
          for (int i = 0; i < LPS; ++i) fetch_part(sg, i);
        }
      if (D - 1 < n_stages) {
#pragma unroll
        for (int i = 0; i < H1; ++i) fetch_part(D - 1, i);
      }
      between();
      // outstanding at most: the stages after stage 0 (and the half stage D - 1)
      if (D - 1 < n_stages) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS + H1) : "memory");
      else PfVmWait<0, D - 2, LPS, 0>::run(n_stages - 1);
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();          // stage 0 has landed everywhere
    asm volatile("" ::: "memory");
    if constexpr (TAIL) {
      if (st_fix == 0) fix_tail(0);
    }
    // Operand reads run two groups of products ahead of their use (a group = the MB products that
    // share one token operand, about 130 cycles): with the four wavefronts reading in step and the
    // incoming tiles being written, one group of cover left the products waiting for LDS.
    u32x4_t a0[MB], a1[MB], b[4];
#pragma unroll
    for (int i = 0; i < MB; ++i) a0[i] = read_a(0, i, 0);
    b[0] = read_b(0, 0, 0);
    b[1] = read_b(0, 1, 0);
    // (TB = 2: b[0..1] are the token operands of k-step 0, b[2..3] those of k-step 1)
    // one stage; F2: the second half of stage st + 2 is still to be requested, F3: stage st + 3 exists
    auto stage4 = [&](int st, auto f2, auto f3) {
      constexpr bool F2 = decltype(f2)::value, F3 = decltype(f3)::value;
      const int buf = st & (PF_STAGES - 1);
      const int nbuf = (st + 1) & (PF_STAGES - 1);
      // token operand of group g of this stage (g = 4 * k-step + token block); 8, 9 = next stage's 0, 1
      auto read_bg = [&](int g) -> u32x4_t { return g < 8 ? read_b(buf, g & 3, g >> 2) : read_b(nbuf, g - 8, 0); };
      // ---- k-step 0 of the stage; the feature operands of k-step 1 are read along the way.
      // At most one memory instruction follows each product: its issue then hides behind the
      // product's 32 cycles in the matrix pipeline (several in a row after a group held the next
      // product up by about 40 cycles per group).
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          acc[i][j] = mfma32<DT>(a0[i], b[j], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
          if (F2 && i == 0 && H1 + j < LPS) fetch_part(st + 2, H1 + j);
          if (i == 1 || MB == 1) b[(j + 2) & 3] = read_bg(j + 2);
          if (i == 2 && j < 3 && (j == 0 ? 0 : j + 1) < MB) a1[j == 0 ? 0 : j + 1] = read_a(buf, j == 0 ? 0 : j + 1, 1);
          if (i == 3 && j == 0 && MB > 1) a1[1] = read_a(buf, 1, 1);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- stage st + 1 has landed (this wavefront's part), barrier: it has landed everywhere and
      // nobody reads the buffer of stage st - 1 any more, which is where stage st + 3 goes
      if (F2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      // bare barrier: the wait above is the only ordering needed (loads into LDS are complete when
      // the counter says so; the buffer about to be refilled was last read a whole k-step ago);
      // the fence of __syncthreads() would drain every outstanding load instead
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      // (the chunk that holds column K - 1 is in the last stage: only the stages that run without further
      // requests can precede it, so the steady-state loop carries no branch for this)
      if constexpr (TAIL && !F2 && !F3) {
        if (st + 1 == st_fix) fix_tail(nbuf);           // (uniform)
      }
      // ---- k-step 1; the operands of the next stage's k-step 0 are read along the way
      // (after the last stage these read a stage buffer nobody writes any more; the values are unused)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          acc[i][j] = mfma32<DT>(a1[i], b[j], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
          if (F3 && i == 0 && j < H1) fetch_part(st + 3, j);
          if (i == 1 || MB == 1) b[(j + 2) & 3] = read_bg(j + 6);
          // a0 is not in use during k-step 1
          if (i == 2 && j < 3 && (j == 0 ? 0 : j + 1) < MB) a0[j == 0 ? 0 : j + 1] = read_a(nbuf, j == 0 ? 0 : j + 1, 0);
          if (i == 3 && j == 0 && MB > 1) a0[1] = read_a(nbuf, 1, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    // TB = 2: the operands of a whole k-step are read while the previous one is multiplied
    // (MB + TB reads and up to H1 load requests over the MB * TB products of a k-step); loads run
    // D = NST - 1 stages ahead.  STEADY: stage st + D exists (no conditions in the loop body).
    auto stage2 = [&](int st, auto steady) {
      constexpr bool STEADY = decltype(steady)::value;
      constexpr int D = NST - 1;
      const int buf = st % NST;
      const int nbuf = (st + 1) % NST;
      const bool i2 = STEADY || st + D - 1 < n_stages;     // second half of stage st + D - 1 still to request
      const bool i3 = STEADY || st + D < n_stages;         // stage st + D exists
      constexpr int NS = MB * TB;                          // products = slots of a k-step
      static_assert(TB == 4 || (MB + TB <= NS && LPS - H1 <= NS && H1 <= NS), "slots of a k-step");
#pragma unroll
      for (int j = 0; j < TB; ++j) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          const int slot = j * MB + i;
          acc[i][j] = mfma32<DT>(a0[i], b[j], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
          if (slot < MB) a1[slot] = read_a(buf, slot, 1);
          else if (slot - MB < TB) b[2 + slot - MB] = read_b(buf, slot - MB, 1);
          if (slot >= NS - (LPS - H1) && i2) fetch_part(st + D - 1, H1 + slot - (NS - (LPS - H1)));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // stage st + 1 has landed once at most the loads of the stages st + 2 .. st + D - 1 are outstanding
      if (STEADY) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");
      } else {
        int rem = n_stages - (st + 2);
        rem = rem < 0 ? 0 : rem > D - 2 ? D - 2 : rem;
        PfVmWait<0, D - 2, LPS, 0>::run(rem);
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();          // ... everywhere, and nobody reads the buffer of stage st - 1 any more
      asm volatile("" ::: "memory");
      if constexpr (TAIL && !STEADY) {
        if (st + 1 == st_fix) fix_tail(nbuf);
      }
#pragma unroll
      for (int j = 0; j < TB; ++j) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          const int slot = j * MB + i;
          acc[i][j] = mfma32<DT>(a1[i], b[2 + j], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
          if (slot < MB) a0[slot] = read_a(nbuf, slot, 0);
          else if (slot - MB < TB) b[slot - MB] = read_b(nbuf, slot - MB, 0);
          if (slot >= NS - H1 && i3) fetch_part(st + D, slot - (NS - H1));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    {
      const std::true_type yes;
      const std::false_type no;
      int st = 0;
      if constexpr (TB == 4) {
        for (; st + 3 < n_stages; ++st) stage4(st, yes, yes);
        if (st + 2 < n_stages) { stage4(st, yes, no); ++st; }
        for (; st < n_stages; ++st) stage4(st, no, no);
      } else {
        for (; st + NST - 1 < n_stages; ++st) stage2(st, yes);
        for (; st < n_stages; ++st) stage2(st, no);
      }
    }
  };
  if constexpr (GLU) {
    // Both products of the tile in this workgroup (Sec. 4.1: gate and up share x and the output
    // columns): the gate product first; its silu goes into registers while the up product's first
    // stages are on their way; the full-width gate and up results never reach memory.
    product(P.prob[0], [] {});
    __syncthreads();       // every wavefront has read its last gate-product operands: the stage buffers are free
    product(P.prob[1], [&] {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            // (the sums are taken out of the accumulator registers here, by hand: the compiler would
            // move all 256 of them to ordinary registers at the end of the gate product's loop, where
            // they would have to live through the requests above)
            float z[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(z[e]) : "a"(acc[i][j][4 * g + e]));
              acc[i][j][4 * g + e] = 0.f;
            }
            gpk[i][j][g].x = pack2<DT>(silu_f32(z[0]), silu_f32(z[1]));
            gpk[i][j][g].y = pack2<DT>(silu_f32(z[2]), silu_f32(z[3]));
            // (the packed values are made opaque here: otherwise the compiler defers silu to the
            // epilogue and keeps all 256 raw gate sums alive through the second product's loop)
            asm volatile("" : "+v"(gpk[i][j][g].x), "+v"(gpk[i][j][g].y));
          }
    });
  } else {
    product(P.prob[pi], [] {});
  }
  const PfProblem &Q = P.prob[pi];         // (GLU: the gate problem; output buffer and width are the same for both)
  // (lane-derived values are taken afresh so that none has to live through the main loop)
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int lane_e = tid_e & 63, wave_e = tid_e >> 6, wf_e = wave_e & 1, wt_e = wave_e >> 1;
  if constexpr (SPLIT) {
    // element 4 g + e of block (i, j) is feature 32 i + 8 g + 4 (lane / 32) + e, token 32 j + lane % 32:
    // four consecutive features = one 16-byte store; the buffer has whole tiles, no bounds to check
    const long long F = (long long)P.n_fblocks * (32 * MF);
    float *dst = P.part + (long long)kpart * P.part_stride + (long long)(tok0 + wt_e * 128 + (lane_e & 31)) * F +
                 (fb * BF_TILES + wf_e * MF) * 16 + 4 * (lane_e >> 5);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4_t v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *reinterpret_cast<f32x4_t *>(dst + (long long)(32 * j) * F + 32 * i + 8 * g) = v;
        }
    return;
  }
  // accumulators -> bf16 pairs first (registers only): it overlaps the wait for the slowest wavefront.
  // (GLU: not ahead of the barrier: 128 registers of pairs beside the 128 of the gate values would not
  // fit; every pair is formed right before it is written to LDS instead)
  uint2 pk[GLU ? 1 : MB][GLU ? 1 : TB][4];
  if constexpr (!GLU) {
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float b[4] = {0.f, 0.f, 0.f, 0.f};
      if (POST && Q.bias != nullptr) {
        // element 4 g + e of block (i, j) is feature 32 i + 8 g + 4 (lane / 32) + e of this wavefront's 16 MF features
        const int f0 = (fb * BF_TILES + wf_e * MF) * 16 + 32 * i + 8 * g + 4 * (lane_e >> 5);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (f0 + e < Q.width) b[e] = cvt_in<DT>(Q.bias[f0 + e]);
      }
#pragma unroll
      for (int j = 0; j < TB; ++j) {
        float v[4] = {acc[i][j][4 * g + 0], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        if (POST) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = act_f32(v[e] + b[e], Q.post_act);
        }
        pk[GLU ? 0 : i][GLU ? 0 : j][g].x = pack2<DT>(v[0], v[1]);
        pk[GLU ? 0 : i][GLU ? 0 : j][g].y = pack2<DT>(v[2], v[3]);
      }
    }
  }

  // ---- epilogue: through LDS (free once the barrier below has passed), so that the global
  // stores are 16 bytes per lane and whole contiguous rows per group of lanes (storing straight
  // from the accumulator arrangement, 32 bytes per row and instruction, measured slower).
  // Accumulator element 4 g + e of block (i, j) is feature 32 i + 8 g + 4 (l / 32) + e of token
  // 32 j + l % 32.  Each wavefront keeps its tile [128 tokens][16 MF features] as bf16 in its own
  // LDS region: rows of CPR 16-byte chunks (8 features each), chunk position XORed with the row
  // number, the two 8-byte halves of a chunk swapped in rows with bit 3 set (16 consecutive rows
  // of one 8-byte write then cover 128 bytes of distinct banks).  Only the wavefront itself
  // touches the region: no barrier.
  constexpr int CPR = 2 * MF;                      // chunks per row
  constexpr int PITCH = CPR * 16;
  constexpr int RPI = 64 / CPR;                    // token rows per store instruction
  static_assert(4 * WTOK * PITCH <= (int)sizeof(PfShared<MF, TB>), "epilogue tile fits the stage buffers");
  unsigned char *E = smem_raw + wave_e * (WTOK * PITCH);
  // this lane's chunk: 8 consecutive features
  const int c = lane_e & (CPR - 1), rsub = lane_e / CPR;
  uint16_t *const out = Q.out;
  const long long ldo = Q.ldo;
  const int width = Q.width;
  const int col = (fb * BF_TILES + wf_e * MF) * 16 + c * 8;
  const bool lane_on = col < width;
  const bool wide = col + 8 <= width && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) && (ldo & 7) == 0;
  const int tok_base = tok0 + wt_e * WTOK + rsub;
  uint16_t *dst = out + (long long)tok_base * ldo + col;
  constexpr int NQ = WTOK / RPI;                   // store instructions per wavefront
  constexpr int NBATCH = (ROPE ? 8 : 4) * TB / 4, BQ = NQ / NBATCH;   // ... handled in batches (register budget)
  const bool lane_wide = lane_on && wide;
  constexpr int GR = 3;                            // table batches in registers: loads run two batches ahead
  // ROPE: this lane's 8 table values per row (cosines for the chunks of a head's first half, sines for
  // the others; the lane 8 further round the row of 16 lanes holds the other kind), two batches ahead
  // like the gate values.  All lanes load: the table row is clamped to the last token, never skipped.
  f32x4_t tab[GR][ROPE ? BQ : 1][2];
  auto load_tab = [&](int bt) {
    if constexpr (ROPE) {
      static_assert(!ROPE || CPR == 16, "one wavefront's features are one head of 128");
#pragma unroll
      for (int qq = 0; qq < BQ; ++qq) {
        const int tok = min(tok_base + (bt * BQ + qq) * RPI, P.T - 1);
        const float *tb = Q.rope + (long long)tok * 128 + (c & 7) * 8 + (c & 8) * 8;
        tab[bt % GR][qq][0] = *reinterpret_cast<const f32x4_t *>(tb);
        tab[bt % GR][qq][1] = *reinterpret_cast<const f32x4_t *>(tb + 4);
      }
    }
  };
  load_tab(0);
  __syncthreads();         // the epilogue reuses the LDS buffers (the loads above are in flight meanwhile)
  {
    const int wrow = lane_e & 31, wswz = lane_e & (CPR - 1);
    const int whalf = ((lane_e >> 5) ^ ((lane_e >> 3) & 1)) * 8;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < TB; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          if constexpr (GLU) {     // h = silu(gate) * up in fp32, one rounding of the result
            const uint2 sg = gpk[GLU ? i : 0][GLU ? j : 0][g];
            float u[4];            // (read out of the accumulator registers one by one, see the gate product above)
#pragma unroll
            for (int e = 0; e < 4; ++e) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(u[e]) : "a"(acc[i][j][4 * g + e]));
            w.x = pack2<DT>(u[0] * lo_f32<DT>(sg.x), u[1] * hi_f32<DT>(sg.x));
            w.y = pack2<DT>(u[2] * lo_f32<DT>(sg.y), u[3] * hi_f32<DT>(sg.y));
          } else {
            w = pk[GLU ? 0 : i][GLU ? 0 : j][g];
          }
          *reinterpret_cast<uint2 *>(E + (32 * j + wrow) * PITCH + (((4 * i + g) ^ wswz) * 16) + whalf) = w;
          // (one pair at a time, in source order: scheduled freely, all 256 sums are read out of the
          // accumulator registers first, which does not fit beside the gate values)
          if constexpr (GLU) __builtin_amdgcn_sched_barrier(0);
        }
  }
  if (ROPE && NBATCH > 1) load_tab(1);
  // LDS reads of the next batch are issued before the stores of this one (different units)
  u32x4_t d[2][BQ];
  auto read_batch = [&](int bt, u32x4_t (&dd)[BQ]) {
#pragma unroll
    for (int qq = 0; qq < BQ; ++qq) {
      const int row = (bt * BQ + qq) * RPI + rsub;
      dd[qq] = *reinterpret_cast<const u32x4_t *>(E + row * PITCH + ((c ^ (row & (CPR - 1))) * 16));
    }
  };
  auto store_batch = [&](int bt, u32x4_t (&dd)[BQ]) {
#pragma unroll
    for (int qq = 0; qq < BQ; ++qq) {
      const int q = bt * BQ + qq;
      if (((q * RPI) >> 3) & 1) dd[qq] = u32x4_t{dd[qq][2], dd[qq][3], dd[qq][0], dd[qq][1]};
      if constexpr (ROPE) {
        // This lane's chunk c holds features 8 (c % 8) .. + 7 of the first (c < 8) or the second half
        // of a head, the lane 8 further round its row of 16 lanes holds the other element of each pair
        // and needs the same 8 angles: lanes c < 8 load the cosines, the others the sines, and the
        // values cross within the row (all lanes take part: the table row is clamped, not skipped).
        const f32x4_t m0 = tab[bt % GR][ROPE ? qq : 0][0], m1 = tab[bt % GR][ROPE ? qq : 0][1];
        const bool first = c < 8;
        u32x4_t r;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float mine_l = w < 2 ? m0[2 * w] : m1[2 * w - 4], mine_h = w < 2 ? m0[2 * w + 1] : m1[2 * w - 3];
          const float othr_l = across8(mine_l), othr_h = across8(mine_h);
          const uint32_t pw = across8(dd[qq][w]);                      // the partner elements
          const float cl = first ? mine_l : othr_l, ch = first ? mine_h : othr_h;
          const float sl = first ? -othr_l : mine_l, sh = first ? -othr_h : mine_h;   // a cos - b sin | b cos + a sin
          r[w] = pack2<DT>(lo_f32<DT>(dd[qq][w]) * cl + lo_f32<DT>(pw) * sl,
                           hi_f32<DT>(dd[qq][w]) * ch + hi_f32<DT>(pw) * sh);
        }
        dd[qq] = r;
      }
      if (lane_wide && tok_base + q * RPI < P.T)
        *reinterpret_cast<u32x4_t *>(dst + (long long)(q * RPI) * ldo) = dd[qq];
    }
  };
  read_batch(0, d[0]);
#pragma unroll
  for (int bt = 0; bt < NBATCH; ++bt) {
    if (ROPE && bt + 2 < NBATCH) load_tab(bt + 2);
    if (bt + 1 < NBATCH) read_batch(bt + 1, d[(bt + 1) & 1]);
    store_batch(bt, d[bt & 1]);
  }
  // rare: output rows that are not 16-byte aligned, or the valid columns end inside this chunk
  if (lane_on && !wide) {
    for (int q = 0; q < NQ; ++q) {
      if (tok_base + q * RPI >= P.T) break;
      const int row = q * RPI + rsub;
      u32x4_t d = *reinterpret_cast<const u32x4_t *>(E + row * PITCH + ((c ^ (row & (CPR - 1))) * 16));
      if (((q * RPI) >> 3) & 1) d = u32x4_t{d[2], d[3], d[0], d[1]};
      uint16_t *o = dst + (long long)(q * RPI) * ldo;
      for (int e = 0; e < 8; ++e) {
        if (col + e >= width) break;
        unsigned v = (d[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
        o[e] = (uint16_t)v;
      }
    }
  }
#else
  (void)P; (void)bid; (void)n_tblocks; (void)fb_shift;
#endif
}

template <int DT, int MF, bool GLU, int POST = PF_POST_NONE, bool SPLIT = false, bool ROPE = false, int TB = 4>
__global__ __launch_bounds__(PF_THREADS) void prefill_kernel(const PfParams P) {
  prefill_body<DT, MF, GLU, POST, SPLIT, ROPE, TB>(P, (int)blockIdx.x, P.n_tblocks, 0);
}

// One launch with two tile shapes: the first P.n_big workgroups take 256 x 256 tiles of the feature
// blocks [0, P.fb_shift2), the others 128 x 256 tiles of the remaining feature blocks.  For large
// launches whose last round of 256 x 256 tiles would leave more than half of the compute units
// idle: that round's feature blocks run as twice as many smaller tiles, which take about 0.64 of a
// large tile's time each.
template <int DT, bool GLU, int POST, bool ROPE>
__global__ __launch_bounds__(PF_THREADS) void prefill_mixed_kernel(const PfParams P) {
  if ((int)blockIdx.x < P.n_big) prefill_body<DT, 8, GLU, POST, false, ROPE, 4>(P, (int)blockIdx.x, P.n_tblocks, 0);
  else prefill_body<DT, 8, GLU, POST, false, ROPE, 2>(P, (int)blockIdx.x - P.n_big, P.n_tblocks2, P.fb_shift2);
}

}  // namespace deinfer
