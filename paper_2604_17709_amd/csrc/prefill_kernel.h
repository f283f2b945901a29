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
// (32 * MF) features; each wavefront owns 128 tokens x (16 * MF) features: MF x 8 accumulator
// fragments of the 16x16x32 bf16 MFMA (features = MFMA rows, tokens = MFMA columns, so a lane
// ends up with 4 consecutive features of one token).  MF = 8 for a single product (256
// accumulator registers), MF = 4 for the GLU pair (2 x 128).
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
constexpr int PF_STAGES = 4;               // LDS stage buffers
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
#ifdef DEINFER_PF_TRACE
  unsigned long long *trace;   // diagnostic build only: per-workgroup cycle counts
#endif
};

template <int MF>
struct PfShared {
  uint4 w[PF_STAGES][2 * MF][64];                  // [stage][feature tile][lane]
  unsigned char x[PF_STAGES][PF_BT * PF_XPITCH];   // [stage][token row * 64 bytes], slots swizzled
};

template <int MF, bool DUAL>
__global__ __launch_bounds__(PF_THREADS) void prefill_kernel(const PfParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  PfShared<MF> &S = *reinterpret_cast<PfShared<MF> *>(smem_raw);
  constexpr int BF_TILES = 2 * MF;                 // 16-feature tiles per workgroup
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave & 1, wt = wave >> 1;         // wavefront position: features x tokens

  // consecutive workgroups share a feature block and differ in the token block: the token
  // blocks of one feature block run at the same time, spread over the XCDs, so each L2
  // streams those weights once
  const int tb = blockIdx.x % P.n_tblocks;
  const int fb = blockIdx.x / P.n_tblocks;
  const int tok0 = tb * PF_BT;

  constexpr int MB = MF / 2;                       // 32-feature blocks per wavefront
  f32x16_t acc[DUAL ? 2 : 1][MB][4];               // [product][feature block][32-token block]
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[p][i][j][e] = 0.f;

#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
    const PfProblem &Q = P.prob[p];
    // ---- load assignment (every instruction moves 1 KiB: lane l -> LDS base + 16 l).
    // Buffer addressing: a scalar resource descriptor, a scalar byte offset for the k position
    // and one 32-bit per-lane offset, which leaves the registers to the accumulators; reads
    // beyond a descriptor's size (token rows >= T, feature tiles past the last one) return
    // zeros instead of faulting.  (Host guarantees every tensor here is below 2^31 bytes.)
    constexpr int WT = BF_TILES / 4;       // feature tiles fetched per wavefront and stage
    constexpr int LPS = WT + 4;            // load instructions per wavefront and stage
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
      wres[i] = __builtin_amdgcn_make_buffer_rsrc((void *)Q.seg[sgi].frags, 0,
                                                  (int)((unsigned)(seg_end - Q.seg[sgi].tile0) * (unsigned)Q.KB * 1024u), 0x00020000);
      wtile_off[i] = (unsigned)(gt - Q.seg[sgi].tile0) * (unsigned)Q.KB * 1024u;
    }
    const unsigned wlane = lane * 16;
    // activations: instruction i of wavefront w covers tile rows 16 (4 i + w) .. + 15; lane l holds
    // slot l % 4 of row l / 4 and fetches k-chunk slot ^ ((row >> 2) & 3) = (l & 3) ^ ((l >> 4) & 3)
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)((unsigned)P.T * (unsigned)(Q.lda * 2)), 0x00020000);
    const int chunk = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) xrow[i] = (unsigned)(tok0 + 16 * (4 * i + wave) + (lane >> 2)) * (unsigned)(Q.lda * 2);
    const int n_stages = Q.KB;

    // one load instruction (index 0 .. LPS - 1) of stage st: weight tiles first, then activation rows.
    // Activation chunks beyond K re-read valid columns (k clamped to K - 8), which meet zero weights.
    const unsigned xchunk = (unsigned)(chunk * 16), xklim = (unsigned)(Q.K * 2 - 16);
    auto fetch_part = [&](int st, int idx) {
      const int buf = st & (PF_STAGES - 1);
      if (idx < WT) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wres[idx], (DEINFER_LOCAL void *)&S.w[buf][uwave * WT + idx][0], 16,
                                                 wlane, wtile_off[idx] + (unsigned)st * 1024u, 0, 0);
      } else {
        const int i = idx - WT;
        unsigned kb = (unsigned)st * (PF_BK * 2) + xchunk;
        kb = kb < xklim ? kb : xklim;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LOCAL void *)&S.x[buf][16 * (4 * i + uwave) * PF_XPITCH], 16,
                                                 xrow[i] + kb, 0, 0, 0);
      }
    };
    // Operand reads for the 32x32x16 product: lane l works on row (feature or token) l % 32 and on
    // the 8 consecutive k of group 2 s + l / 32 of the stage's four k-groups, s = 0, 1 being the
    // two k-steps of a stage.  In a packed 16-feature fragment that k-group of feature f % 16
    // sits at lane position (f % 16) + 16 * group.
    const int a_off = ((lane >> 4) & 1) * 64 + (lane & 15) + 16 * (lane >> 5);     // in uint4 units
    const int b_row = wt * 128 + (lane & 31);
    const int b_swz = ((lane & 31) >> 2) & 3;
    auto read_a = [&](int buf, int ib, int ks) -> u32x4_t {
      return *reinterpret_cast<const u32x4_t *>(&S.w[buf][wf * MF + 2 * ib][0] + a_off + 32 * ks);
    };
    auto read_b = [&](int buf, int jb, int ks) -> u32x4_t {
      const int slot = (2 * ks + (lane >> 5)) ^ b_swz;
      return *reinterpret_cast<const u32x4_t *>(&S.x[buf][(b_row + 32 * jb) * PF_XPITCH + slot * 16]);
    };
#ifdef DEINFER_PF_TRACE
    unsigned long long c_wait = 0, c_bar = 0, c0 = __builtin_readcyclecounter(), c1, c2, c3;
#endif
    constexpr int H1 = LPS / 2;            // loads 0 .. H1 - 1 of stage s + 3 go out during k-step 1 of stage s,
                                           // loads H1 .. LPS - 1 during k-step 0 of stage s + 1: at most one
                                           // load after each group of products, so their issue never holds
                                           // the matrix pipeline up
    static_assert(LPS - H1 <= 4 && H1 <= 4, "one load per token block and k-step");
#pragma unroll
    for (int i = 0; i < LPS; ++i) fetch_part(0, i);
    if (n_stages > 1) {
#pragma unroll
      for (int i = 0; i < LPS; ++i) fetch_part(1, i);
    }
    if (n_stages > 2) {
#pragma unroll
      for (int i = 0; i < H1; ++i) fetch_part(2, i);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS + H1) : "memory");
    } else if (n_stages > 1) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();          // stage 0 has landed everywhere
    asm volatile("" ::: "memory");
    u32x4_t a0[MB], a1[MB], bc, bn;
#pragma unroll
    for (int i = 0; i < MB; ++i) a0[i] = read_a(0, i, 0);
    bc = read_b(0, 0, 0);
    // one stage; F2: the second half of stage st + 2 is still to be requested, F3: stage st + 3 exists
    auto stage = [&](int st, auto f2, auto f3) {
      constexpr bool F2 = decltype(f2)::value, F3 = decltype(f3)::value;
      const int buf = st & (PF_STAGES - 1);
      const int nbuf = (st + 1) & (PF_STAGES - 1);
      // ---- k-step 0 of the stage; the feature operands of k-step 1 are read along the way
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bn = j < 3 ? read_b(buf, j + 1, 0) : read_b(buf, 0, 1);
        if (j < MB) a1[j] = read_a(buf, j, 1);
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          acc[p][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a0[i]), as_bf16x8(bc), acc[p][i][j], 0, 0, 0);
          if (F2 && i == 0 && H1 + j < LPS) fetch_part(st + 2, H1 + j);
        }
        bc = bn;
      }
      // ---- stage st + 1 has landed (this wavefront's part), barrier: it has landed everywhere and
      // nobody reads the buffer of stage st - 1 any more, which is where stage st + 3 goes
#ifdef DEINFER_PF_TRACE
      c1 = __builtin_readcyclecounter();
#endif
      if (F2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#ifdef DEINFER_PF_TRACE
      c2 = __builtin_readcyclecounter();
#endif
      // bare barrier: the wait above is the only ordering needed (loads into LDS are complete when
      // the counter says so; the buffer about to be refilled was last read a whole k-step ago);
      // the fence of __syncthreads() would drain every outstanding load instead
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
#ifdef DEINFER_PF_TRACE
      c3 = __builtin_readcyclecounter();
      c_wait += c2 - c1; c_bar += c3 - c2;
#endif
      // ---- k-step 1; the operands of the next stage's k-step 0 are read along the way
      // (after the last stage these read a stage buffer nobody writes any more; the values are unused)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bn = j < 3 ? read_b(buf, j + 1, 1) : read_b(nbuf, 0, 0);
        if (j < MB) a0[j] = read_a(nbuf, j, 0);              // a0 is not in use during k-step 1
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          acc[p][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a1[i]), as_bf16x8(bc), acc[p][i][j], 0, 0, 0);
          if (F3 && i == 0 && j < H1) fetch_part(st + 3, j);
        }
        bc = bn;
      }
    };
    {
      const std::true_type yes;
      const std::false_type no;
      int st = 0;
      for (; st + 3 < n_stages; ++st) stage(st, yes, yes);
      if (st + 2 < n_stages) { stage(st, yes, no); ++st; }
      for (; st < n_stages; ++st) stage(st, no, no);
    }
#ifdef DEINFER_PF_TRACE
    if (P.trace && blockIdx.x < 1024 && p == 0 && (tid & 63) == 0) {
      unsigned long long *tr = P.trace + (blockIdx.x * 4 + wave) * 4;
      tr[0] = __builtin_readcyclecounter() - c0; tr[1] = c_wait; tr[2] = c_bar; tr[3] = (unsigned long long)n_stages;
    }
#endif
    __syncthreads();       // the next product (GLU call) reuses the LDS buffers
  }

  // ---- epilogue: through LDS (free by now; the barrier above has passed), so that the global
  // stores are 16 bytes per lane and whole contiguous rows per group of lanes.
  // Accumulator element 4 g + e of block (i, j) is feature 32 i + 8 g + 4 (l / 32) + e of token
  // 32 j + l % 32.  Each wavefront keeps its tile [128 tokens][16 MF features] as bf16 in its own
  // LDS region: rows of CPR 16-byte chunks (8 features each), chunk position XORed with the row
  // number, the two 8-byte halves of a chunk swapped in rows with bit 4 set (conflict-free
  // writes for MF = 8).  Only the wavefront itself touches the region: no barrier.
  const PfProblem &Q = P.prob[0];
  constexpr int CPR = 2 * MF;                      // chunks per row
  constexpr int PITCH = CPR * 16;
  constexpr int RPI = 64 / CPR;                    // token rows per store instruction
  static_assert(4 * 128 * PITCH <= (int)sizeof(PfShared<MF>), "epilogue tile fits the stage buffers");
  unsigned char *E = smem_raw + wave * (128 * PITCH);
  {
    const int wrow = lane & 31, wswz = lane & (CPR - 1);
    const int whalf = ((lane >> 5) ^ ((lane >> 4) & 1)) * 8;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = acc[0][i][j][4 * g + e];
            if (DUAL) v[e] = silu_f32(v[e]) * acc[DUAL ? 1 : 0][i][j][4 * g + e];
          }
          uint2 pk;
          pk.x = pack_bf16x2(v[0], v[1]);
          pk.y = pack_bf16x2(v[2], v[3]);
          *reinterpret_cast<uint2 *>(E + (32 * j + wrow) * PITCH + (((4 * i + g) ^ wswz) * 16) + whalf) = pk;
        }
  }
  {
    // this lane's chunk: 8 features inside one 16-feature tile, hence inside one segment
    const int c = lane & (CPR - 1), rsub = lane / CPR;
    const int gt = fb * BF_TILES + wf * MF + (c >> 1);
    int sgi = 0;
    if (Q.n_seg > 1 && gt >= Q.seg[1].tile0) sgi = 1;
    if (Q.n_seg > 2 && gt >= Q.seg[2].tile0) sgi = 2;
    uint16_t *out = Q.seg[0].out;
    long long ldo = Q.seg[0].ldo;
    int tile0 = Q.seg[0].tile0, width = Q.seg[0].width;
    if (sgi == 1) { out = Q.seg[1].out; ldo = Q.seg[1].ldo; tile0 = Q.seg[1].tile0; width = Q.seg[1].width; }
    if (sgi == 2) { out = Q.seg[2].out; ldo = Q.seg[2].ldo; tile0 = Q.seg[2].tile0; width = Q.seg[2].width; }
    const int col = (gt - tile0) * 16 + (c & 1) * 8;
    const bool lane_on = gt < Q.n_ftiles && col < width;
    const bool wide = col + 8 <= width && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) && (ldo & 7) == 0;
    const int tok_base = tok0 + wt * 128 + rsub;
    uint16_t *dst = out + (long long)tok_base * ldo + col;
#pragma unroll
    for (int q = 0; q < 128 / RPI; ++q) {
      const int row = q * RPI + rsub;
      u32x4_t d = *reinterpret_cast<const u32x4_t *>(E + row * PITCH + ((c ^ (row & (CPR - 1))) * 16));
      if (((q * RPI) >> 4) & 1) d = u32x4_t{d[2], d[3], d[0], d[1]};
      if (lane_on && tok_base + q * RPI < P.T) {
        uint16_t *o = dst + (long long)(q * RPI) * ldo;
        if (wide) {
          *reinterpret_cast<u32x4_t *>(o) = d;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (col + e < width) o[e] = (uint16_t)(d[e >> 1] >> ((e & 1) * 16));
        }
      }
    }
  }
#else
  (void)P;
#endif
}

}  // namespace deinfer
