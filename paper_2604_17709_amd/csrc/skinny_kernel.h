// Memory-bound ("decode", T <= 128 tokens) kernels for PACKED bf16 factor pairs.
//
// Both stages of y = (x U) V (Sec. 4.1) are the product  out[T x F] = act[T x K] . W^T  with few
// token rows: every weight is used for T <= 128 tokens, so the weights must stream from HBM
// exactly once at full rate while the activations (a few hundred KiB) come from L2.
//
// Work split: the feature axis is cut into groups of 128, 96 or 64 features (NW = 4, 3 or 2
// wavefronts x one 32-feature block), the k axis into P ranges; one workgroup = one (group,
// k-range) rectangle.  The host takes the narrower groups where they fill clearly more of the
// compute units than the 128-feature split with the same or fewer k-ranges.
//   * weights: every wavefront loads its own fragments straight into registers (two 16-byte
//     loads per lane and k-block cover two packed 16-feature fragments, non-temporal: they are
//     never needed again), one stage (4 k-blocks = 8 KiB per wavefront) ahead of the products;
//   * activations: the [T x 128 k] slab of a stage is shared by the four wavefronts: it goes
//     from global memory straight into LDS (16-byte slots of a 256-byte row, slot index XORed
//     with the row number, so the operand reads are conflict free), double buffered;
//   * products: 32x32x16 bf16 MFMA, features = rows, tokens = columns, fp32 accumulators;
//   * the rectangle's fp32 result goes to a partial buffer; a second small kernel adds the P
//     partial sums in a fixed order (deterministic), applies the epilogue (bf16 rounding of t,
//     SiLU-GLU of the MLP call) and writes the outputs.  (Letting the last workgroup of a
//     feature group do the sum inside the streaming kernel was measured slower, also with the
//     k-ranges of a group placed on one XCD so that the partial sums stay in one L2: one
//     workgroup's read-back of P tiles takes longer than a launch that uses the whole device,
//     and groups that are no multiple of 8 unbalance the XCDs' streams.)
// Every wavefront keeps three stages of weight loads in flight (four register sets, four LDS
// slabs); one or two workgroups per compute unit.  A per-workgroup trace (wall-clock stamps
// in an instrumented build) of the largest launch of a 7B block at T = 64 (172 workgroups, 19 stages)
// shows: all workgroups start within 0.2 us, the first stage lands 3.0 us later, the other 18
// stages take 19 us (5.2 TB/s of weights), 1 us of stores.  The same loop without the activation
// loads takes 15.7 us, without the products 17.7 us, without both 15.0 us (6.6 TB/s): the
// activation slabs, which every workgroup re-reads from L2 (half the weight bytes at T = 64),
// cost more than the products.  A layout in which a workgroup's stage is one contiguous 32 KiB
// piece timed the same as the per-tile layout.
#pragma once
#include "common.h"

namespace deinfer {

#if defined(__HIP_DEVICE_COMPILE__)
#define DEINFER_LDS_PTR __attribute__((address_space(3)))
#else
#define DEINFER_LDS_PTR
#endif

constexpr int SK_KB = 4;                   // k-blocks per stage at most (k-ranges are multiples of it)
constexpr int SK_MAX_PARTS = 16;           // k-ranges per product at most
constexpr int SK_SLABS = 4;                // activation slabs in LDS = weight register sets

struct SkProblem {           // one product  act[T x K] . W^T,  W packed as [tiles][KB][64] fragments
  const uint16_t *act;       // row-major bf16
  long long lda;
  const uint4 *frags;
  int K;                     // valid k (columns of act), at least 8; columns K .. (K rounded up to 8) - 1 of a row
                             // are readable memory of unknown contents
  int KB;                    // 32-wide k-blocks of the packed weights (zero padded)
  int n_ftiles;              // 16-feature tiles
  int group0;                // first feature group of this product in the launch
  int kb_per_part;           // k-blocks per k-range (a multiple of SK_KB)
  // direct launches only (SkParams::direct): where the product goes
  uint16_t *out;             // row-major, 16-bit storage type
  long long ldo;
  int width;                 // valid output columns
};

struct SkParams {
  int T;
  int n_prob;
  int n_groups;              // feature groups of all products; grid = n_groups * P
  int P;
  SkProblem prob[3];
  float *part;               // [P][NB * 32][n_groups * 128] fp32
  long long part_stride;     // NB * 32 * n_groups * 128
  // direct = 1 (only with P = 1, where the rectangle is the whole sum): the workgroup rounds and
  // stores its outputs itself, out = act(sum + bias[column]), and no reduce launch follows
  int direct;
  const uint16_t *bias;      // single product only; may be null
  int act;                   // see act_f32
};

// NB = 32-token blocks (1, 2 or 4); KBS = k-blocks per stage (4, or 2: half the slab, so that two
// workgroups fit a compute unit also with 128 tokens)
// DT = storage type of weights and activations (DT_BF16 or DT_F16)
// NW = wavefronts per workgroup = 32-feature blocks per feature group (4, 3 or 2): narrower groups
// give more workgroups without more k-ranges (no extra partial sums) at the price of activation
// traffic, which one slab per group and stage makes proportional to the number of groups.
// TAIL: the valid columns K of the activation rows may be no multiple of 8 (the caller's rank-space rows of
// an upward projection alone): what the last chunk holds beyond column K - 1 is cleared in LDS
// (lds_zero_chunk_tail in common.h).  A variant of its own: as a run-time branch per stage the step cost
// 2 % of every call's time.
template <int DT, int NB, int KBS, int NW, bool TAIL = false>
__global__ __launch_bounds__(64 * NW, NW >= 3 ? 2 : 1) void skinny_kernel(const SkParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  constexpr int XROW = KBS * 64;          // bytes per token row of a stage's activation slab
  constexpr int SPR = KBS * 4;            // 16-byte slots per row = lanes per row of a slab load
  constexpr int RPI = 64 / SPR;           // rows per slab load instruction
  // Slot swizzle of a token row: a quarter-wave reads 16 consecutive rows at one logical slot, and the
  // 16 physical (row, slot) positions must fall into 16 different groups of four banks.  A 256-byte row
  // spans all 64 banks (the slot alone decides: XOR with row % 16); a 128-byte row spans half of them
  // (row parity picks the half, so the slot is XORed with (row / 2) % 8).
  auto swz = [](int row) { return SPR == 16 ? (row & 15) : ((row >> 1) & (SPR - 1)); };
  __shared__ __attribute__((aligned(16))) unsigned char xs[SK_SLABS][NB * 32 * XROW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // consecutive workgroups share the k-range (the same activation slab, kept hot in L2)
  const int g = blockIdx.x % P.n_groups;
  const int part = blockIdx.x / P.n_groups;
  int pi = 0;
  if (P.n_prob > 1 && g >= P.prob[1].group0) pi = 1;
  if (P.n_prob > 2 && g >= P.prob[2].group0) pi = 2;
  const SkProblem &Q = P.prob[pi];
  const int fblk = (g - Q.group0) * NW + wave;         // this wavefront's 32-feature block
  const int kb_begin = part * Q.kb_per_part;
  int kb_end = kb_begin + Q.kb_per_part;
  kb_end = kb_end < Q.KB ? kb_end : Q.KB;
  const int n_stages = kb_end > kb_begin ? (kb_end - kb_begin + KBS - 1) / KBS : 0;

  // ---- weights: buffer addressing; a lane offset beyond the descriptor's size reads zeros, which
  // is how feature tiles past the last one and k-blocks past the range contribute nothing
  const unsigned wbytes = (unsigned)Q.n_ftiles * (unsigned)Q.KB * 1024u;
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.frags, 0, (int)wbytes, 0x00020000);
  // lane l holds feature l % 32 (tile 2 fblk + (l / 16) % 2, row l % 16) and k-group 2 s + l / 32
  const unsigned wtile = (unsigned)(2 * fblk + ((lane >> 4) & 1));
  const unsigned wlane = wtile * (unsigned)Q.KB * 1024u + (unsigned)(((lane & 15) + 16 * (lane >> 5)) * 16);
  const bool wtile_ok = (int)wtile < Q.n_ftiles;
  constexpr unsigned OOB = 0x7ffffff0u;
  // ---- activations
  const unsigned xbytes = (unsigned)(((long long)(P.T - 1) * Q.lda + ((Q.K + 7) & ~7)) * 2);
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)xbytes, 0x00020000);
  constexpr int NI = NB * 32 / RPI;                     // slab load instructions per stage
  constexpr int NX = (NI + NW - 1) / NW;                // ... per wavefront (where NW does not divide NI a wavefront repeats
                                                        // its previous instruction: every wavefront issues the same number)
  unsigned xrow[NX], xchunk[NX];
  int xm[NX];
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    int m = i * NW + wave;                              // instruction m covers rows RPI m .. RPI m + RPI - 1
    if (m >= NI) m -= NW;
    xm[i] = m;
    const int row = RPI * m + lane / SPR;
    xrow[i] = row < P.T ? (unsigned)row * (unsigned)(Q.lda * 2) : OOB;
    xchunk[i] = (unsigned)(((lane & (SPR - 1)) ^ swz(row)) * 16);
  }
  const unsigned xkend = (unsigned)(((Q.K + 7) >> 3) * 16);      // bytes of a row up to the end of the chunk that holds column K - 1
  const unsigned xklim = (unsigned)(Q.K * 2 - 16);               // (K a multiple of 8: the last chunk)
  // the chunk with columns that are not to be used: its stage (of this workgroup's k-range) and its slot there
  const int krem = Q.K & 7;
  const int kb_fix = Q.K >> 5;
  const int st_fix = (TAIL && krem != 0 && kb_fix >= kb_begin && kb_fix < kb_end) ? (kb_fix - kb_begin) / KBS : -1;
  const int slot_fix = ((kb_fix - kb_begin) % KBS) * 4 + ((Q.K >> 3) & 3);

  auto fetch_x = [&](int st, int buf) {
    const unsigned kbyte0 = (unsigned)(kb_begin + st * KBS) * 64u;
    const unsigned dead = st < n_stages ? 0u : OOB;     // uniform; OR-ed in: no branch around the loads
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      // chunks beyond K re-read a chunk of valid columns (the last one; TAIL: the first one), which meets zero weights
      unsigned kb = kbyte0 + xchunk[i];
      kb = TAIL ? (kb < xkend ? kb : 0u) : (kb < xklim ? kb : xklim);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LDS_PTR void *)&xs[buf][xm[i] * RPI * XROW], 16,
                                               (xrow[i] + kb) | dead, 0, 0, 0);
    }
  };
  auto fetch_w = [&](u32x4_t (&w)[KBS * 2], int st) {
#pragma unroll
    for (int kbi = 0; kbi < KBS; ++kbi) {
      const int kb = kb_begin + st * KBS + kbi;
      const unsigned off = (wtile_ok && kb < kb_end) ? wlane : OOB;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        w[kbi * 2 + ks] = __builtin_amdgcn_raw_buffer_load_b128(wres, off, kb * 1024 + ks * 512, 2);
    }
  };

  f32x16_t acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  const int b_row = lane & 31;
  // A stage is 8 steps (k-block, half) of NB products.  The token operands are read from LDS
  // DEPTH steps ahead of their use into rotating registers, one read after each product (left to
  // itself the compiler reads and waits right before every pair of products, which leaves the
  // matrix pipeline idle two thirds of the time at T = 128).
  constexpr int STEPS = KBS * 2;
  constexpr int DEPTH = NB >= 4 ? 2 : NB == 2 ? 3 : 6;
  auto read_b = [&](int buf, int step, int j) -> u32x4_t {
    const int slot = (step * 2 + (lane >> 5)) ^ swz(b_row);               // step = 2 * k-block + half: 16-byte slot 2 * step + lane / 32
    return *reinterpret_cast<const u32x4_t *>(&xs[buf][(32 * j + b_row) * XROW + slot * 16]);
  };
  // One load of stage `fst` (index 0 .. 7: weights into wn, 8 .. 8 + NX - 1: activation slab rows into slab fbuf).
  auto fetch_one = [&](u32x4_t (&wn)[KBS * 2], int fst, int fbuf, int idx) {
    if (idx < KBS * 2) {
      const int kb = kb_begin + fst * KBS + (idx >> 1);
      const unsigned off = (wtile_ok && kb < kb_end) ? wlane : OOB;
      wn[idx] = __builtin_amdgcn_raw_buffer_load_b128(wres, off, kb * 1024 + (idx & 1) * 512, 2);
    } else {
      const int i = idx - KBS * 2;
      const unsigned dead = fst < n_stages ? 0u : OOB;
      unsigned kb = (unsigned)(kb_begin + fst * KBS) * 64u + xchunk[i];
      kb = TAIL ? (kb < xkend ? kb : 0u) : (kb < xklim ? kb : xklim);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LDS_PTR void *)&xs[fbuf][xm[i] * RPI * XROW], 16,
                                               (xrow[i] + kb) | dead, 0, 0, 0);
    }
  };
  // The products of the stage in slab `buf`; the loads of stage `fst` are issued along the way,
  // spread evenly behind the products (all of them in front would hold the first product up
  // for their issue time).
  auto compute = [&](const u32x4_t (&w)[KBS * 2], int buf, u32x4_t (&wn)[KBS * 2], int fst, int fbuf) {
    constexpr int NLOAD = KBS * 2 + NX, NPOS = STEPS * NB;
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

  // Stage s uses register set / slab s % 4.  Every stage issues exactly 8 + NX loads (those past
  // the k-range read zeros through an out-of-range offset and cost no traffic), so "all but the
  // loads of the next stage have arrived" is one constant wait.
  if (n_stages > 0) {
    u32x4_t w0[KBS * 2], w1[KBS * 2], w2[KBS * 2], w3[KBS * 2];
    fetch_w(w0, 0); fetch_x(0, 0);
    fetch_w(w1, 1); fetch_x(1, 1);
    fetch_w(w2, 2); fetch_x(2, 2);
    auto stage = [&](const u32x4_t (&w)[KBS * 2], u32x4_t (&wn)[KBS * 2], int st, int slab) {
      // stage st has arrived (this wavefront's part): all but the loads of the next two stages
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((SK_SLABS - 2) * (KBS * 2 + NX)) : "memory");
      __builtin_amdgcn_s_barrier();                     // ... everywhere; nobody reads slab (st - 1) % 4 any more
      asm volatile("" ::: "memory");
      if constexpr (TAIL) {
        if (st == st_fix) {                             // (uniform) the chunk that holds column K - 1 is in this slab
          if (tid < NB * 32) lds_zero_chunk_tail(&xs[slab][tid * XROW + ((slot_fix ^ swz(tid)) * 16)], krem);
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
      }
      compute(w, slab, wn, st + SK_SLABS - 1, slab == 0 ? SK_SLABS - 1 : slab - 1);
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

  // ---- result: element 4 q + e of block j is feature 8 q + 4 (l / 32) + e, token 32 j + l % 32
  if (P.direct) {
    const int col0 = fblk * 32 + 4 * (lane >> 5);         // first of this lane's columns for q = 0
    uint16_t *o = Q.out + (long long)(lane & 31) * Q.ldo;
    const bool vec = (reinterpret_cast<uintptr_t>(Q.out) & 7u) == 0 && (Q.ldo & 3) == 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int col = col0 + 8 * q;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (P.bias != nullptr) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (col + e < Q.width) bv[e] = cvt_in<DT>(P.bias[col + e]);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        if (32 * j + (lane & 31) >= P.T) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = act_f32(acc[j][4 * q + e] + bv[e], P.act);
        uint16_t *dst = o + (long long)(32 * j) * Q.ldo + col;
        if (vec && col + 4 <= Q.width) {
          *reinterpret_cast<uint2 *>(dst) = uint2{pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3])};
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < Q.width) dst[e] = cvt_out<DT>(v[e]);
        }
      }
    }
    return;
  }
  const long long F = (long long)P.n_groups * (32 * NW);
  float *dst = P.part + (long long)part * P.part_stride + (long long)(lane & 31) * F +
               (long long)g * (32 * NW) + wave * 32 + 4 * (lane >> 5);
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    if (32 * j + (lane & 31) < P.T) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4_t v = {acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]};
        *reinterpret_cast<f32x4_t *>(dst + (long long)(32 * j) * F + 8 * q) = v;
      }
    }
  }
#else
  (void)P;
#endif
}

// ---- sum of the partial results + epilogue ------------------------------------------------------
struct SkOut {               // a run of columns of the partial buffer that belongs to one output
  int col0;                  // first column in the partial buffer
  int width;                 // valid columns
  uint16_t *out;             // bf16 row-major
  long long ldo;
  int width2;                // optional second copy of the first width2 columns (rank-space output) ...
  uint16_t *out2;            // ... or null
  long long ldo2;
};
struct SkReduceParams {
  const float *part;
  long long part_stride;
  int P, T, F;               // F = columns of the partial buffer
  int n_out;
  SkOut o[3];
  int glu_delta;             // > 0: o[0] columns are the gate product, the up product sits glu_delta columns later
  const uint16_t *bias;      // single non-GLU product: out = act(sum + bias[column]); may be null
  int act;                   // see act_f32
};

// one thread = 8 consecutive columns of one token row
template <int DT>
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const SkReduceParams R) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int c8 = R.F / 8;
  const int tok = (int)(idx / c8);
  const int col = (int)(idx % c8) * 8;
  if (tok >= R.T) return;
  int oi = -1;
#pragma unroll
  for (int i = 0; i < 3; ++i)
    if (i < R.n_out && col >= R.o[i].col0 && col < R.o[i].col0 + R.o[i].width) oi = i;
  if (oi < 0) return;
  const SkOut &o = R.o[oi];
  float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float u[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float *src = R.part + (long long)tok * R.F + col;
  // eight parts at a time: all loads first (independent, one round trip), then the sums in part
  // order (deterministic)
  constexpr int CH = 8;
  auto chunk = [&](const int p0) {
    f32x4_t a[CH][2];
#pragma unroll
    for (int p = 0; p < CH; ++p) {
      a[p][0] = a[p][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (p0 + p < R.P) {
        a[p][0] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(src + (p0 + p) * R.part_stride));
        a[p][1] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(src + (p0 + p) * R.part_stride + 4));
      }
    }
    if (R.glu_delta > 0) {
      f32x4_t b[CH][2];
#pragma unroll
      for (int p = 0; p < CH; ++p) {
        b[p][0] = b[p][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (p0 + p < R.P) {
          b[p][0] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(src + (p0 + p) * R.part_stride + R.glu_delta));
          b[p][1] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(src + (p0 + p) * R.part_stride + R.glu_delta + 4));
        }
      }
#pragma unroll
      for (int p = 0; p < CH; ++p)
#pragma unroll
        for (int e = 0; e < 4; ++e) { u[e] += b[p][0][e]; u[4 + e] += b[p][1][e]; }
    }
#pragma unroll
    for (int p = 0; p < CH; ++p)
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] += a[p][0][e]; v[4 + e] += a[p][1][e]; }
  };
  chunk(0);                                               // the usual case: at most eight parts, no loop
  for (int p0 = CH; p0 < R.P; p0 += CH) chunk(p0);
  if (R.glu_delta > 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = silu_f32(v[e]) * u[e];
  }
  const int oc = col - o.col0;
  if (R.glu_delta <= 0 && (R.bias != nullptr || R.act != ACT_NONE)) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      v[e] = act_f32(v[e] + ((R.bias != nullptr && oc + e < o.width) ? cvt_in<DT>(R.bias[oc + e]) : 0.f), R.act);
  }
  const u32x4_t pk = {pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3]), pack2<DT>(v[4], v[5]), pack2<DT>(v[6], v[7])};
  uint16_t *dst = o.out + (long long)tok * o.ldo + oc;
  if (oc + 8 <= o.width && ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0)) {
    *reinterpret_cast<u32x4_t *>(dst) = pk;
  } else {
    for (int e = 0; e < 8; ++e)
      if (oc + e < o.width) dst[e] = (uint16_t)(pk[e >> 1] >> ((e & 1) * 16));
  }
  if (o.out2 && oc < o.width2) {
    uint16_t *d2 = o.out2 + (long long)tok * o.ldo2 + oc;
    for (int e = 0; e < 8; ++e)
      if (oc + e < o.width2) d2[e] = (uint16_t)(pk[e >> 1] >> ((e & 1) * 16));
  }
}

}  // namespace deinfer
