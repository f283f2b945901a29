// Memory-bound ("decode") kernels for PACKED bf16 factor pairs; the library uses them for the
// smaller calls of at most 8 tokens (one 16-token tile, NT = 1; the code also covers 2, 4 and 8
// tiles; the host takes the feature-group kernels of skinny_kernel.h where those are faster).
//
// A call is three launches on the caller's stream; kernel boundaries are the only
// synchronisation (on this part a boundary costs about a microsecond, a software barrier
// across the eight XCDs several):
//
//   down    t_part = x . [U_a | U_b | U_c]   downward projections of up to three pairs as
//           one concatenated product (Sec. 4.1).  The fragment stream of the packed U image
//           is cut into equal contiguous ranges, one per workgroup, so every compute unit
//           pulls the same number of bytes whatever the ranks are.  A 16-wide rank tile that
//           straddles range boundaries is produced in parts: workgroup g writes its fp32
//           partial sums for the tile into part buffer (g - first workgroup of the tile).
//   reduce  t = bf16(sum of the parts, in part order)   one nearest-even rounding; also
//           hands out the optional rank-space results (low-rank KV cache, Sec. 2.1).
//           t (<= 1.3 MB) stays in L2 / Infinity Cache and is written in MFMA-fragment
//           order (16 tokens x 32 rank columns per 1 KiB), so that the up kernel reads its
//           activation operand with the same fully coalesced loads as the weights.
//   up      y = t . V per pair (upward projections), 16 output features per work item, the
//           4 wavefronts of a workgroup split the rank dimension and reduce through LDS
//           ("split-r"); optional SiLU-GLU epilogue for the gate/up call.
//
// Operands: weights are the MFMA A operand (16 features x 32 k fragments, one coalesced
// 1 KiB load per wavefront), activations the B operand (16 tokens x 32 k), so the
// accumulator holds [feature][token]; T is padded to a multiple of 16 tokens.
//
// Streaming: the work of a workgroup is a short list of "batches" (a run of up to
// 4 * FM k-blocks of one tile; wavefront w takes k-blocks w, w + 4, ...): request all
// fragments of the batch, multiply, next batch.  Memory latency is hidden the GPU way, by
// occupancy: 256-thread workgroups (the wave dispatcher is a measurable part of a short
// kernel: about 8 ns per wavefront and XCD) with at least two resident per compute unit, so
// that one streams while another reduces.  The up
// kernel runs one work item per workgroup and leaves load balancing to the hardware
// dispatcher.  (A register-level software pipeline across batches was tried first: the
// compiler kept placing waited register copies on the loop back-edge, which serialised it.)
#pragma once
#include "common.h"

namespace deinfer {

constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / kWave;
constexpr int DEC_MAX_PARTS = 8;            // part buffers: a rank tile spans at most this many workgroups

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
  int Rtot_pad;         // pitch of t and of the part buffers, in elements
  uint16_t *t;          // bf16, fragment order: [T16 / 16][Rtot_pad / 32][64 lanes][8]
  float *part;          // [DEC_MAX_PARTS][T16][Rtot_pad] fp32 partial sums
  long long part_stride;  // elements between part buffers = T16 * Rtot_pad
  int n_items2;         // work items of the up kernel
  int G1;               // workgroups of the down kernel: every one takes a non-empty range
  int direct1;                // 1: one workgroup per rank tile sums the whole k range and writes t itself (no reduce kernel)
  const uint16_t *bias;       // single non-GLU pair: y = act(product + bias[feature]); may be null
  int act;                    // see act_f32
};

// Values that are the same in every lane are moved to scalar registers explicitly (the
// parameter block is read from LDS, so the compiler would otherwise keep them per lane).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T *uni_ptr(T *p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
  return reinterpret_cast<T *>((unsigned long long)lo | ((unsigned long long)hi << 32));
}

// Pointers that were read from LDS have lost their address space; these casts put them back
// into the global one so that plain global (not flat) memory instructions are used.
#ifndef DEINFER_GLOBAL
#if defined(__HIP_DEVICE_COMPILE__)
#define DEINFER_GLOBAL __attribute__((address_space(1)))
#else
#define DEINFER_GLOBAL
#endif
#endif
typedef const DEINFER_GLOBAL u32x4_t *gc_u32x4_p;
typedef DEINFER_GLOBAL float4 *g_float4_p;
typedef DEINFER_GLOBAL uint2 *g_uint2_p;
typedef DEINFER_GLOBAL uint16_t *g_u16_p;

// fragments per wavefront and batch
// (one token tile: 16 per batch in the down kernel - d_in = 4096 is exactly two batches - and 20 in
// the up kernel, where a rank of up to 2560 then is a single round trip)
template <int NT, int PHASE>
struct DecFM { static constexpr int value = NT == 1 ? (PHASE == 2 ? 20 : 16) : NT == 2 ? 6 : NT == 4 ? 3 : 2; };

struct Batch {
  const u32x4_t *a;     // fragment of k-block 0 of this tile (lane offset not included)
  const uint16_t *b;    // activation element (row 0, k 0) of this pair
  int kb0, kb1;         // k-blocks [kb0, kb1) of the tile, kb1 - kb0 <= 4 * FM
  int k_lim;            // number of valid activation columns
  bool valid;
  bool end_seg;         // last batch of its segment
  int tile, pi;         // down: the rank tile and its pair
  int part;             // down: part buffer this workgroup writes for the tile
  int otile, sub;       // up: output tile and, for the GLU call, which pair (0 gate, 1 up)
};

__device__ __forceinline__ void scalarize(Batch &d) {
  d.a = uni_ptr(d.a); d.b = uni_ptr(d.b);
  d.kb0 = uni(d.kb0); d.kb1 = uni(d.kb1); d.k_lim = uni(d.k_lim);
  d.end_seg = uni(d.end_seg) != 0; d.tile = uni(d.tile); d.pi = uni(d.pi); d.part = uni(d.part);
  d.otile = uni(d.otile); d.sub = uni(d.sub);
}

// Walks the batches of one workgroup, either of the down kernel (PHASE 1) or of the up
// kernel (PHASE 2).  All members are wave-uniform.
template <int NT, bool DUAL, int PHASE>
struct Cursor {
  static constexpr int SPAN = DEC_WAVES * DecFM<NT, PHASE>::value;
  int tile, kbp;        // down: position (rank tile, k-block inside it)
  int tile_e, kb_e;     // down: end of the range (tile index, exclusive k-block inside it)
  int g, G1;
  unsigned total;
  int it, sub, kb, G;   // up: position

  __device__ __forceinline__ void init(const DecParams &P, int g_, int G_) {
    g = g_; G = G_; G1 = P.G1;
    if (PHASE == 1) {
      // host guarantees n_rtiles * KB1 * (G1 + 1) < 2^31
      total = (unsigned)P.n_rtiles * (unsigned)P.KB1;
      const unsigned ua = (unsigned)g * total / (unsigned)G1;
      const unsigned ub = (unsigned)(g + 1) * total / (unsigned)G1;     // > ua since G1 <= total
      tile = (int)(ua / (unsigned)P.KB1);
      kbp = (int)(ua - (unsigned)tile * (unsigned)P.KB1);
      tile_e = (int)((ub - 1) / (unsigned)P.KB1);
      kb_e = (int)(ub - (unsigned)tile_e * (unsigned)P.KB1);
    } else {
      it = g; sub = 0; kb = 0;
    }
  }

  __device__ __forceinline__ bool next(const DecParams &P, Batch &d) {
    d.valid = false;
    if (PHASE == 1) {
      if (tile > tile_e) return false;
      const int seg_end = tile < tile_e ? P.KB1 : kb_e;
      int pi = 0;
      if (P.n_pairs > 1 && tile >= P.p[1].tile0) pi = 1;
      if (P.n_pairs > 2 && tile >= P.p[2].tile0) pi = 2;
      d.valid = true;
      d.tile = tile; d.pi = pi;
      d.a = reinterpret_cast<const u32x4_t *>(P.p[pi].Up) + (long long)(tile - P.p[pi].tile0) * P.KB1 * 64;
      d.b = P.x;
      d.kb0 = kbp;
      d.kb1 = kbp + SPAN < seg_end ? kbp + SPAN : seg_end;
      d.k_lim = P.d_in;
      d.end_seg = d.kb1 == seg_end;
      // first workgroup whose range reaches into this tile
      const unsigned tbeg = (unsigned)tile * (unsigned)P.KB1;
      const int g_first = (int)(((tbeg + 1u) * (unsigned)G1 + total - 1u) / total) - 1;
      d.part = g - g_first;
      d.otile = 0; d.sub = 0;
      if (d.end_seg) { ++tile; kbp = 0; } else { kbp = d.kb1; }
      scalarize(d);
      return true;
    } else {
      if (it >= P.n_items2) return false;
      int pi = 0, otile = it;
      if (DUAL) {
        pi = sub;
      } else {
        if (P.n_pairs > 1 && otile >= P.p[0].n_otiles) { otile -= P.p[0].n_otiles; pi = 1; }
        if (P.n_pairs > 2 && pi == 1 && otile >= P.p[1].n_otiles) { otile -= P.p[1].n_otiles; pi = 2; }
      }
      const int KB2 = P.p[pi].r_pad >> 5;
      d.valid = true;
      d.pi = pi; d.otile = otile; d.sub = sub; d.tile = 0; d.part = 0;
      d.a = reinterpret_cast<const u32x4_t *>(P.p[pi].Vp) + (long long)otile * KB2 * 64;
      d.b = P.t + (long long)(P.p[pi].tile0 >> 1) * 512;   // the pair's first k-block (fragments of 512 elements)
      d.kb0 = kb;
      d.kb1 = kb + SPAN < KB2 ? kb + SPAN : KB2;
      d.k_lim = P.p[pi].r_pad;
      d.end_seg = d.kb1 == KB2;
      if (d.end_seg) {
        kb = 0;
        if (DUAL && sub == 0) sub = 1;
        else { sub = 0; it += G; }     // G = grid size: with one item per workgroup this ends the walk
      } else {
        kb = d.kb1;
      }
      scalarize(d);
      return true;
    }
  }
};

template <int NT, int PHASE>
struct Frags {
  u32x4_t a[DecFM<NT, PHASE>::value];
  u32x4_t b[DecFM<NT, PHASE>::value][NT];
};

#ifndef DEINFER_LOCAL
#if defined(__HIP_DEVICE_COMPILE__)
#define DEINFER_LOCAL __attribute__((address_space(3)))
#else
#define DEINFER_LOCAL
#endif
#endif

// Request the fragments of batch d (k-blocks kb0 + wave, + 4, ... below kb1; the predicate is
// wave-uniform).  Weights: one coalesced 1 KiB fragment per k-block.
// Activations of the up kernel (PHASE 2) are the fragment-ordered t: one coalesced 1 KiB load
// per token tile and k-block.
// Activations of the down kernel (PHASE 1) come from the caller's row-major x.  With one token
// tile each lane (token l % 16, k-group l / 16) reads its 8 columns directly.  With more token
// tiles that pattern (every quad of lanes in four different rows) would make the address unit
// the bottleneck, so the 16 x 32 tile is moved by one global-to-LDS load in which a quad covers
// 64 contiguous bytes of a row (lane l: row l / 4, slot l % 4, fetching k-group
// slot ^ ((row >> 2) & 3)), into a region private to the wavefront, and read back in operand
// order, conflict free; no workgroup barrier is involved.  A lane whose columns lie beyond d_in
// re-reads the last 8 valid columns of its row, which meet zero-padded weights.
template <int NT, int PHASE>
__device__ __forceinline__ void load_frags(const Batch &d, int wave, int lane, int k_lane,
                                           const int (&rowoff)[NT], Frags<NT, PHASE> &F, uint4 *xlds) {
  constexpr int FM = DecFM<NT, PHASE>::value;
  constexpr bool XLDS = (PHASE == 1 && NT >= 2);
  const gc_u32x4_p a = (gc_u32x4_p)d.a;
  const DEINFER_GLOBAL char *b = (const DEINFER_GLOBAL char *)d.b;
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    const int kb = d.kb0 + wave + f * DEC_WAVES;
    if (kb < d.kb1) {
      F.a[f] = __builtin_nontemporal_load(a + (kb * 64 + lane));
      if (XLDS) {
        int k = kb * 32 + (((lane & 3) ^ ((lane >> 4) & 3)) << 3);      // row = lane / 4: (row >> 2) & 3 = lane >> 4
        k = k < d.k_lim - 8 ? k : d.k_lim - 8;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          __builtin_amdgcn_global_load_lds((const DEINFER_GLOBAL void *)(b + (unsigned)((rowoff[nt] + k) * 2)),
                                           (DEINFER_LOCAL void *)(xlds + (f * NT + nt) * 64), 16, 0, 0);
      } else if (PHASE == 1) {
        int k = kb * 32 + k_lane;
        k = k < d.k_lim - 8 ? k : d.k_lim - 8;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          F.b[f][nt] = *(gc_u32x4_p)(b + (unsigned)((rowoff[nt] + k) * 2));
      } else {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)     // rowoff[nt] = first fragment of token tile nt
          F.b[f][nt] = *((gc_u32x4_p)b + ((rowoff[nt] + kb) * 64 + lane));
      }
    }
  }
  if (XLDS) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the LDS tiles (and the weights) have landed
    const int lrow = lane & 15, lkg = lane >> 4;
    const int slot = lrow * 4 + (lkg ^ ((lrow >> 2) & 3));
#pragma unroll
    for (int f = 0; f < FM; ++f) {
      if (d.kb0 + wave + f * DEC_WAVES < d.kb1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          F.b[f][nt] = *reinterpret_cast<const u32x4_t *>(xlds + (f * NT + nt) * 64 + slot);
      }
    }
  }
}
template <int DT, int NT, int PHASE>
__device__ __forceinline__ void multiply(const Batch &d, int wave, const Frags<NT, PHASE> &F, f32x4_t (&acc)[NT]) {
  constexpr int FM = DecFM<NT, PHASE>::value;
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    if (d.kb0 + wave + f * DEC_WAVES < d.kb1) {     // wave-uniform
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[nt] = mfma16<DT>(F.a[f], F.b[f][nt], acc[nt]);
    }
  }
}

// PHASE 1: down kernel (grid = P.G1).  PHASE 2: up kernel (grid = any, items round-robin).
template <int DT, int NT, bool DUAL, int PHASE>
__global__ __launch_bounds__(DEC_THREADS, 2) void decode_kernel(const DecParams Pk) {
  __shared__ float4 red[(DUAL && PHASE == 2) ? 2 : 1][DEC_WAVES][NT][kWave];
  constexpr bool XLDS = (PHASE == 1 && NT >= 2);
  __shared__ uint4 xstage[XLDS ? DEC_WAVES * DecFM<NT, PHASE>::value * NT * 64 : 1];   // per-wavefront x tiles
  // The parameter block is fetched once, by one vector load per thread, and read from LDS
  // afterwards: lazily scheduled scalar loads from the kernel-argument segment would put
  // several dependent memory round trips in front of the first weight request.
  constexpr int PW = (int)((sizeof(DecParams) + 3) / 4);
  static_assert(PW <= DEC_THREADS, "parameter block too large");
  __shared__ __attribute__((aligned(16))) unsigned p_words[PW + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
#if defined(__HIP_DEVICE_COMPILE__)
  {
    typedef const __attribute__((address_space(4))) unsigned *kernarg_words_t;
    kernarg_words_t ka = (kernarg_words_t)__builtin_amdgcn_kernarg_segment_ptr();
    if (tid < PW) p_words[tid] = ka[tid];
  }
#endif
  __syncthreads();
  (void)Pk;
  const DecParams &P = *reinterpret_cast<const DecParams *>(p_words);
  const int lrow = lane & 15, lkg = lane >> 4;
  const int G = gridDim.x, g = blockIdx.x;

  // per-lane activation row offsets (elements): x rows are clamped to the last token, t rows are padded
  // (host guarantees that T * ldx and T16 * Rtot_pad fit 30 bits)
  uint4 *const xlds = xstage + (XLDS ? wave * DecFM<NT, PHASE>::value * NT * 64 : 0);
  int rowoff[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int tok = nt * 16 + (XLDS ? (lane >> 2) : lrow);
    if (PHASE == 1) {
      tok = tok < P.T ? tok : P.T - 1;
      rowoff[nt] = tok * (int)P.ldx;
    } else {
      rowoff[nt] = nt * (P.Rtot_pad >> 5);      // fragment index of (token tile nt, k-block 0)
    }
  }

  Cursor<NT, DUAL, PHASE> cur;
  cur.init(P, g, G);
  Frags<NT, PHASE> F;
  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // One batch: request its fragments, multiply, and close the segment if it ends here.
  auto step = [&](const Batch &dc) {
    load_frags<NT, PHASE>(dc, wave, lane, lkg * 8, rowoff, F, xlds);
    multiply<DT, NT, PHASE>(dc, wave, F, acc);
    // Every request of this batch has been consumed by now, so this wait costs nothing; it is here for
    // the compiler's wait-count pass.  Requests and products sit in separate branches on the same
    // wave-uniform conditions, which the pass cannot pair up: without a wait that it can see it takes
    // a request of the previous batch as possibly still in flight when the next batch computes its
    // addresses, and where the register allocator reuses a fragment register for an address it then
    // waits for ALL requests before each new one (seen: 20 serialised round trips in the up kernel).
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0), other counters untouched
    if (!dc.end_seg) return;

    // ---- segment end: reduce the partial accumulators of the wavefronts through LDS and hand the result on
    const int rb = (DUAL && PHASE == 2) ? dc.sub : 0;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      red[rb][wave][nt][lane] = make_float4(acc[nt][0], acc[nt][1], acc[nt][2], acc[nt][3]);
      acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    if (DUAL && PHASE == 2 && dc.sub == 0) return;    // gate done, up follows: reduce both at once
    __syncthreads();
    for (int nt = wave; nt < NT; nt += DEC_WAVES) {    // token tiles are shared out among the wavefronts
      float4 s = red[0][0][nt][lane];
#pragma unroll
      for (int w = 1; w < DEC_WAVES; ++w) {
        const float4 v = red[0][w][nt][lane];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      const int tok = nt * 16 + lrow;
      if (PHASE == 1 && P.direct1) {
        // this workgroup summed the whole k range of its rank tile: the result is final.  Round once
        // to bf16 and store it where the upward kernel expects its activation operand (fragment
        // order: (token tile, k-block) -> 1 KiB, lane = token % 16 + 16 * ((k % 32) / 8)); rows
        // beyond T are zero.  Also the optional rank-space output (low-rank KV cache, Sec. 2.1).
        const int col = dc.tile * 16 + lkg * 4;
        if (tok >= P.T) s = make_float4(0.f, 0.f, 0.f, 0.f);
        uint2 pk;
        pk.x = pack2<DT>(s.x, s.y);
        pk.y = pack2<DT>(s.z, s.w);
        const int frag = nt * (P.Rtot_pad >> 5) + (col >> 5);
        const int tl = lrow + 16 * ((col & 31) >> 3);
        *(g_uint2_p)((const DEINFER_GLOBAL uint16_t *)uni_ptr(P.t) + (frag * 512 + tl * 8 + (col & 7))) = pk;
        int pi = 0;
        if (P.n_pairs > 1 && dc.tile >= P.p[1].tile0) pi = 1;
        if (P.n_pairs > 2 && dc.tile >= P.p[2].tile0) pi = 2;
        const DecPair &pr = P.p[pi];
        if (pr.t_out != nullptr && tok < P.T) {
          const int c0 = col - pr.tile0 * 16;
          const float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (c0 + v < pr.r) ((g_u16_p)pr.t_out)[(long long)tok * pr.ldt_out + c0 + v] = cvt_out<DT>(sv[v]);
        }
      } else if (PHASE == 1) {
        // fp32 partial sums of this workgroup's share of the tile: 4 consecutive rank columns
        if (tok < P.T) {
          const DEINFER_GLOBAL float *base = (const DEINFER_GLOBAL float *)uni_ptr(P.part) + (long long)dc.part * P.part_stride;
          *(g_float4_p)(base + (tok * P.Rtot_pad + dc.tile * 16 + lkg * 4)) = s;
        }
      } else {
        if (DUAL) {
          float4 s2 = red[(DUAL && PHASE == 2) ? 1 : 0][0][nt][lane];
#pragma unroll
          for (int w = 1; w < DEC_WAVES; ++w) {
            const float4 v = red[(DUAL && PHASE == 2) ? 1 : 0][w][nt][lane];
            s2.x += v.x; s2.y += v.y; s2.z += v.z; s2.w += v.w;
          }
          s.x = silu_f32(s.x) * s2.x; s.y = silu_f32(s.y) * s2.y;
          s.z = silu_f32(s.z) * s2.z; s.w = silu_f32(s.w) * s2.w;
        }
        const DecPair &pr = P.p[DUAL ? 0 : dc.pi];
        const int f0 = dc.otile * 16 + lkg * 4;
        if (!DUAL && (P.bias != nullptr || P.act != ACT_NONE)) {
          // non-GLU sub-layer: bias and activation on the fp32 sums, before the one rounding
          const g_u16_p bp = (g_u16_p)uni_ptr(P.bias);
          const int act = uni(P.act);
          float b[4] = {0.f, 0.f, 0.f, 0.f};
          if (bp != nullptr) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (f0 + v < pr.d_out) b[v] = cvt_in<DT>(bp[f0 + v]);
          }
          s.x = act_f32(s.x + b[0], act); s.y = act_f32(s.y + b[1], act);
          s.z = act_f32(s.z + b[2], act); s.w = act_f32(s.w + b[3], act);
        }
        if (tok < P.T) {
          uint16_t *dst = pr.y + (long long)tok * pr.ldy + f0;
          if (f0 + 3 < pr.d_out && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
            uint2 pk;
            pk.x = pack2<DT>(s.x, s.y);
            pk.y = pack2<DT>(s.z, s.w);
            *(g_uint2_p)(dst) = pk;
          } else {
            const float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (f0 + v < pr.d_out) ((g_u16_p)dst)[v] = cvt_out<DT>(sv[v]);
          }
        }
      }
    }
    __syncthreads();
  };

  Batch d;
  while (cur.next(P, d)) {
    step(d);
  }
}

// t[tok][c] = bf16(sum over the parts of rank tile c / 16, in part order); rows T..T16-1 of t
// are zero.  One thread per token row and group of 4 rank columns.  Also writes the optional
// rank-space outputs.  Grid: ceil(T16 * Rtot_pad / 4 / 256) x 256 threads.
template <int DT>
__global__ __launch_bounds__(256) void decode_reduce_kernel(const DecParams P, int T16) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int groups = P.Rtot_pad >> 2;
  if (i >= (long long)T16 * groups) return;
  const int tok = (int)(i / groups);
  const int col = (int)(i - (long long)tok * groups) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (tok < P.T) {
    const int tile = col >> 4;
    const unsigned total = (unsigned)P.n_rtiles * (unsigned)P.KB1;
    const unsigned tbeg = (unsigned)tile * (unsigned)P.KB1, tend = tbeg + (unsigned)P.KB1;
    const int g_first = (int)(((tbeg + 1u) * (unsigned)P.G1 + total - 1u) / total) - 1;
    const int g_last = (int)((tend * (unsigned)P.G1 + total - 1u) / total) - 1;
    const float *src = P.part + (long long)tok * P.Rtot_pad + col;
    for (int k = 0; k <= g_last - g_first; ++k) {
      const float4 v = *reinterpret_cast<const float4 *>(src + (long long)k * P.part_stride);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    int pi = 0;
    if (P.n_pairs > 1 && tile >= P.p[1].tile0) pi = 1;
    if (P.n_pairs > 2 && tile >= P.p[2].tile0) pi = 2;
    const DecPair &pr = P.p[pi];
    if (pr.t_out != nullptr) {
      const int c0 = col - pr.tile0 * 16;
      const float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (c0 + v < pr.r) pr.t_out[(long long)tok * pr.ldt_out + c0 + v] = cvt_out<DT>(sv[v]);
    }
  }
  uint2 pk;
  pk.x = pack2<DT>(s.x, s.y);
  pk.y = pack2<DT>(s.z, s.w);
  // fragment order: (token tile, k-block) -> 1 KiB, lane = token % 16 + 16 * ((k % 32) / 8)
  const long long frag = (long long)(tok >> 4) * (P.Rtot_pad >> 5) + (col >> 5);
  const int lane = (tok & 15) + 16 * ((col & 31) >> 3);
  *reinterpret_cast<uint2 *>(P.t + frag * 512 + lane * 8 + (col & 7)) = pk;
}

}  // namespace deinfer
