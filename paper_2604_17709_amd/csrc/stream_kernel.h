// Memory-bound kernel for a stage with many output features (T <= 64 tokens, PACKED bf16 pairs):
// no partial sums leave the workgroup, so the stage is ONE launch with its epilogue inside.
//
//   out[T x F] = act[T x K] . W^T,  W packed as [tiles][KB][64] fragments (Sec. 4.1, either stage)
//
// One workgroup = one block of 32 features; its four wavefronts split the k range of that block
// ("split-r reduction through LDS"): each streams its quarter of the block's weights straight into
// registers (non-temporal, every byte is used once) and keeps its own [T x 64 k] activation slabs
// in its own LDS region (global -> LDS loads, 64-byte rows with XOR-swizzled 16-byte slots).
// Nothing is shared between the wavefronts until the end, so there is no barrier in the loop; a
// wavefront waits only for its own loads.  Four slots (64 k each at T <= 32, 32 k at T <= 64) are in
// flight per wavefront; two workgroups share a compute unit (64 KiB of LDS each).
// The four accumulator sets are added through LDS and the epilogue (bf16 rounding, optional second
// copy of t, SiLU-GLU) writes the final output.  For the GLU call the workgroup owns 32 output
// columns: wavefronts 0, 1 take the two k halves of the gate block, 2, 3 those of the up block.
// Activation traffic is T / 32 times the weight traffic (2 x at T = 64) and comes from L2.
#pragma once
#include "common.h"
#include "skinny_kernel.h"

namespace deinfer {

#if defined(__HIP_DEVICE_COMPILE__)
#define DEINFER_LDS3 __attribute__((address_space(3)))
#else
#define DEINFER_LDS3
#endif

constexpr int ST_THREADS = 256;
constexpr int ST_SLOTS = 4;                // slots in flight per wavefront (register sets / LDS slabs)

struct StProblem {           // one product
  const uint16_t *act;       // row-major bf16 [T x K]
  long long lda;
  const uint4 *frags;
  int K;                     // valid k (columns of act), at least 8; columns K .. (K rounded up to 8) - 1 of a row
                             // are readable memory of unknown contents (lds_zero_chunk_tail in common.h)
  int KB;                    // 32-wide k-blocks of the packed weights (zero padded)
  int n_ftiles;              // 16-feature tiles
  int block0;                // first 32-feature block of this product in the launch
  uint16_t *out;             // bf16 row-major output of this product
  long long ldo;
  int width;                 // valid output columns
  int width2;                // optional second copy of the first width2 columns (rank-space output) ...
  uint16_t *out2;            // ... or null
  long long ldo2;
};

struct StParams {
  int T;
  int n_prob;
  int glu;                   // 1: prob[0] = gate, prob[1] = up (same shapes); output silu(gate) * up through prob[0]
  StProblem prob[3];
  const uint16_t *bias;      // single non-GLU product: out = act(product + bias[column]); may be null
  int act;                   // see act_f32
};

// NB = 32-token blocks (1 or 2)
// TAIL: as in skinny_kernel.h (rank-space rows whose valid columns are no multiple of 8)
template <int DT, int NB, bool TAIL = false>
__global__ __launch_bounds__(ST_THREADS, 2) void stream_kernel(const StParams P) {
#if defined(__HIP_DEVICE_COMPILE__)      // the body uses device-only builtins; the host pass only needs the stub
  constexpr int ST_SKB = 2 / NB;                                    // k-blocks per slot: 16 KiB of slab per wavefront
  constexpr int SLAB = ST_SKB * NB * 32 * 64;                       // bytes of one slot's activation slab
  __shared__ __attribute__((aligned(16))) unsigned char lds[4 * ST_SLOTS * SLAB];
  static_assert(4 * ST_SLOTS * SLAB >= 4 * NB * 4 * 64 * 16, "the reduction buffer fits the slab space");
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = blockIdx.x;
  int pi = 0;
  if (!P.glu) {
    if (P.n_prob > 1 && blk >= P.prob[1].block0) pi = 1;
    if (P.n_prob > 2 && blk >= P.prob[2].block0) pi = 2;
  } else {
    pi = wave >> 1;                                   // gate: wavefronts 0, 1; up: 2, 3
  }
  const StProblem &Q = P.prob[pi];
  const int fblk = P.glu ? blk : blk - Q.block0;      // 32-feature block inside the product
  // this wavefront's k range
  const int n_split = P.glu ? 2 : 4;
  const int ksub = P.glu ? (wave & 1) : wave;
  const int per = (Q.KB + n_split - 1) / n_split;
  const int kb_begin = ksub * per;
  int kb_end = kb_begin + per;
  kb_end = kb_end < Q.KB ? kb_end : Q.KB;
  const int n_slots = kb_end > kb_begin ? (kb_end - kb_begin + ST_SKB - 1) / ST_SKB : 0;

  // ---- weights: a lane offset beyond the descriptor's size reads zeros (tiles past the last one,
  // k-blocks past the range, slots past the last one) and costs no traffic
  constexpr unsigned OOB = 0x7ffffff0u;
  const unsigned wbytes = (unsigned)Q.n_ftiles * (unsigned)Q.KB * 1024u;
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.frags, 0, (int)wbytes, 0x00020000);
  // lane l holds feature l % 32 (tile 2 fblk + (l / 16) % 2, row l % 16) and k-group 2 s + l / 32
  const unsigned wtile = (unsigned)(2 * fblk + ((lane >> 4) & 1));
  const unsigned wlane = (int)wtile < Q.n_ftiles
                             ? wtile * (unsigned)Q.KB * 1024u + (unsigned)(((lane & 15) + 16 * (lane >> 5)) * 16) : OOB;
  // ---- activations: 16 rows x 64 bytes per load instruction; lane l holds slot l % 4 of row l / 4
  // and fetches k-chunk slot ^ ((row >> 2) & 3)
  const unsigned xbytes = (unsigned)(((long long)(P.T - 1) * Q.lda + ((Q.K + 7) & ~7)) * 2);
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void *)Q.act, 0, (int)xbytes, 0x00020000);
  constexpr int NXI = NB * 2;                          // load instructions per k-block
  unsigned xrow[NXI];
#pragma unroll
  for (int i = 0; i < NXI; ++i) {
    const int row = 16 * i + (lane >> 2);
    xrow[i] = row < P.T ? (unsigned)row * (unsigned)(Q.lda * 2) : OOB;
  }
  const unsigned xchunk = (unsigned)((((lane & 3) ^ ((lane >> 4) & 3))) * 16);
  const unsigned xkend = (unsigned)(((Q.K + 7) >> 3) * 16);      // bytes of a row up to the end of the chunk that holds column K - 1
  const unsigned xklim = (unsigned)(Q.K * 2 - 16);               // (K a multiple of 8: the last chunk)
  unsigned char *const slab0 = lds + wave * (ST_SLOTS * SLAB);      // this wavefront's slabs
  // the chunk with columns that are not to be used: its slot (of this wavefront's k range), k-block and position there
  const int krem = Q.K & 7;
  const int kb_fix = Q.K >> 5;
  const int s_fix = (TAIL && krem != 0 && kb_fix >= kb_begin && kb_fix < kb_end) ? (kb_fix - kb_begin) / ST_SKB : -1;
  const int kbi_fix = (kb_fix - kb_begin) % ST_SKB;

  auto fetch = [&](u32x4_t (&w)[ST_SKB * 2], int slot, int buf) {
#pragma unroll
    for (int kbi = 0; kbi < ST_SKB; ++kbi) {
      const int kb = kb_begin + slot * ST_SKB + kbi;
      const bool live = kb < kb_end;                                 // uniform
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        w[kbi * 2 + ks] = __builtin_amdgcn_raw_buffer_load_b128(wres, live ? wlane : OOB, kb * 1024 + ks * 512, 2);
      // chunks beyond K re-read a chunk of valid columns (the last one; TAIL: the first one), which meets zero weights
      unsigned kbyte = (unsigned)kb * 64u + xchunk;
      kbyte = TAIL ? (kbyte < xkend ? kbyte : 0u) : (kbyte < xklim ? kbyte : xklim);
#pragma unroll
      for (int i = 0; i < NXI; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (DEINFER_LDS3 void *)(slab0 + buf * SLAB + (kbi * NB * 32 + 16 * i) * 64), 16,
                                                 live ? xrow[i] + kbyte : OOB, 0, 0, 0);
    }
  };

  f32x16_t acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  const int b_row = lane & 31;
  const int b_swz = (b_row >> 2) & 3;
  auto compute = [&](const u32x4_t (&w)[ST_SKB * 2], int buf) {
#pragma unroll
    for (int kbi = 0; kbi < ST_SKB; ++kbi)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int slot16 = ((2 * ks + (lane >> 5)) ^ b_swz) * 16;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const u32x4_t b = *reinterpret_cast<const u32x4_t *>(slab0 + buf * SLAB + (kbi * NB * 32 + 32 * j + b_row) * 64 + slot16);
          acc[j] = mfma32<DT>(w[kbi * 2 + ks], b, acc[j]);
        }
      }
  };

  // Slot s uses register set / slab s % 4.  Every slot issues exactly LPS loads, so "all but the loads
  // of the next two slots have arrived" is one constant wait; the slot count is rounded up to a
  // multiple of four (a slot past the last one multiplies the zeros its loads returned).
  constexpr int LPS = ST_SKB * (2 + NXI);
  if (n_slots > 0) {
    u32x4_t w0[ST_SKB * 2], w1[ST_SKB * 2], w2[ST_SKB * 2], w3[ST_SKB * 2];
    fetch(w0, 0, 0);
    fetch(w1, 1, 1);
    fetch(w2, 2, 2);
    auto slot = [&](const u32x4_t (&w)[ST_SKB * 2], u32x4_t (&wn)[ST_SKB * 2], int s, int buf) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((ST_SLOTS - 2) * LPS) : "memory");   // slot s has arrived
      fetch(wn, s + ST_SLOTS - 1, buf == 0 ? ST_SLOTS - 1 : buf - 1);              // slab (s - 1) % 4 is free: this wavefront read it
      if constexpr (TAIL) {
        if (s == s_fix) {                               // (uniform) this wavefront's own slab: no barrier, LDS accesses of a wavefront stay in order
          if (lane < NB * 32)
            lds_zero_chunk_tail(slab0 + buf * SLAB + (kbi_fix * NB * 32 + lane) * 64 + ((((Q.K >> 3) & 3) ^ ((lane >> 2) & 3)) * 16), krem);
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
      }
      compute(w, buf);
    };
    for (int s = 0; s < n_slots; s += 4) {
      slot(w0, w3, s, 0);
      slot(w1, w0, s + 1, 1);
      slot(w2, w1, s + 2, 2);
      slot(w3, w2, s + 3, 3);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // drain the out-of-range tail loads before LDS is reused
  }

  // ---- sum of the four accumulator sets through LDS.  Element 4 q + e of block j is feature
  // 8 q + 4 (l / 32) + e, token 32 j + l % 32.
  __syncthreads();
  float4 *red = reinterpret_cast<float4 *>(lds);                    // [wave][j][q][lane]
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      red[((wave * NB + j) * 4 + q) * 64 + lane] = make_float4(acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]);
  __syncthreads();
  const StProblem &O = P.glu ? P.prob[0] : Q;
  // the NB * 4 (j, q) groups are shared out among the wavefronts
  for (int jq = wave; jq < NB * 4; jq += 4) {
    const int j = jq >> 2, q = jq & 3;
    float4 s0 = red[((0 * NB + j) * 4 + q) * 64 + lane];
    float4 s1 = red[((1 * NB + j) * 4 + q) * 64 + lane];
    float4 s2 = red[((2 * NB + j) * 4 + q) * 64 + lane];
    float4 s3 = red[((3 * NB + j) * 4 + q) * 64 + lane];
    float v[4];
    if (P.glu) {
      const float g[4] = {s0.x + s1.x, s0.y + s1.y, s0.z + s1.z, s0.w + s1.w};
      const float u[4] = {s2.x + s3.x, s2.y + s3.y, s2.z + s3.z, s2.w + s3.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = silu_f32(g[e]) * u[e];
    } else {
      v[0] = (s0.x + s1.x) + (s2.x + s3.x); v[1] = (s0.y + s1.y) + (s2.y + s3.y);
      v[2] = (s0.z + s1.z) + (s2.z + s3.z); v[3] = (s0.w + s1.w) + (s2.w + s3.w);
    }
    const int tok = 32 * j + (lane & 31);
    const int col = fblk * 32 + 8 * q + 4 * (lane >> 5);
    if (!P.glu && (P.bias != nullptr || P.act != ACT_NONE)) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        v[e] = act_f32(v[e] + ((P.bias != nullptr && col + e < O.width) ? cvt_in<DT>(P.bias[col + e]) : 0.f), P.act);
    }
    if (tok < P.T && col < O.width) {
      uint2 pk;
      pk.x = pack2<DT>(v[0], v[1]);
      pk.y = pack2<DT>(v[2], v[3]);
      uint16_t *dst = O.out + (long long)tok * O.ldo + col;
      if (col + 4 <= O.width && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
        *reinterpret_cast<uint2 *>(dst) = pk;
      } else {
        for (int e = 0; e < 4; ++e)
          if (col + e < O.width) dst[e] = (uint16_t)((e < 2 ? pk.x : pk.y) >> ((e & 1) * 16));
      }
      if (O.out2 && col < O.width2) {
        uint16_t *d2 = O.out2 + (long long)tok * O.ldo2 + col;
        for (int e = 0; e < 4; ++e)
          if (col + e < O.width2) d2[e] = (uint16_t)((e < 2 ? pk.x : pk.y) >> ((e & 1) * 16));
      }
    }
  }
#else
  (void)P;
#endif
}

}  // namespace deinfer
