// Host side of the C ABI declared in include/deinfer.h: argument validation (host only,
// before any device call), workspace carving, kernel selection and launch.
#include "../../include/deinfer.h"
#include "../../include/deinfer_testing.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <mutex>

#include "common.h"
#include "decode_kernel.h"
#include "generic_kernels.h"
#include "pack_kernels.h"
#include "prefill_kernel.h"
#include "skinny_kernel.h"
#include "skinny_glu_kernel.h"
#include "stream_kernel.h"
#include "probe_kernels.h"
#include "paged_kernels.h"

using namespace deinfer;

namespace {

thread_local char g_err[512] = "no error";
// Test and measurement aids (include/deinfer_testing.h): state of the calling thread only
thread_local int g_token_tile = 0;       // 0: chosen per launch; 128 or 256: forced; DEINFER_TOKEN_TILE_BOTH: two shapes in one launch
thread_local int g_feature_tile = 0;     // 0: chosen per launch; 128 or 256: forced where the token tile is 128
thread_local int g_glu_width = 0;        // deinfer_set_decode_glu_one_launch: 0 chosen per call; 1 forced; -1 never
thread_local int g_prof_kernel = 0;      // deinfer_set_profile_events: which internal launch to bracket
thread_local hipEvent_t g_prof_ev[2] = {nullptr, nullptr};

// Brackets one internal kernel launch with the caller's two events (measurement aid).
struct ProfScope {
  bool on; hipStream_t s;
  ProfScope(int kernel_id, hipStream_t s_) : on(g_prof_kernel == kernel_id && g_prof_ev[0] && g_prof_ev[1]), s(s_) {
    if (on) (void)hipEventRecord(g_prof_ev[0], s);
  }
  ~ProfScope() { if (on) (void)hipEventRecord(g_prof_ev[1], s); }
};

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_size(int dtype) { return dtype == DEINFER_F32 ? 4 : 2; }
static_assert(DT_BF16 == DEINFER_BF16 && DT_F16 == DEINFER_F16, "the kernels' storage-type codes are the boundary's dtype codes");
// Calls f with a value of the element type of `dtype` (float, uint16_t for bf16, f16_bits for fp16).
template <typename F>
int by_dtype(int dtype, F f) {
  if (dtype == DEINFER_F32) return f(float{});
  if (dtype == DEINFER_F16) return f(f16_bits{});
  return f(uint16_t{});
}
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- workspace layout -------------------------------------------------------------
// [0, 256)   status words (reserved; cleared by deinfer_workspace_init)
// [256, ...) scratch without invariants:
//            decode:  t [T16 x Rtot_pad] bf16, then DEC_MAX_PARTS part buffers [T16 x Rtot_pad] fp32
//            prefill: t [T x Rtot_pad] bf16
//            generic: t [T x Rtot] fp32
constexpr size_t WS_HEADER = 256;

// Calls of up to this many tokens take the memory-bound schedules (run_decode, run_skinny), longer
// ones the compute-bound one (run_prefill).
#ifndef DEINFER_SKINNY_MAX_T
#define DEINFER_SKINNY_MAX_T 128
#endif
constexpr int64_t SKINNY_MAX_T = DEINFER_SKINNY_MAX_T;
static_assert(SKINNY_MAX_T >= 16 && SKINNY_MAX_T <= 128, "the streaming kernels hold at most four 32-token blocks");

struct Geometry {          // derived sizes of one pair
  int64_t r_pad, KB1, KB2, n_rtiles, n_otiles;
  size_t u_bytes, v_bytes;
};
Geometry geometry(const deinfer_factors_t *f) {
  Geometry g;
  g.r_pad = round_up(f->r, 32);
  g.KB1 = ceil_div(f->d_in, 32);
  g.KB2 = g.r_pad / 32;
  g.n_rtiles = g.r_pad / 16;
  g.n_otiles = ceil_div(f->d_out, 16);
  g.u_bytes = (size_t)g.n_rtiles * g.KB1 * 1024;
  g.v_bytes = (size_t)g.n_otiles * g.KB2 * 1024;
  return g;
}

int device_cus() {
  static std::atomic<int> cached[64];       // (threads may race to fill an entry: they store the same value)
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  if (dev < 0 || dev >= 64) return -1;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return -1;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// ---- split of a memory-bound call with 16 < T <= 128 tokens
struct SkPlan {              // split of one call; a pure function of the shapes (also sizes the workspace)
  int NB;                    // 32-token blocks: 1, 2 or 4
  int NW[2];                 // wavefronts per workgroup = 32-feature blocks per feature group, stage 1 / stage 2
  int groups[2];             // feature groups of stage 1 / stage 2
  int P[2];                  // k-ranges of stage 1 / stage 2
  bool direct2;              // stage 2 has one k-range and no GLU: the streaming kernel stores the outputs itself
  int64_t rtot_pad;
  size_t t_bytes, part_bytes;
};

// A non-GLU second stage with at least this many 128-feature groups takes one k-range although two
// would fit: the streaming kernel then stores the outputs itself, and the saved reduce launch is worth
// more than the second half of the compute units (measured with 96 groups: 1-3 us per call faster;
// with 64-80 groups slower)
constexpr int SK_DIRECT_MIN_GROUPS = 96;
// Narrower feature groups are taken if they give at least this many percent of the workgroups of the
// wider split (105, 115 and 130 were timed: the lowest was best or equal on every block).
constexpr int SK_NARROW_GAIN_PCT = 105;

SkPlan skinny_plan(int64_t T, const deinfer_factors_t *const *f, int n, bool glu) {
  SkPlan pl;
  pl.NB = T <= 32 ? 1 : T <= 64 ? 2 : 4;
  pl.rtot_pad = 0;
  int64_t tiles[2][3] = {{0, 0, 0}, {0, 0, 0}};
  for (int i = 0; i < n; ++i) {
    const Geometry ge = geometry(f[i]);
    tiles[0][i] = ge.n_rtiles; tiles[1][i] = ge.n_otiles;
    pl.rtot_pad += ge.r_pad;
  }
  auto groups_of = [&](int s, int nw) {
    int g = 0;
    for (int i = 0; i < n; ++i) g += (int)ceil_div(tiles[s][i], (int64_t)(2 * nw));
    return g;
  };
  // About one long-lived workgroup per compute unit, and never a few more: two
  // workgroups fit a unit, so 258 of them on 256 units put two pairs on one unit each, and the launch
  // waits for those (traced: 15.4 us instead of 11.5 us for 86 groups x 3 ranges).  Hence the largest
  // number of k-ranges P with groups x P <= 256.
  // (the compute units of the current device; 256, the count of the device this is written for, where
  // no device can be asked: the host-only size query on a machine without a GPU)
  const int cus_now = device_cus();
  const int target = cus_now > 0 ? cus_now : 256;
  for (int s = 0; s < 2; ++s) {
    // more than 8 ranges only for a very long k (first stage of the second MLP layer of the largest
    // models): every range keeps at least 64 k-blocks (70B shapes, k = 28672, 20 groups: 12 ranges,
    // 70 -> 65 us at T = 128; the 7B shapes, k = 11008, were slower with more than 8)
    int cap = 8;
    if (s == 0) {
      const int by_k = (int)(ceil_div(f[0]->d_in, 32) / 64);
      cap = by_k > SK_MAX_PARTS ? SK_MAX_PARTS : by_k > 8 ? by_k : 8;
    }
    const int g4 = groups_of(s, 4);
    const bool direct = s == 1 && !glu && (g4 > target / 2 || g4 >= SK_DIRECT_MIN_GROUPS);
    if (direct) cap = 1;
    auto ranges = [&](int g) { const int p = target / (g > 0 ? g : 1); return p < 1 ? 1 : p > cap ? cap : p; };
    // Narrower feature groups (96 or 64 features: 3 or 2 wavefronts per workgroup) give more
    // workgroups without more k-ranges, i.e. without more partial sums, but one activation slab per
    // group and stage: taken where they fill clearly more of the device than the 128-feature split
    int nw = 4, g = g4, p = ranges(g4);
    for (int cand = 3; cand >= 2; --cand) {
      const int gc = groups_of(s, cand), pc = ranges(gc);
      if (gc * pc <= target && gc * pc * 100 >= g * p * SK_NARROW_GAIN_PCT) { nw = cand; g = gc; p = pc; }
    }
    pl.NW[s] = nw; pl.groups[s] = g; pl.P[s] = p;
    if (s == 1) pl.direct2 = direct;
  }
  pl.t_bytes = (size_t)round_up((int64_t)pl.NB * 32 * (pl.rtot_pad > 0 ? pl.rtot_pad : 32) * 2, 256);
  const size_t p0 = (size_t)pl.P[0] * pl.NB * 32 * (size_t)pl.groups[0] * (32 * pl.NW[0]) * 4;
  const size_t p1 = (size_t)pl.P[1] * pl.NB * 32 * (size_t)pl.groups[1] * (32 * pl.NW[1]) * 4;
  pl.part_bytes = (size_t)round_up((int64_t)(p0 > p1 ? p0 : p1), 256);
  return pl;
}

// ---- k-split of the first stage of a compute-bound call
// Stage 1 has a long k (d_in) and few features (the ranks), so its 256 x 256 tiles can be far fewer
// than the compute units (a few hundred tokens), or fill the last round of workgroups badly (160
// tiles of k = 28672 on 256 units: the second MLP layer of the 70B shapes at 4096 tokens).  The k
// range is then cut into parts (fp32 partial products, summed by the reduce kernel of the T <= 128
// path).  Stage 2 (short k, many features) is left whole: its partial products would cost more than
// they save.  The number of parts minimises an estimate of the launch time in units of one pipeline
// stage of one tile (about 0.7 us): rounds of workgroups x (stages + epilogue) + the reduce launch.
struct PfSplitPlan {
  int n_parts, kb_per_part, n_fblocks, n_tblocks;
  size_t part_bytes;          // 0: no split
};
PfSplitPlan prefill_split_plan(int64_t T, const deinfer_factors_t *const *f, int n) {
  PfSplitPlan pl;
  memset(&pl, 0, sizeof(pl));
  int64_t tiles = 0;
  for (int i = 0; i < n; ++i) tiles += geometry(f[i]).n_rtiles;
  const int64_t KB = ceil_div(f[0]->d_in, 32);
  pl.n_tblocks = (int)ceil_div(T, 256);
  pl.n_fblocks = (int)ceil_div(tiles, 16);
  pl.n_parts = 1; pl.kb_per_part = (int)KB;
  const int64_t wgs = (int64_t)pl.n_tblocks * pl.n_fblocks;
  if (wgs <= 0 || KB < 16) return pl;
  const int cus_now = device_cus();
  const int64_t cus = cus_now > 0 ? cus_now : 256;
  // measured on the device: epilogue of a tile that rounds and stores t (about 8 stages) or stores
  // its fp32 partial products (about 20: 256 KiB per workgroup, all units at once); a 128 x 256 tile
  // takes 0.64 of a 256 x 256 tile in the last round of a large launch and 0.78 in a launch of its own
  // (70B shapes, o-projection at 4096 tokens: 138 us unsplit against 106 + 18 us as two parts); the reduce launch reads its partial products at about 0.3 us per
  // MB (0.43 stages) after about 4 us (6 stages) of fixed cost
  constexpr double E_PLAIN = 8.0, E_PART = 20.0, SMALL_TILE = 0.64, SMALL_TILES_ONLY = 0.78, REDUCE_PER_MB = 0.43, REDUCE_FIXED = 6.0;
  auto rounds = [&](int64_t w, bool two_shapes) {
    const int64_t full = w / cus, tail = w % cus;
    if (tail == 0) return (double)full;
    if (two_shapes && full >= 1 && 2 * tail <= cus) return (double)full + SMALL_TILE;   // the last round as 128 x 256 tiles
    return (double)full + 1.0;
  };
  const double whole = (2 * wgs <= cus ? SMALL_TILES_ONLY : rounds(wgs, true)) * ((double)KB + E_PLAIN);
  const double part_mb = (double)pl.n_tblocks * 256.0 * (double)pl.n_fblocks * 256.0 * 4.0 / 1.0e6;
  const int64_t p_max = KB / 8 < SK_MAX_PARTS ? KB / 8 : SK_MAX_PARTS;     // at least 8 pipeline stages per part
  double best = 0.93 * whole;                                             // a split has to win by 7 %
  for (int64_t p = 2; p <= p_max; ++p) {
    const int64_t kbp = ceil_div(KB, p);
    if (ceil_div(KB, kbp) != p) continue;                                  // every part is non-empty
    const double est = rounds(wgs * p, false) * ((double)kbp + E_PART) + (double)p * part_mb * REDUCE_PER_MB + REDUCE_FIXED;
    if (est < best) { best = est; pl.n_parts = (int)p; pl.kb_per_part = (int)kbp; }
  }
  if (pl.n_parts > 1)
    pl.part_bytes = (size_t)pl.n_parts * pl.n_tblocks * 256 * (size_t)pl.n_fblocks * 256 * sizeof(float);
  return pl;
}

int validate_pair(const deinfer_factors_t *f, const char *name) {
  if (!f) return fail(DEINFER_ERR_INVALID_ARG, "%s: factor descriptor is NULL", name);
  if (f->d_in <= 0 || f->d_out <= 0 || f->r < 0)
    return fail(DEINFER_ERR_INVALID_ARG, "%s: bad sizes d_in=%lld d_out=%lld r=%lld", name,
                (long long)f->d_in, (long long)f->d_out, (long long)f->r);
  if (f->d_in > (1 << 30) || f->d_out > (1 << 30) || f->r > (1 << 30))
    return fail(DEINFER_ERR_INVALID_ARG, "%s: sizes above 2^30 are not supported", name);
  if (f->dtype != DEINFER_F32 && f->dtype != DEINFER_BF16 && f->dtype != DEINFER_F16)
    return fail(DEINFER_ERR_UNSUPPORTED, "%s: unknown dtype %d", name, f->dtype);
  if (f->layout != DEINFER_LAYOUT_RAW && f->layout != DEINFER_LAYOUT_PACKED)
    return fail(DEINFER_ERR_UNSUPPORTED, "%s: unknown layout %d", name, f->layout);
  if (f->r > 0 && (!f->U || !f->V)) return fail(DEINFER_ERR_INVALID_ARG, "%s: U or V is NULL", name);
  if (f->layout == DEINFER_LAYOUT_RAW) {
    if (f->r > 0 && (f->ldu < f->r || f->ldv < f->d_out))
      return fail(DEINFER_ERR_INVALID_ARG, "%s: leading dimension too small (ldu=%lld r=%lld ldv=%lld d_out=%lld)",
                  name, (long long)f->ldu, (long long)f->r, (long long)f->ldv, (long long)f->d_out);
    if (f->r > 0 && (!aligned(f->U, elem_size(f->dtype)) || !aligned(f->V, elem_size(f->dtype))))
      return fail(DEINFER_ERR_MISALIGNED, "%s: U / V not aligned to the element size", name);
  } else {
    if (f->dtype != DEINFER_BF16 && f->dtype != DEINFER_F16)
      return fail(DEINFER_ERR_UNSUPPORTED, "%s: the packed layout holds 16-bit types (bf16, fp16) only", name);
    if (f->r > 0 && (!aligned(f->U, 16) || !aligned(f->V, 16)))
      return fail(DEINFER_ERR_MISALIGNED, "%s: packed U / V must be 16-byte aligned", name);
  }
  return DEINFER_OK;
}

size_t workspace_need_of(int64_t T, const deinfer_factors_t *const *pairs, int n) {
  int64_t rtot = 0, rtot_pad = 0;
  for (int i = 0; i < n; ++i) { rtot += pairs[i]->r; rtot_pad += round_up(pairs[i]->r, 32); }
  const bool packed = pairs[0]->layout == DEINFER_LAYOUT_PACKED;
  size_t scratch;
  if (!packed) {
    scratch = (size_t)T * (size_t)(rtot > 0 ? rtot : 1) * sizeof(float);
  } else {
    const size_t rp = (size_t)(rtot_pad > 0 ? rtot_pad : 32);
    // T <= 16: t in fragment order and up to DEC_MAX_PARTS fp32 part buffers of one 16-token tile
    const size_t tdec = T <= 16 ? (size_t)round_up((int64_t)16 * rp * 2, 256) + (size_t)DEC_MAX_PARTS * 16 * rp * 4 : 0;
    size_t tpre = T > SKINNY_MAX_T ? (size_t)round_up(T, 256) * rp * 2 : 0;
    if (T > SKINNY_MAX_T) tpre = (size_t)round_up((int64_t)tpre, 256) + prefill_split_plan(T, pairs, n).part_bytes;
    scratch = round_up((int64_t)tdec, 256) + round_up((int64_t)tpre, 256);
    if (T <= SKINNY_MAX_T) { // (the upward-projection-only call uses this schedule for every such T)
      for (int glu = 0; glu < 2; ++glu) {      // (the call is not known here: room for either kind)
        const SkPlan pl = skinny_plan(T, pairs, n, glu != 0);
        const size_t sk = pl.t_bytes + pl.part_bytes;
        if (sk > scratch) scratch = sk;
      }
    }
  }
  return WS_HEADER + (size_t)round_up((int64_t)scratch, 256);
}

// Bytes that a call with these pairs may use.  Pairs of rank 0 are dropped before the dispatch (their
// outputs are zero-filled), and the remaining group may split differently (fewer feature groups admit
// more k-ranges, i.e. more partial sums): room for the group as given and for the group that runs.
size_t workspace_need(int64_t T, const deinfer_factors_t *const *pairs, int n) {
  size_t need = workspace_need_of(T, pairs, n);
  const deinfer_factors_t *rest[3];
  int m = 0;
  for (int i = 0; i < n && i < 3; ++i)
    if (pairs[i]->r > 0) rest[m++] = pairs[i];
  if (m > 0 && m < n) {
    const size_t reduced = workspace_need_of(T, rest, m);
    if (reduced > need) need = reduced;
  }
  return need;
}

int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(DEINFER_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
  return DEINFER_OK;
}

template <typename TC>
int zero_output(void *y, int64_t ldy, int64_t T, int64_t n, hipStream_t s) {
  const int64_t cnt = T * n;
  hipLaunchKernelGGL((zero2d_kernel<TC>), dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, s,
                     static_cast<TC *>(y), ldy, (int)T, (int)n);
  return check_launch("zero-fill");
}

// ---- one call = a group of 1..3 pairs that share x --------------------------------
struct Group {
  const void *x; int64_t T, ldx;
  int n;                                   // pairs
  const deinfer_factors_t *f[3];
  void *out[3]; int64_t ldo[3];            // per pair output (GLU: only [0])
  void *t_out[3]; int64_t ldt[3];          // optional rank-space outputs
  bool glu;
  bool up_only;                            // x is the rank-space intermediate t: only the upward projection runs
  bool rows_padded;                        // up_only: x (x2) already is the zero-padded copy in the workspace
  const void *bias; int act;               // single non-GLU pair only: y = act(product + bias), bias per output feature
  bool down_only;                          // only the downward projections run; every pair hands out its t through t_out
  const void *x2; int64_t ldx2;            // up_only GLU call: rank-space rows of the second (up) pair
  const float *rope; int64_t rope_dim;     // single up_only pair: rotary embedding of the output from a [T][rope_dim] cos | sin table
  void *ws; size_t ws_bytes; hipStream_t stream;
};

template <int DT, int NT>
int launch_decode_nt(const DecParams &P, bool glu, int grid2, hipStream_t s, bool down_only) {
  {
    ProfScope ps(DEINFER_PROF_DECODE_DOWN, s);
    hipLaunchKernelGGL((decode_kernel<DT, NT, false, 1>), dim3(P.G1), dim3(DEC_THREADS), 0, s, P);
  }
  if (int rc = check_launch("decode down kernel")) return rc;
  if (!P.direct1) {
    const int T16 = NT * 16;
    const long long n = (long long)T16 * (P.Rtot_pad / 4);
    {
      ProfScope ps(DEINFER_PROF_DECODE_REDUCE, s);
      hipLaunchKernelGGL(decode_reduce_kernel<DT>, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, P, T16);
    }
    if (int rc = check_launch("decode reduce kernel")) return rc;
  }
  if (down_only) return DEINFER_OK;
  {
    ProfScope ps(DEINFER_PROF_DECODE_UP, s);
    if (glu) hipLaunchKernelGGL((decode_kernel<DT, NT, true, 2>), dim3(grid2), dim3(DEC_THREADS), 0, s, P);
    else     hipLaunchKernelGGL((decode_kernel<DT, NT, false, 2>), dim3(grid2), dim3(DEC_THREADS), 0, s, P);
  }
  return check_launch("decode up kernel");
}

// Largest number of workgroups a single rank tile is spread over when `total` fragments
// (tiles of KB1) are cut into G1 equal ranges.
int max_parts(long long total, int KB1, int G1) {
  int worst = 1;
  const long long n_tiles = total / KB1;
  for (long long tile = 0; tile < n_tiles; ++tile) {
    const long long tbeg = tile * KB1, tend = tbeg + KB1;
    const int g_first = (int)(((tbeg + 1) * G1 + total - 1) / total) - 1;
    const int g_last = (int)((tend * G1 + total - 1) / total) - 1;
    if (g_last - g_first + 1 > worst) worst = g_last - g_first + 1;
  }
  return worst;
}

// Call of at most 16 tokens on packed pairs.
int run_decode(const Group &gq) {
  const int64_t T = gq.T;
  const int cus = device_cus();
  if (cus <= 0) return fail(DEINFER_ERR_DEVICE, "no usable HIP device");
  const int nt = 1;          // 16-token tiles
  char *ws = static_cast<char *>(gq.ws);
  DecParams P;
  memset(&P, 0, sizeof(P));
  P.x = static_cast<const uint16_t *>(gq.x);
  P.ldx = gq.ldx; P.T = (int)T; P.d_in = (int)gq.f[0]->d_in; P.KB1 = (int)ceil_div(gq.f[0]->d_in, 32);
  P.bias = static_cast<const uint16_t *>(gq.bias); P.act = gq.act;
  P.n_pairs = gq.n;
  int tile0 = 0, items = 0;
  for (int i = 0; i < gq.n; ++i) {
    const Geometry ge = geometry(gq.f[i]);
    DecPair &d = P.p[i];
    d.Up = static_cast<const uint4 *>(gq.f[i]->U);
    d.Vp = static_cast<const uint4 *>(gq.f[i]->V);
    d.y = static_cast<uint16_t *>(gq.out[i]);
    d.ldy = gq.ldo[i];
    d.t_out = static_cast<uint16_t *>(gq.t_out[i]);
    d.ldt_out = gq.ldt[i];
    d.r = (int)gq.f[i]->r; d.r_pad = (int)ge.r_pad; d.d_out = (int)gq.f[i]->d_out;
    d.n_otiles = (int)ge.n_otiles; d.tile0 = tile0;
    tile0 += (int)ge.n_rtiles;
    items += (int)ge.n_otiles;
  }
  P.n_rtiles = tile0;
  P.Rtot_pad = tile0 * 16;
  P.n_items2 = gq.glu ? P.p[0].n_otiles : items;
  const long long total = (long long)P.n_rtiles * P.KB1;
  if (total * (long long)(2 * cus + 1) >= (1ll << 31) || T * gq.ldx >= (1ll << 30) || (long long)nt * 16 * P.Rtot_pad >= (1ll << 30))
    return fail(DEINFER_ERR_UNSUPPORTED, "problem too large for the decode schedule (%lld fragments)", total);
  // (a workgroup alone on its compute unit streams at 25-45 GB/s: fewer tiles than units with a long k,
  // at least 8192, are faster as equal fragment ranges over twice the units plus the reduce launch;
  // measured on the second MLP layer's downward projection: 70B shapes 50 -> 41 us, 7B shapes 25 -> 23 us)
  const bool few_long = P.n_rtiles < cus && P.KB1 >= 256;
  if (P.n_rtiles >= cus / 4 && !few_long) {
    // enough rank tiles to keep the device streaming with one workgroup per tile: each sums the whole
    // k range of its tile and writes t itself, which saves the partial sums and the reduce launch
    P.G1 = P.n_rtiles;
    P.direct1 = 1;
  } else {
    // two workgroups per compute unit for the down kernel (one streams while the other reduces)
    int G1 = (int)(total < 2 * cus ? total : 2 * cus);
    while (G1 > 1 && max_parts(total, P.KB1, G1) > DEC_MAX_PARTS) G1 = G1 * 7 / 8;
    P.G1 = G1;
  }
  const size_t t_bytes = (size_t)round_up((int64_t)nt * 16 * P.Rtot_pad * 2, 256);
  if (WS_HEADER + t_bytes + (P.direct1 ? 0 : (size_t)DEC_MAX_PARTS * nt * 16 * P.Rtot_pad * 4) > gq.ws_bytes)
    return fail(DEINFER_ERR_WORKSPACE, "workspace too small for the decode schedule: %zu bytes given", gq.ws_bytes);
  P.t = reinterpret_cast<uint16_t *>(ws + WS_HEADER);
  P.part = reinterpret_cast<float *>(ws + WS_HEADER + t_bytes);
  P.part_stride = (long long)nt * 16 * P.Rtot_pad;
  const int grid2 = P.n_items2;     // one work item per workgroup
  // (the kernel is written for 1, 2, 4 or 8 token tiles; calls with more than 16 tokens take the
  // streaming kernels of skinny_host.inc, so only the one-tile form is instantiated)
  return gq.f[0]->dtype == DEINFER_F16 ? launch_decode_nt<DT_F16, 1>(P, gq.glu, grid2, gq.stream, gq.down_only)
                                      : launch_decode_nt<DT_BF16, 1>(P, gq.glu, grid2, gq.stream, gq.down_only);
}

template <typename TE>
int run_generic(const Group &gq) {
  const int64_t T = gq.T;
  int64_t rtot = 0;
  for (int i = 0; i < gq.n; ++i) rtot += gq.f[i]->r;
  float *t32 = reinterpret_cast<float *>(static_cast<char *>(gq.ws) + WS_HEADER);
  const int64_t ldt = rtot;
  const TE *x = static_cast<const TE *>(gq.x);
  int64_t off[3] = {0, 0, 0};
  int64_t acc = 0;
  for (int i = 0; i < gq.n; ++i) { off[i] = acc; acc += gq.f[i]->r; }
  if (gq.up_only && gq.glu) {
    const deinfer_factors_t *fg = gq.f[0], *fu = gq.f[1];
    dim3 grid((unsigned)ceil_div(fg->d_out, GT), (unsigned)ceil_div(T, GT));
    hipLaunchKernelGGL((gemm_generic_kernel<TE, TE, TE, true>), grid, dim3(GTHREADS), 0, gq.stream,
                       x, gq.ldx, static_cast<const TE *>(fg->V), fg->ldv, (int)fg->r,
                       static_cast<const TE *>(gq.x2), gq.ldx2, static_cast<const TE *>(fu->V), fu->ldv, (int)fu->r,
                       static_cast<TE *>(gq.out[0]), gq.ldo[0], (int)T, (int)fg->d_out);
    return check_launch("generic GLU upward projection");
  }
  if (gq.up_only) {
    // the caller's rank-space rows are the activation operand of the upward projection
    const deinfer_factors_t *f = gq.f[0];
    dim3 grid((unsigned)ceil_div(f->d_out, GT), (unsigned)ceil_div(T, GT));
    hipLaunchKernelGGL((gemm_generic_kernel<TE, TE, TE, false>), grid, dim3(GTHREADS), 0, gq.stream,
                       x, gq.ldx, static_cast<const TE *>(f->V), f->ldv, (int)f->r,
                       (const TE *)nullptr, (int64_t)0, (const TE *)nullptr, (int64_t)0, 0,
                       static_cast<TE *>(gq.out[0]), gq.ldo[0], (int)T, (int)f->d_out);
    return check_launch("generic upward projection");
  }
  // stage 1: t[:, off_i : off_i + r_i] = x . U_i   (downward projections, Sec. 4.1)
  for (int i = 0; i < gq.n; ++i) {
    const deinfer_factors_t *f = gq.f[i];
    dim3 grid((unsigned)ceil_div(f->r, GT), (unsigned)ceil_div(T, GT));
    hipLaunchKernelGGL((gemm_generic_kernel<TE, TE, float, false>), grid, dim3(GTHREADS), 0, gq.stream,
                       x, gq.ldx, static_cast<const TE *>(f->U), f->ldu, (int)f->d_in,
                       (const TE *)nullptr, (int64_t)0, (const TE *)nullptr, (int64_t)0, 0,
                       t32 + off[i], ldt, (int)T, (int)f->r);
    if (int rc = check_launch("generic stage 1")) return rc;
    if (gq.t_out[i]) {
      const int64_t cnt = T * f->r;
      hipLaunchKernelGGL((copy2d_kernel<float, TE>), dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, gq.stream,
                         t32 + off[i], ldt, static_cast<TE *>(gq.t_out[i]), gq.ldt[i], (int)T, (int)f->r);
      if (int rc = check_launch("rank-space copy")) return rc;
    }
  }
  if (gq.down_only) return DEINFER_OK;
  // stage 2: upward projections
  if (gq.glu) {
    const deinfer_factors_t *fg = gq.f[0], *fu = gq.f[1];
    dim3 grid((unsigned)ceil_div(fg->d_out, GT), (unsigned)ceil_div(T, GT));
    hipLaunchKernelGGL((gemm_generic_kernel<float, TE, TE, true>), grid, dim3(GTHREADS), 0, gq.stream,
                       t32 + off[0], ldt, static_cast<const TE *>(fg->V), fg->ldv, (int)fg->r,
                       t32 + off[1], ldt, static_cast<const TE *>(fu->V), fu->ldv, (int)fu->r,
                       static_cast<TE *>(gq.out[0]), gq.ldo[0], (int)T, (int)fg->d_out);
    return check_launch("generic GLU stage 2");
  }
  for (int i = 0; i < gq.n; ++i) {
    const deinfer_factors_t *f = gq.f[i];
    dim3 grid((unsigned)ceil_div(f->d_out, GT), (unsigned)ceil_div(T, GT));
    hipLaunchKernelGGL((gemm_generic_kernel<float, TE, TE, false>), grid, dim3(GTHREADS), 0, gq.stream,
                       t32 + off[i], ldt, static_cast<const TE *>(f->V), f->ldv, (int)f->r,
                       (const float *)nullptr, (int64_t)0, (const TE *)nullptr, (int64_t)0, 0,
                       static_cast<TE *>(gq.out[i]), gq.ldo[i], (int)T, (int)f->d_out,
                       static_cast<const TE *>(gq.bias), gq.act);
    if (int rc = check_launch("generic stage 2")) return rc;
  }
  return DEINFER_OK;
}

// The compute-bound path (T > 128) lives in its own file; it uses Group and the helpers above.
#include "skinny_host.inc"
#include "prefill_host.inc"

int run_group(Group gq) {
  // ---- validation (host only)
  if (gq.T < 0) return fail(DEINFER_ERR_INVALID_ARG, "T is negative");
  for (int i = 0; i < gq.n; ++i) {
    static const char *names[3] = {"pair 0", "pair 1", "pair 2"};
    if (int rc = validate_pair(gq.f[i], names[i])) return rc;
    if (gq.f[i]->d_in != gq.f[0]->d_in || gq.f[i]->dtype != gq.f[0]->dtype || gq.f[i]->layout != gq.f[0]->layout)
      return fail(DEINFER_ERR_INVALID_ARG, "pairs of one call must share d_in, dtype and layout");
  }
  if (gq.glu && gq.f[0]->d_out != gq.f[1]->d_out)
    return fail(DEINFER_ERR_INVALID_ARG, "gate and up must have the same output width");
  if (gq.T == 0) return DEINFER_OK;
  const int dtype = gq.f[0]->dtype;
  const size_t es = elem_size(dtype);
  if (!gq.x) return fail(DEINFER_ERR_INVALID_ARG, "activation pointer is NULL");
  if (gq.up_only) {
    if (gq.ldx < gq.f[0]->r) return fail(DEINFER_ERR_INVALID_ARG, "ldt smaller than r");
    if (gq.glu) {
      if (!gq.x2) return fail(DEINFER_ERR_INVALID_ARG, "rank-space pointer of the up pair is NULL");
      if (gq.ldx2 < gq.f[1]->r) return fail(DEINFER_ERR_INVALID_ARG, "ldt of the up pair smaller than r");
      if (!aligned(gq.x2, es)) return fail(DEINFER_ERR_MISALIGNED, "rank-space pointer of the up pair not aligned to the element size");
    }
  } else if (gq.ldx < gq.f[0]->d_in) {
    return fail(DEINFER_ERR_INVALID_ARG, "ldx smaller than d_in");
  }
  if (!aligned(gq.x, es)) return fail(DEINFER_ERR_MISALIGNED, "activation pointer not aligned to the element size");
  const int n_out = gq.down_only ? 0 : gq.glu ? 1 : gq.n;
  if (gq.down_only)
    for (int i = 0; i < gq.n; ++i)
      if (!gq.t_out[i] && gq.f[i]->r > 0) return fail(DEINFER_ERR_INVALID_ARG, "rank-space output %d is NULL", i);
  for (int i = 0; i < n_out; ++i) {
    if (!gq.out[i]) return fail(DEINFER_ERR_INVALID_ARG, "output pointer %d is NULL", i);
    if (gq.ldo[i] < gq.f[i]->d_out) return fail(DEINFER_ERR_INVALID_ARG, "output %d: leading dimension smaller than d_out", i);
    if (!aligned(gq.out[i], es)) return fail(DEINFER_ERR_MISALIGNED, "output %d not aligned to the element size", i);
  }
  for (int i = 0; i < gq.n; ++i)
    if (gq.t_out[i]) {
      if (gq.ldt[i] < gq.f[i]->r) return fail(DEINFER_ERR_INVALID_ARG, "rank-space output %d: leading dimension smaller than r", i);
      if (!aligned(gq.t_out[i], es)) return fail(DEINFER_ERR_MISALIGNED, "rank-space output %d misaligned", i);
    }
  if (!gq.ws) return fail(DEINFER_ERR_WORKSPACE, "workspace pointer is NULL");
  if (!aligned(gq.ws, 256)) return fail(DEINFER_ERR_MISALIGNED, "workspace must be 256-byte aligned");
  const size_t need = workspace_need(gq.T, gq.f, gq.n);
  if (gq.ws_bytes < need)
    return fail(DEINFER_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", gq.ws_bytes, need);
  const bool packed = gq.f[0]->layout == DEINFER_LAYOUT_PACKED;
  if (packed && gq.up_only) {
    // The packed kernels read the activation operand in 16-byte chunks of 8 columns; the chunk that
    // holds column r - 1 of a rank that is no multiple of 8 reaches past the caller's valid columns
    // (the weights there are zero, but 0 x NaN is NaN).  The kernels set those elements to zero once
    // the chunk is in LDS (lds_zero_chunk_tail), so 16-byte aligned rows with a pitch of whole chunks
    // are read in place (r >= 8).  Any other rows are first copied into the workspace, where a full
    // call keeps its own rank-space intermediate, with zeros in the padding columns: one small launch more.
    bool repack = false;
    for (int i = 0; i < gq.n && !gq.rows_padded; ++i) {
      const void *xi = i == 1 ? gq.x2 : gq.x;
      const int64_t ld = i == 1 ? gq.ldx2 : gq.ldx;
      const int64_t r = gq.f[i]->r;
      if (!aligned(xi, 16) || ld % 8 != 0 || (r % 8 != 0 && r < 8)) repack = true;
    }
    if (repack) {
      int64_t pitch = 0, col[3] = {0, 0, 0};
      for (int i = 0; i < gq.n; ++i) { col[i] = pitch; pitch += round_up(gq.f[i]->r, 32); }
      // (T rows of `pitch` columns fit the region of the intermediate of either schedule: it has at
      // least T rows of the 32-padded ranks; the bound is checked, not assumed)
      if (WS_HEADER + (size_t)gq.T * (size_t)pitch * 2 > gq.ws_bytes || gq.T * pitch >= (1ll << 30))
        return fail(DEINFER_ERR_WORKSPACE, "workspace too small for the padded copy of the rank-space rows");
      uint16_t *t = reinterpret_cast<uint16_t *>(static_cast<char *>(gq.ws) + WS_HEADER);
      for (int i = 0; i < gq.n; ++i) {
        const int64_t width = round_up(gq.f[i]->r, 32);
        if (width == 0) continue;
        const int64_t cnt = gq.T * (width / 8);
        const void *xi = i == 1 ? gq.x2 : gq.x;
        const int64_t ld = i == 1 ? gq.ldx2 : gq.ldx;
        hipLaunchKernelGGL(pad_rows16_kernel, dim3((unsigned)ceil_div(cnt, (int64_t)256)), dim3(256), 0, gq.stream,
                           static_cast<const uint16_t *>(xi), ld, t + col[i], pitch, (int)gq.T, (int)gq.f[i]->r, (int)width,
                           (aligned(xi, 16) && ld % 8 == 0) ? 1 : 0);
        if (int rc = check_launch("padded copy of the rank-space rows")) return rc;
      }
      gq.x = t; gq.ldx = pitch;
      if (gq.n > 1) { gq.x2 = t + col[1]; gq.ldx2 = pitch; }
      gq.rows_padded = true;
    }
  } else if (packed) {
    if (!aligned(gq.x, 16) || gq.ldx % 8 != 0 || gq.f[0]->d_in % 8 != 0)
      return fail(DEINFER_ERR_MISALIGNED,
                  "packed pairs need 16-byte aligned activations, ldx %% 8 == 0 and d_in %% 8 == 0");
  }

  // ---- bias / activation of the non-GLU sub-layer: single pair only
  if (gq.bias != nullptr || gq.act != ACT_NONE) {
    if (gq.n != 1 || gq.glu || gq.up_only) return fail(DEINFER_ERR_INVALID_ARG, "bias and activation go with a single pair");
    if (gq.act != ACT_NONE && gq.act != ACT_RELU && gq.act != ACT_GELU) return fail(DEINFER_ERR_UNSUPPORTED, "unknown activation %d", gq.act);
    if (gq.bias && !aligned(gq.bias, packed ? 16 : es))
      return fail(DEINFER_ERR_MISALIGNED, packed ? "packed pairs need a 16-byte aligned bias" : "bias not aligned to the element size");
    if (gq.f[0]->r == 0) {       // empty product: y = act(bias)
      const int64_t cnt = gq.T * gq.f[0]->d_out;
      if (cnt == 0) return DEINFER_OK;
      by_dtype(dtype, [&](auto tag) {
        using TE = decltype(tag);
        hipLaunchKernelGGL((bias_act_fill_kernel<TE>), dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, gq.stream,
                           static_cast<TE *>(gq.out[0]), gq.ldo[0], (int)gq.T, (int)gq.f[0]->d_out,
                           static_cast<const TE *>(gq.bias), gq.act);
        return 0;
      });
      return check_launch("bias / activation fill");
    }
  }

  // ---- pairs of rank 0: the output is exactly zero (empty sum)
  bool any_zero = false;
  for (int i = 0; i < gq.n; ++i) any_zero |= (gq.f[i]->r == 0);
  if (any_zero && gq.down_only) {          // a pair of rank 0 has no rank-space columns: drop it
    Group rest = gq;
    rest.n = 0;
    for (int i = 0; i < gq.n; ++i)
      if (gq.f[i]->r != 0) {
        rest.f[rest.n] = gq.f[i]; rest.t_out[rest.n] = gq.t_out[i]; rest.ldt[rest.n] = gq.ldt[i];
        ++rest.n;
      }
    if (rest.n == 0) return DEINFER_OK;
    gq = rest;
  } else if (any_zero) {
    if (gq.glu) {   // silu(0) * u == 0 and silu(g) * 0 == 0
      return by_dtype(dtype, [&](auto tag) { return zero_output<decltype(tag)>(gq.out[0], gq.ldo[0], gq.T, gq.f[0]->d_out, gq.stream); });
    }
    Group rest = gq;
    rest.n = 0;
    for (int i = 0; i < gq.n; ++i) {
      if (gq.f[i]->r == 0) {
        int rc = by_dtype(dtype, [&](auto tag) { return zero_output<decltype(tag)>(gq.out[i], gq.ldo[i], gq.T, gq.f[i]->d_out, gq.stream); });
        if (rc) return rc;
      } else {
        rest.f[rest.n] = gq.f[i]; rest.out[rest.n] = gq.out[i]; rest.ldo[rest.n] = gq.ldo[i];
        rest.t_out[rest.n] = gq.t_out[i]; rest.ldt[rest.n] = gq.ldt[i];
        ++rest.n;
      }
    }
    if (rest.n == 0) return DEINFER_OK;
    gq = rest;
  }

  // ---- dispatch
  if (gq.rope != nullptr) {
    // the large-T kernel rotates in its epilogue when one wavefront's 128 features are one head and
    // its 16-byte stores apply; otherwise the product is written first and rotated in place
    const bool fused = packed && gq.T > SKINNY_MAX_T && gq.rope_dim == 128 && gq.f[0]->d_out % 128 == 0 &&
                       aligned(gq.out[0], 16) && gq.ldo[0] % 8 == 0;
    if (!fused) {
      Group plain = gq;
      plain.rope = nullptr;
      if (int rc = run_group(plain)) return rc;
      const int64_t n = gq.T * gq.f[0]->d_out / 2;
      if (ceil_div(n, (int64_t)256) > INT32_MAX) return fail(DEINFER_ERR_UNSUPPORTED, "up + rope: output too large");
      by_dtype(dtype, [&](auto tag) {
        using TE = decltype(tag);
        hipLaunchKernelGGL((rope_from_table_kernel<TE>), dim3((unsigned)ceil_div(n, (int64_t)256)), dim3(256), 0, gq.stream,
                           static_cast<TE *>(gq.out[0]), (long long)gq.T, (long long)gq.ldo[0],
                           (int)(gq.f[0]->d_out / gq.rope_dim), (int)gq.rope_dim, gq.rope);
        return 0;
      });
      return check_launch("rotary embedding from the table");
    }
  }
  if (!packed) return by_dtype(dtype, [&](auto tag) { return run_generic<decltype(tag)>(gq); });
  if (gq.T <= 16 && !gq.up_only) {
    // The kernels of run_decode (one workgroup per 16-feature tile, two launches per call) against the
    // streaming kernels of run_skinny (feature groups x k-ranges, three or four launches): the former
    // win for the smaller calls of at most 8 tokens; they lose where their tiles do not fit the device
    // evenly (more rank tiles than compute units: the units that get two take twice as long) or where
    // the second stage has thousands of tiles, and everywhere from 9 tokens on.  Measured per call on
    // 7B-, 70B- and OPT-30B-shaped blocks at 1, 8 and 16 tokens.
    int64_t rtiles = 0, otiles = 0;
    for (int i = 0; i < gq.n; ++i) { const Geometry ge = geometry(gq.f[i]); rtiles += ge.n_rtiles; otiles += ge.n_otiles; }
    const int cus = device_cus();
    if (cus <= 0) return fail(DEINFER_ERR_DEVICE, "no usable HIP device");
    if (gq.T <= 8 && rtiles <= cus && otiles <= 4 * cus) return run_decode(gq);
  }
  if (gq.T <= SKINNY_MAX_T) return run_skinny(gq);
  return run_prefill(gq);
}

}  // namespace

extern "C" {

const char *deinfer_last_error(void) { return g_err; }

int deinfer_version(void) { return 1000; }

int deinfer_set_profile_events(int which, void *start_event, void *stop_event) {
  if (which < 0 || which > DEINFER_PROF_PREFILL_UP) return fail(DEINFER_ERR_INVALID_ARG, "unknown launch id %d", which);
  g_prof_kernel = (start_event && stop_event) ? which : 0;
  g_prof_ev[0] = static_cast<hipEvent_t>(start_event);
  g_prof_ev[1] = static_cast<hipEvent_t>(stop_event);
  return DEINFER_OK;
}

int deinfer_set_prefill_token_tile(int tokens) {
  if (tokens != 0 && tokens != 128 && tokens != 256 && tokens != DEINFER_TOKEN_TILE_BOTH)
    return fail(DEINFER_ERR_INVALID_ARG, "token tile: 0, 128, 256 or DEINFER_TOKEN_TILE_BOTH (both shapes in one launch), got %d", tokens);
  g_token_tile = tokens;
  return DEINFER_OK;
}

int deinfer_set_decode_glu_one_launch(int mode) {
  if (mode != 0 && mode != 1 && mode != -1) return fail(DEINFER_ERR_INVALID_ARG, "GLU second stage: 0, 1 or -1, got %d", mode);
  g_glu_width = mode;
  return DEINFER_OK;
}

int deinfer_set_prefill_feature_tile(int features) {
  if (features != 0 && features != 128 && features != 256) return fail(DEINFER_ERR_INVALID_ARG, "feature tile: 0, 128 or 256, got %d", features);
  g_feature_tile = features;
  return DEINFER_OK;
}

int deinfer_probe_stream_read(const void *buf, size_t bytes, void *sink, size_t sink_bytes, void *stream) {
  if (!buf || !sink) return fail(DEINFER_ERR_INVALID_ARG, "probe: buffer or sink is NULL");
  if (!aligned(buf, 16) || !aligned(sink, 16)) return fail(DEINFER_ERR_MISALIGNED, "probe: buffer and sink must be 16-byte aligned");
  if (bytes < 1024 || bytes % 1024 != 0) return fail(DEINFER_ERR_INVALID_ARG, "probe: bytes must be a positive multiple of 1024");
  if (sink_bytes < DEINFER_PROBE_SINK_BYTES) return fail(DEINFER_ERR_WORKSPACE, "probe: sink smaller than DEINFER_PROBE_SINK_BYTES");
  const int cus = device_cus();
  if (cus <= 0) return fail(DEINFER_ERR_DEVICE, "cannot query the device");
  const size_t n_kb = bytes / 1024;
  const unsigned grid = (unsigned)(n_kb < (size_t)cus ? n_kb : (size_t)cus);
  hipLaunchKernelGGL(probe_stream_read_kernel, dim3(grid), dim3(PROBE_READ_THREADS), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4_t *>(buf), n_kb, static_cast<u32x4_t *>(sink));
  return check_launch("stream-read probe");
}

int deinfer_probe_mfma_bf16(const void *operands, size_t operand_bytes, int64_t n_rounds, void *sink, size_t sink_bytes,
                            void *stream, double *flops_out) {
  if (!operands || !sink) return fail(DEINFER_ERR_INVALID_ARG, "probe: operands or sink is NULL");
  if (!aligned(operands, 16) || !aligned(sink, 16)) return fail(DEINFER_ERR_MISALIGNED, "probe: operands and sink must be 16-byte aligned");
  if (operand_bytes < (size_t)PROBE_MFMA_THREADS * 32) return fail(DEINFER_ERR_INVALID_ARG, "probe: operands must hold 8192 bytes");
  if (n_rounds <= 0 || n_rounds > (1 << 24)) return fail(DEINFER_ERR_INVALID_ARG, "probe: n_rounds out of range");
  const int cus = device_cus();
  if (cus <= 0) return fail(DEINFER_ERR_DEVICE, "cannot query the device");
  if (sink_bytes < DEINFER_PROBE_SINK_BYTES || (size_t)cus * PROBE_MFMA_THREADS * sizeof(float) > sink_bytes)
    return fail(DEINFER_ERR_WORKSPACE, "probe: sink smaller than DEINFER_PROBE_SINK_BYTES");
  hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3((unsigned)cus), dim3(PROBE_MFMA_THREADS), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4_t *>(operands), (int)n_rounds, static_cast<float *>(sink));
  if (flops_out)      // 32 x 32 x 16 multiply-adds per product
    *flops_out = 2.0 * 32 * 32 * 16 * (double)PROBE_MFMA_ACC * (double)n_rounds * (PROBE_MFMA_THREADS / 64) * (double)cus;
  return check_launch("MFMA probe");
}

int deinfer_kv_compact_plan(const int32_t *block_table, int64_t n_seqs, int64_t table_pitch, const int32_t *n_blocks,
                            int64_t n_pool_blocks, int64_t buffer_blocks, int64_t block_tokens,
                            int32_t *plan, int64_t plan_capacity_runs, int32_t *remap, int64_t remap_pitch,
                            int32_t *positions) {
  if (n_seqs < 0 || table_pitch < 0 || n_pool_blocks < 0 || buffer_blocks < 0 || plan_capacity_runs < 0)
    return fail(DEINFER_ERR_INVALID_ARG, "kv plan: negative size");
  if (!plan) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: plan is NULL");
  if (n_seqs > 0 && (!block_table || !n_blocks)) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: block table or block counts are NULL");
  if (n_pool_blocks > INT32_MAX || buffer_blocks > INT32_MAX || plan_capacity_runs > (INT32_MAX - KV_PLAN_HEADER) / 3)
    return fail(DEINFER_ERR_INVALID_ARG, "kv plan: sizes above 2^31 are not supported");
  if (positions && block_tokens <= 0) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: block_tokens must be positive when positions are asked for");
  if (positions && buffer_blocks * block_tokens > INT32_MAX) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: too many token slots");
  int64_t n_runs = 0, d = 0;
  int64_t run_src = 0, run_len = 0;          // the open run; its destination is d - run_len
  for (int64_t s = 0; s < n_seqs; ++s) {
    const int64_t nb = n_blocks[s];
    if (nb < 0 || nb > table_pitch) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: sequence %lld has %lld blocks, the table holds %lld per sequence", (long long)s, (long long)nb, (long long)table_pitch);
    if (remap && nb > remap_pitch) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: sequence %lld has %lld blocks, the remapping list holds %lld per sequence", (long long)s, (long long)nb, (long long)remap_pitch);
    for (int64_t i = 0; i < nb; ++i) {
      const int64_t p = block_table[s * table_pitch + i];
      if (p < 0 || p >= n_pool_blocks) return fail(DEINFER_ERR_INVALID_ARG, "kv plan: sequence %lld block %lld names physical block %lld outside the pool of %lld", (long long)s, (long long)i, (long long)p, (long long)n_pool_blocks);
      if (d >= buffer_blocks) return fail(DEINFER_ERR_WORKSPACE, "kv plan: the sequences hold more than the %lld blocks of the compact buffer", (long long)buffer_blocks);
      if (run_len > 0 && run_src + run_len == p) {
        ++run_len;                              // physically contiguous with the block before it in the walk
      } else {
        if (run_len > 0) {
          if (n_runs >= plan_capacity_runs) return fail(DEINFER_ERR_WORKSPACE, "kv plan: more than %lld runs", (long long)plan_capacity_runs);
          int32_t *r = plan + KV_PLAN_HEADER + 3 * n_runs++;
          r[0] = (int32_t)run_src; r[1] = (int32_t)(d - run_len); r[2] = (int32_t)run_len;
        }
        run_src = p; run_len = 1;
      }
      if (remap) remap[s * remap_pitch + i] = (int32_t)d;
      if (positions)
        for (int64_t j = 0; j < block_tokens; ++j) positions[d * block_tokens + j] = (int32_t)(i * block_tokens + j);
      ++d;
    }
    if (remap) for (int64_t i = nb; i < remap_pitch; ++i) remap[s * remap_pitch + i] = -1;
  }
  if (run_len > 0) {
    if (n_runs >= plan_capacity_runs) return fail(DEINFER_ERR_WORKSPACE, "kv plan: more than %lld runs", (long long)plan_capacity_runs);
    int32_t *r = plan + KV_PLAN_HEADER + 3 * n_runs++;
    r[0] = (int32_t)run_src; r[1] = (int32_t)(d - run_len); r[2] = (int32_t)run_len;
  }
  if (positions)
    for (int64_t j = d * block_tokens; j < buffer_blocks * block_tokens; ++j) positions[j] = 0;
  plan[0] = (int32_t)n_runs; plan[1] = (int32_t)d; plan[2] = 0; plan[3] = 0;
  return DEINFER_OK;
}

int deinfer_kv_compact_copy(const void *pool, int64_t n_pool_blocks, int64_t block_bytes, const int32_t *plan,
                            int64_t plan_capacity_runs, void *buffer, int64_t buffer_blocks, void *stream) {
  if (n_pool_blocks < 0 || buffer_blocks < 0 || plan_capacity_runs < 0 || block_bytes <= 0)
    return fail(DEINFER_ERR_INVALID_ARG, "kv copy: bad size");
  if (block_bytes % 16 != 0) return fail(DEINFER_ERR_MISALIGNED, "kv copy: block_bytes must be a multiple of 16");
  if (n_pool_blocks > INT32_MAX || buffer_blocks > INT32_MAX || plan_capacity_runs > (INT32_MAX - KV_PLAN_HEADER) / 3)
    return fail(DEINFER_ERR_INVALID_ARG, "kv copy: sizes above 2^31 are not supported");
  if (buffer_blocks == 0 || plan_capacity_runs == 0) return DEINFER_OK;
  if (!pool || !plan || !buffer) return fail(DEINFER_ERR_INVALID_ARG, "kv copy: pool, plan or buffer is NULL");
  if (!aligned(pool, 16) || !aligned(buffer, 16) || !aligned(plan, 4))
    return fail(DEINFER_ERR_MISALIGNED, "kv copy: pool and buffer must be 16-byte aligned");
  // the grid depends on capacities only: a captured launch serves every later plan
  const int64_t pieces = buffer_blocks * ceil_div(block_bytes, (int64_t)KV_PIECE);
  const unsigned grid = (unsigned)(pieces < 4096 ? pieces : 4096);
  hipLaunchKernelGGL(kv_compact_copy_kernel, dim3(grid), dim3(KV_COPY_THREADS), 0, static_cast<hipStream_t>(stream),
                     static_cast<const unsigned char *>(pool), (long long)n_pool_blocks, (long long)block_bytes, plan,
                     (int)plan_capacity_runs, static_cast<unsigned char *>(buffer), (long long)buffer_blocks);
  return check_launch("kv compact copy");
}

int deinfer_rope_inplace(void *x, int64_t T, int64_t ldx, int64_t n_heads, int64_t head_dim, const int32_t *positions,
                         double theta, int dtype, void *stream) {
  if (T < 0 || n_heads <= 0 || head_dim <= 0 || head_dim % 2 != 0)
    return fail(DEINFER_ERR_INVALID_ARG, "rope: T >= 0, n_heads > 0 and an even head_dim > 0 are required");
  if (dtype != DEINFER_F32 && dtype != DEINFER_BF16 && dtype != DEINFER_F16) return fail(DEINFER_ERR_UNSUPPORTED, "rope: unknown dtype %d", dtype);
  if (!(theta > 0.0)) return fail(DEINFER_ERR_INVALID_ARG, "rope: theta must be positive");
  if (n_heads > (1 << 20) || head_dim > (1 << 20) || ldx < n_heads * head_dim)
    return fail(DEINFER_ERR_INVALID_ARG, "rope: ldx smaller than n_heads * head_dim, or sizes out of range");
  if (T == 0) return DEINFER_OK;
  if (!x || !positions) return fail(DEINFER_ERR_INVALID_ARG, "rope: x or positions is NULL");
  if (!aligned(x, elem_size(dtype)) || !aligned(positions, 4)) return fail(DEINFER_ERR_MISALIGNED, "rope: x not aligned to its element size");
  const int64_t chunks = ceil_div(head_dim / 2, (int64_t)8);
  const int64_t n = T * chunks;
  if (ceil_div(n, (int64_t)256) > INT32_MAX) return fail(DEINFER_ERR_UNSUPPORTED, "rope: too many tokens");
  const dim3 grid((unsigned)ceil_div(n, (int64_t)256));
  hipStream_t s = static_cast<hipStream_t>(stream);
  by_dtype(dtype, [&](auto tag) {
    using TE = decltype(tag);
    hipLaunchKernelGGL((rope_inplace_kernel<TE>), grid, dim3(256), 0, s, static_cast<TE *>(x), (long long)T,
                       (long long)ldx, (int)n_heads, (int)head_dim, positions, log2(theta));
    return 0;
  });
  return check_launch("rope");
}

int deinfer_rank_for_ratio(int64_t m, int64_t n, double param_reduction, int64_t *r_out) {
  if (!r_out) return fail(DEINFER_ERR_INVALID_ARG, "r_out is NULL");
  if (m <= 0 || n <= 0) return fail(DEINFER_ERR_INVALID_ARG, "m and n must be positive");
  if (!(param_reduction >= 0.0 && param_reduction <= 1.0))
    return fail(DEINFER_ERR_INVALID_ARG, "param_reduction must lie in [0, 1]");
  const long long keep_ppm = llround((1.0 - param_reduction) * 1.0e6);
  const __int128 num = (__int128)keep_ppm * (__int128)m * (__int128)n;
  const __int128 den = (__int128)1000000 * ((__int128)m + (__int128)n);
  *r_out = (int64_t)(num / den);
  return DEINFER_OK;
}

int deinfer_packed_bytes(const deinfer_factors_t *raw, size_t *bytes) {
  if (!bytes) return fail(DEINFER_ERR_INVALID_ARG, "bytes is NULL");
  if (!raw) return fail(DEINFER_ERR_INVALID_ARG, "raw descriptor is NULL");
  if (raw->d_in <= 0 || raw->d_out <= 0 || raw->r < 0) return fail(DEINFER_ERR_INVALID_ARG, "bad sizes");
  const Geometry g = geometry(raw);
  *bytes = (size_t)round_up((int64_t)g.u_bytes, 256) + (size_t)round_up((int64_t)g.v_bytes, 256);
  return DEINFER_OK;
}

int deinfer_pack_factors(const deinfer_factors_t *raw, void *dst, size_t dst_bytes,
                         deinfer_factors_t *packed, void *stream) {
  if (int rc = validate_pair(raw, "raw")) return rc;
  if (!packed) return fail(DEINFER_ERR_INVALID_ARG, "packed descriptor is NULL");
  if (raw->layout != DEINFER_LAYOUT_RAW) return fail(DEINFER_ERR_INVALID_ARG, "source pair is not in RAW layout");
  if (raw->dtype != DEINFER_BF16 && raw->dtype != DEINFER_F16)
    return fail(DEINFER_ERR_UNSUPPORTED, "only pairs of a 16-bit type (bf16, fp16) can be packed");
  size_t need = 0;
  deinfer_packed_bytes(raw, &need);
  if (need > 0 && !dst) return fail(DEINFER_ERR_INVALID_ARG, "dst is NULL");
  if (!aligned(dst, 256)) return fail(DEINFER_ERR_MISALIGNED, "dst must be 256-byte aligned");
  if (dst_bytes < need) return fail(DEINFER_ERR_WORKSPACE, "dst too small: %zu bytes given, %zu needed", dst_bytes, need);
  const Geometry g = geometry(raw);
  hipStream_t s = static_cast<hipStream_t>(stream);
  char *d = static_cast<char *>(dst);
  uint4 *du = reinterpret_cast<uint4 *>(d);
  uint4 *dv = reinterpret_cast<uint4 *>(d + round_up((int64_t)g.u_bytes, 256));
  if (raw->r > 0) {
    // U: source [d_in x r], k = d_in, features = r (zero-padded to r_pad)
    int64_t n = g.n_rtiles * g.KB1 * 64;
    hipLaunchKernelGGL(pack_fragments_kernel, dim3((unsigned)(ceil_div(n, 256) < 65535 ? ceil_div(n, 256) : 65535)), dim3(256), 0, s,
                       static_cast<const uint16_t *>(raw->U), raw->ldu, (int)raw->d_in, (int)raw->r,
                       (int)g.n_rtiles, (int)g.KB1, du);
    if (int rc = check_launch("pack U")) return rc;
    // V: source [r x d_out], k = r (zero-padded), features = d_out
    n = g.n_otiles * g.KB2 * 64;
    hipLaunchKernelGGL(pack_fragments_kernel, dim3((unsigned)(ceil_div(n, 256) < 65535 ? ceil_div(n, 256) : 65535)), dim3(256), 0, s,
                       static_cast<const uint16_t *>(raw->V), raw->ldv, (int)raw->r, (int)raw->d_out,
                       (int)g.n_otiles, (int)g.KB2, dv);
    if (int rc = check_launch("pack V")) return rc;
  }
  *packed = *raw;
  packed->U = du;
  packed->V = dv;
  packed->ldu = 0;
  packed->ldv = 0;
  packed->layout = DEINFER_LAYOUT_PACKED;
  return DEINFER_OK;
}

int deinfer_workspace_bytes(int64_t T, const deinfer_factors_t *const *pairs, int n_pairs, size_t *bytes) {
  if (!bytes) return fail(DEINFER_ERR_INVALID_ARG, "bytes is NULL");
  if (T < 0) return fail(DEINFER_ERR_INVALID_ARG, "T is negative");
  if (!pairs || n_pairs < 1 || n_pairs > 3) return fail(DEINFER_ERR_INVALID_ARG, "need 1..3 pairs");
  for (int i = 0; i < n_pairs; ++i) {
    if (!pairs[i]) return fail(DEINFER_ERR_INVALID_ARG, "pair %d is NULL", i);
    if (pairs[i]->r < 0 || pairs[i]->d_in <= 0 || pairs[i]->d_out <= 0) return fail(DEINFER_ERR_INVALID_ARG, "pair %d: bad sizes", i);
  }
  *bytes = workspace_need(T, pairs, n_pairs);
  return DEINFER_OK;
}

int deinfer_workspace_init(void *ws, size_t ws_bytes, void *stream) {
  if (!ws) return fail(DEINFER_ERR_WORKSPACE, "workspace pointer is NULL");
  if (!aligned(ws, 256)) return fail(DEINFER_ERR_MISALIGNED, "workspace must be 256-byte aligned");
  if (ws_bytes < WS_HEADER) return fail(DEINFER_ERR_WORKSPACE, "workspace smaller than its header (%zu bytes)", WS_HEADER);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t hw = WS_HEADER / 4;
  hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)ceil_div((int64_t)hw, 256)), dim3(256), 0, s,
                     static_cast<uint32_t *>(ws), hw, 0u);
  return check_launch("workspace init");
}

int deinfer_workspace_check(void *ws, size_t ws_bytes, void *stream) {
  if (!ws) return fail(DEINFER_ERR_WORKSPACE, "workspace pointer is NULL");
  if (ws_bytes < WS_HEADER) return fail(DEINFER_ERR_WORKSPACE, "workspace smaller than its header");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipStreamSynchronize(s) != hipSuccess) return fail(DEINFER_ERR_DEVICE, "stream synchronise failed");
  unsigned words[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (hipMemcpy(words, ws, sizeof(words), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(DEINFER_ERR_DEVICE, "reading the workspace status failed");
  if (words[4] != 0) return fail(DEINFER_ERR_DEVICE, "a kernel reported an error in the workspace status words");
  return DEINFER_OK;
}

int deinfer_lowrank_linear(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f,
                           void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = x; g.T = T; g.ldx = ldx; g.n = 1; g.f[0] = f; g.out[0] = y; g.ldo[0] = ldy;
  g.glu = false; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

// ---- the entry point that takes no workspace: its scratch is a static device array
}  // extern "C"

namespace {
// One copy per GPU that loads the library, held until the process ends.  In host code the name is
// only a handle for hipGetSymbolAddress: the device address it yields (one per device) is what
// kernels and host calls are given.
static __device__ __align__(256) unsigned char scratch[DEINFER_STATIC_SCRATCH_BYTES];
void *g_scratch_ptr[64];                 // per device, set once (under g_scratch_mutex)
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
int static_scratch(void **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(DEINFER_ERR_DEVICE, "no usable HIP device");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return fail(DEINFER_ERR_DEVICE, "cannot locate the static scratch array on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;            // (a static device array starts zero-filled: the status words need no clearing)
  }
  *out = g_scratch_ptr[dev];
  return DEINFER_OK;
}
}  // namespace

extern "C" {

int deinfer_lowrank_linear_static(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f,
                                  void *y, int64_t ldy, void *stream) {
  if (int rc = validate_pair(f, "pair 0")) return rc;
  if (T < 0) return fail(DEINFER_ERR_INVALID_ARG, "T is negative");
  const deinfer_factors_t *pairs[1] = {f};
  const size_t need = workspace_need(T, pairs, 1);
  if (need > (size_t)DEINFER_STATIC_SCRATCH_BYTES)
    return fail(DEINFER_ERR_WORKSPACE, "this call needs %zu bytes of scratch, the static scratch array holds %zu: "
                "use deinfer_lowrank_linear with a workspace of the caller's", need, (size_t)DEINFER_STATIC_SCRATCH_BYTES);
  void *ws = nullptr;                    // (T == 0 returns before the workspace is looked at)
  if (T > 0)
    if (int rc = static_scratch(&ws)) return rc;
  return deinfer_lowrank_linear(x, T, ldx, f, y, ldy, ws, (size_t)DEINFER_STATIC_SCRATCH_BYTES, stream);
}

int deinfer_lowrank_up(const void *t, int64_t T, int64_t ldt, const deinfer_factors_t *f,
                       void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = t; g.T = T; g.ldx = ldt; g.n = 1; g.f[0] = f; g.out[0] = y; g.ldo[0] = ldy;
  g.glu = false; g.up_only = true; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_rope_table(const int32_t *positions, int64_t T, int64_t head_dim, double theta, float *table, void *stream) {
  if (T < 0 || head_dim <= 0 || head_dim % 2 != 0 || head_dim > (1 << 20))
    return fail(DEINFER_ERR_INVALID_ARG, "rope table: T >= 0 and an even head_dim in (0, 2^20] are required");
  if (!(theta > 0.0)) return fail(DEINFER_ERR_INVALID_ARG, "rope table: theta must be positive");
  if (T == 0) return DEINFER_OK;
  if (!positions || !table) return fail(DEINFER_ERR_INVALID_ARG, "rope table: positions or table is NULL");
  if (!aligned(positions, 4) || !aligned(table, 16)) return fail(DEINFER_ERR_MISALIGNED, "rope table: the table must be 16-byte aligned");
  const int64_t n = T * (head_dim / 2);
  if (ceil_div(n, (int64_t)256) > INT32_MAX) return fail(DEINFER_ERR_UNSUPPORTED, "rope table: too many tokens");
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)ceil_div(n, (int64_t)256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     positions, (long long)T, (int)head_dim, log2(theta), table);
  return check_launch("rope table");
}

int deinfer_lowrank_up_rope(const void *t, int64_t T, int64_t ldt, const deinfer_factors_t *f, const float *table,
                            int64_t head_dim, void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
  if (!f) return fail(DEINFER_ERR_INVALID_ARG, "factor descriptor is NULL");
  if (head_dim <= 0 || head_dim % 2 != 0 || head_dim > (1 << 20) || f->d_out % head_dim != 0)
    return fail(DEINFER_ERR_INVALID_ARG, "up + rope: head_dim must be even, positive and divide d_out");
  if (T > 0 && !table) return fail(DEINFER_ERR_INVALID_ARG, "up + rope: table is NULL");
  if (!aligned(table, 16)) return fail(DEINFER_ERR_MISALIGNED, "up + rope: the table must be 16-byte aligned");
  if (T > INT32_MAX / 2) return fail(DEINFER_ERR_UNSUPPORTED, "up + rope: too many tokens");
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = t; g.T = T; g.ldx = ldt; g.n = 1; g.f[0] = f; g.out[0] = y; g.ldo[0] = ldy;
  g.glu = false; g.up_only = true; g.rope = table; g.rope_dim = head_dim;
  g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_lowrank_linear_act(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f, const void *bias, int act,
                               void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
  if (!f) return fail(DEINFER_ERR_INVALID_ARG, "factor descriptor is NULL");
  if (act != DEINFER_ACT_NONE && act != DEINFER_ACT_RELU && act != DEINFER_ACT_GELU)
    return fail(DEINFER_ERR_UNSUPPORTED, "unknown activation %d", act);
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = x; g.T = T; g.ldx = ldx; g.n = 1; g.f[0] = f; g.out[0] = y; g.ldo[0] = ldy;
  g.glu = false; g.bias = bias; g.act = act; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_lowrank_down_proj(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *const *f, int n_pairs,
                              void *const *t_out, const int64_t *ldt, void *ws, size_t ws_bytes, void *stream) {
  if (n_pairs < 1 || n_pairs > 3) return fail(DEINFER_ERR_INVALID_ARG, "1 to 3 pairs per call, got %d", n_pairs);
  if (!f || !t_out || !ldt) return fail(DEINFER_ERR_INVALID_ARG, "pair, output or pitch array is NULL");
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = x; g.T = T; g.ldx = ldx; g.n = n_pairs;
  for (int i = 0; i < n_pairs; ++i) {
    if (!f[i]) return fail(DEINFER_ERR_INVALID_ARG, "factor descriptor %d is NULL", i);
    g.f[i] = f[i]; g.t_out[i] = t_out[i]; g.ldt[i] = ldt[i];
  }
  g.down_only = true; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_lowrank_up_glu_silu(const void *t_gate, int64_t ldtg, const void *t_up, int64_t ldtu, int64_t T,
                                const deinfer_factors_t *fgate, const deinfer_factors_t *fup,
                                void *h, int64_t ldh, void *ws, size_t ws_bytes, void *stream) {
  if (!fgate || !fup) return fail(DEINFER_ERR_INVALID_ARG, "factor descriptor is NULL");
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = t_gate; g.ldx = ldtg; g.x2 = t_up; g.ldx2 = ldtu; g.T = T; g.n = 2; g.f[0] = fgate; g.f[1] = fup;
  g.out[0] = h; g.ldo[0] = ldh; g.glu = true; g.up_only = true;
  g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_lowrank_down(const void *h, int64_t T, int64_t ldh, const deinfer_factors_t *fdown,
                         void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
  return deinfer_lowrank_linear(h, T, ldh, fdown, y, ldy, ws, ws_bytes, stream);
}

int deinfer_lowrank_qkv(const void *x, int64_t T, int64_t ldx,
                        const deinfer_factors_t *fq, const deinfer_factors_t *fk, const deinfer_factors_t *fv,
                        void *q, int64_t ldq, void *k, int64_t ldk, void *v, int64_t ldv,
                        void *t_k, int64_t ldtk, void *t_v, int64_t ldtv,
                        void *ws, size_t ws_bytes, void *stream) {
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = x; g.T = T; g.ldx = ldx; g.n = 3;
  g.f[0] = fq; g.f[1] = fk; g.f[2] = fv;
  g.out[0] = q; g.out[1] = k; g.out[2] = v;
  g.ldo[0] = ldq; g.ldo[1] = ldk; g.ldo[2] = ldv;
  g.t_out[1] = t_k; g.ldt[1] = ldtk; g.t_out[2] = t_v; g.ldt[2] = ldtv;
  g.glu = false; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

int deinfer_lowrank_gateup_silu(const void *x, int64_t T, int64_t ldx,
                                const deinfer_factors_t *fgate, const deinfer_factors_t *fup,
                                void *h, int64_t ldh, void *ws, size_t ws_bytes, void *stream) {
  Group g;
  memset(&g, 0, sizeof(g));
  g.x = x; g.T = T; g.ldx = ldx; g.n = 2;
  g.f[0] = fgate; g.f[1] = fup;
  g.out[0] = h; g.ldo[0] = ldh;
  g.glu = true; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = static_cast<hipStream_t>(stream);
  return run_group(g);
}

}  // extern "C"
