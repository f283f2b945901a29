/*
 * deinfer.h - C ABI of the MI355X (gfx950) low-rank linear-layer library.
 *
 * A decomposed LLM replaces every dense projection W[d_in x d_out] by a factor
 * pair W ~= U . V (DeInfer paper, Sec. 2.1, Eq. 1: W ~= A B with A = U_k sqrt(S_k),
 * B = sqrt(S_k) V_k^T).  The layer then computes two chained products,
 *     t = x . U   (downward projection into the rank space, width r)
 *     y = t . V   (upward projection)
 * (Sec. 4.1).  Naming: U here is the FIRST / downward factor (the paper's A, its
 * "x_v"); V is the SECOND / upward factor (the paper's B, its "x_u").  Row-vector
 * convention y = x U V; every matrix is row-major.
 *
 * General rules for every call
 *  - All data pointers are DEVICE pointers on the calling thread's current HIP
 *    device, owned by the caller, and must stay valid until the stream work is done.
 *  - Calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL =
 *    default stream); they never synchronise the device and never allocate.
 *  - Outputs must not alias inputs or the workspace.
 *  - Return value: DEINFER_OK or a negative deinfer_status_t; on error nothing is
 *    enqueued and deinfer_last_error() describes the problem.  Argument validation
 *    happens on the host before any device call.
 *  - T == 0 is a successful no-op.  A pair with r == 0 yields an all-zero output.
 *  - No bias term (the paper's layers carry none), except the optional one of
 *    deinfer_lowrank_linear_act.
 */
#ifndef DEINFER_H
#define DEINFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DEINFER_OK = 0,
  DEINFER_ERR_INVALID_ARG = -1,  /* NULL pointer, negative size, inconsistent shapes */
  DEINFER_ERR_UNSUPPORTED = -2,  /* dtype / layout / feature combination not available */
  DEINFER_ERR_MISALIGNED = -3,   /* pointer or leading dimension breaks an alignment rule */
  DEINFER_ERR_WORKSPACE = -4,    /* workspace missing or too small */
  DEINFER_ERR_DEVICE = -5        /* the HIP runtime reported an error (no GPU, bad launch) */
} deinfer_status_t;

typedef enum { DEINFER_F32 = 0, DEINFER_BF16 = 1, DEINFER_F16 = 2 } deinfer_dtype_t;

typedef enum {
  DEINFER_LAYOUT_RAW = 0,    /* U[d_in x r] (ldu), V[r x d_out] (ldv), row-major          */
  DEINFER_LAYOUT_PACKED = 1  /* produced by deinfer_pack_factors (bf16 or fp16), see below */
} deinfer_layout_t;

/*
 * One factor pair (Sec. 2.1: an m x n weight becomes (m + n) k parameters; here
 * m = d_in, n = d_out, k = r).  Each pair carries its own rank: different layers,
 * and q / k / v inside one layer, may use different ratios (Sec. 4.3).
 */
typedef struct deinfer_factors {
  const void *U;           /* device; RAW: d_in x r elements, row pitch ldu            */
  const void *V;           /* device; RAW: r x d_out elements, row pitch ldv            */
  int64_t d_in, d_out, r;  /* logical sizes; r >= 0                                     */
  int64_t ldu, ldv;        /* RAW: leading dimensions in elements (>= r, >= d_out).
                              PACKED: ignored                                           */
  int32_t dtype;           /* deinfer_dtype_t of U, V, the activations and the outputs  */
  int32_t layout;          /* deinfer_layout_t                                          */
  double param_reduction;  /* informational: the compression ratio this rank came from  */
} deinfer_factors_t;

/* Human-readable text for the last error on this thread (static storage, never NULL). */
const char *deinfer_last_error(void);

/* Library version, major * 1000 + minor. */
int deinfer_version(void);

/*
 * Rank that keeps a fraction (1 - param_reduction) of the m*n parameters of a weight:
 *     r = floor((1 - param_reduction) * m * n / (m + n))
 * since a pair of inner size k holds (m + n) k parameters (Sec. 2.1).  The ratio is
 * taken at a resolution of 1e-6 and the division is exact integer arithmetic.
 * Host-only.  Errors: INVALID_ARG for m, n <= 0, ratio outside [0, 1] or NULL r_out.
 */
int deinfer_rank_for_ratio(int64_t m, int64_t n, double param_reduction, int64_t *r_out);

/*
 * Packed weight format (the 16-bit types: bf16, fp16).  Weights are static, so they are
 * re-laid once for the matrix cores: each factor is stored transposed ("feature" rows, reduction
 * index contiguous), zero-padded (r to a multiple of 32, feature counts to 16,
 * d_in to 32), and cut into 16-feature x 32-k fragments of 1 KiB held in the lane
 * order of the gfx950 16x16x32 MFMA operand (the same for bf16 and fp16), fragment
 * (tile, kblock) at ((tile * n_kblocks) + kblock) KiB.  A wavefront then reads one fragment with a
 * single fully coalesced 16-byte-per-lane load.  Zero rank rows are exact no-ops.
 *
 * deinfer_packed_bytes: size of the packed image of `raw` (host-only).
 * deinfer_pack_factors: enqueue the re-layout of `raw` (RAW, bf16 or fp16) into dst
 *   (device, 256-byte aligned, >= packed bytes) and fill *packed (host struct) with
 *   a descriptor that points into dst.  dst must outlive every use of *packed.
 */
int deinfer_packed_bytes(const deinfer_factors_t *raw, size_t *bytes);
int deinfer_pack_factors(const deinfer_factors_t *raw, void *dst, size_t dst_bytes,
                         deinfer_factors_t *packed, void *stream);

/*
 * Workspace.  The library never allocates: the rank-space intermediate t (Sec. 4.1) and
 * the partial sums it is built from live in a caller-provided device buffer.
 *  deinfer_workspace_bytes: bytes needed for a call with T tokens over the given pairs
 *    (all pairs of one entry-point call).  Host-only.  Take the maximum over the calls
 *    that will share the workspace.
 *  deinfer_workspace_init: enqueue once on a fresh workspace; clears its status words with
 *    a fill kernel (safe under stream capture).
 *  deinfer_workspace_check: synchronises `stream`, reads the status words back and returns
 *    DEINFER_ERR_DEVICE if a kernel flagged an error there.
 * A workspace is 256-byte aligned and serves one call at a time: calls that overlap in
 * time (different streams) need different workspaces.
 */
int deinfer_workspace_bytes(int64_t T, const deinfer_factors_t *const *pairs, int n_pairs,
                            size_t *bytes);
int deinfer_workspace_init(void *ws, size_t ws_bytes, void *stream);
int deinfer_workspace_check(void *ws, size_t ws_bytes, void *stream);

/*
 * y[T x d_out] = (x[T x d_in] . U) . V            (Sec. 2.1 Eq. 1, Sec. 4.1)
 * One decomposed projection (also the attention O projection).  x, y have the
 * pair's dtype; ldx >= d_in, ldy >= d_out in elements.  Accumulation is fp32; the
 * output is rounded once (nearest-even) to the dtype.
 * PACKED pairs additionally need x 16-byte aligned, ldx % 8 == 0, d_in % 8 == 0.
 */
int deinfer_lowrank_linear(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f,
                           void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/*
 * Attention first sub-layer (Sec. 4.1): the three downward projections are applied
 * as one concatenated product x . [U_q | U_k | U_v], reading x once; each low-rank
 * result is then multiplied by its own upward matrix:
 *   q = (x U_q) V_q,  k = (x U_k) V_k,  v = (x U_v) V_v.
 * The pairs share d_in, dtype and layout; ranks and output widths may differ (GQA,
 * per-matrix ratios).  t_k / t_v (optional, may be NULL) receive the rank-space
 * intermediates x U_k and x U_v, T x r_k and T x r_v with pitches ldtk / ldtv:
 * the low-rank KV cache of Sec. 2.1.
 */
int deinfer_lowrank_qkv(const void *x, int64_t T, int64_t ldx,
                        const deinfer_factors_t *fq, const deinfer_factors_t *fk,
                        const deinfer_factors_t *fv,
                        void *q, int64_t ldq, void *k, int64_t ldk, void *v, int64_t ldv,
                        void *t_k, int64_t ldtk, void *t_v, int64_t ldtv,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * GLU-type MLP first sub-layer (Sec. 4.1 "activation computation", Table 2 GLU-based):
 *   h = silu((x U_g) V_g) * ((x U_u) V_u),   silu(z) = z / (1 + exp(-z)),
 * element-wise product, evaluated in fp32 and rounded once.  Both pairs share d_in
 * and d_out (= FFN width).  The full-width gate and up results are never stored as such: for T > 128,
 * and for 17 .. 128 tokens where the layer is wide enough to fill the device that way, both
 * products of an output tile are accumulated in one workgroup and h is stored once; otherwise
 * they are fp32 partial sums in the workspace until the kernel that sums them applies the
 * activation.
 */
int deinfer_lowrank_gateup_silu(const void *x, int64_t T, int64_t ldx,
                                const deinfer_factors_t *fgate, const deinfer_factors_t *fup,
                                void *h, int64_t ldh, void *ws, size_t ws_bytes, void *stream);

/*
 * deinfer_lowrank_linear for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * product and same kernels as deinfer_lowrank_linear; the scratch (rank-space intermediate,
 * partial sums) is a static device array of DEINFER_STATIC_SCRATCH_BYTES inside the library, one
 * copy per GPU, held until the process ends.  The call allocates nothing (no hipMalloc / hipFree,
 * no allocating library routine); on the first call per device it looks the array's device address
 * up.  Limits: calls whose deinfer_workspace_bytes exceeds DEINFER_STATIC_SCRATCH_BYTES return
 * DEINFER_ERR_WORKSPACE and enqueue nothing (decode-sized calls up to the 70B shapes at 128 tokens
 * fit).  Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams, or graphs replayed concurrently) race; serialise them or use
 * deinfer_lowrank_linear with separate workspaces.  Nothing in the array has to survive between
 * calls and nothing has to be cleared.  Otherwise the contract of deinfer_lowrank_linear.
 */
#define DEINFER_STATIC_SCRATCH_BYTES (32u << 20)
int deinfer_lowrank_linear_static(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f,
                                  void *y, int64_t ldy, void *stream);

/*
 * Upward projection alone (Sec. 2.1 / 4.1: the low-rank KV cache stores k_low_rank = x U_k and
 * v_low_rank = x U_v; keys and values are rebuilt as k = k_low_rank V_k when attention needs
 * them):  y[T x d_out] = t[T x r] . V.   t: device, row-major, pitch ldt >= r, same dtype as
 * the pair.  f must describe a whole valid pair, as for every other call, although only f->V,
 * f->r and f->d_out enter the product.  Only the columns 0 .. r - 1 of every row are read,
 * whatever lies behind them in the row (the rest of a wider cache line, another tensor, NaN).
 * With PACKED pairs, rows with a 16-byte aligned t and ldt % 8 == 0 are read in place
 * (r >= 8 or r % 8 == 0); any other rows are first copied, zero padded, into the workspace (one
 * small launch more; the room is part of deinfer_workspace_bytes).  Otherwise the contract of
 * deinfer_lowrank_linear.
 */
int deinfer_lowrank_up(const void *t, int64_t T, int64_t ldt, const deinfer_factors_t *f,
                       void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/*
 * The two stages as separate calls (Sec. 4.1 puts the one exchange between tensor-parallel ranks
 * of a sub-layer exactly between them: a rank multiplies x by its column slice of the downward
 * matrices, the rank-space results are gathered - or, for the second sub-layer, whose downward
 * matrix is split by rows, summed - and the rank then applies its shard of the upward matrices;
 * on one GPU the calls are what one rank runs on its shard).
 *
 * deinfer_lowrank_down_proj: t_i = x U_i for 1 to 3 pairs that share x (the concatenated
 *   downward projection); t_out[i]: device, T x r_i, pitch ldt[i] >= r_i, written in the pairs'
 *   dtype (bf16 / fp16: one rounding); f, t_out, ldt: host arrays of n_pairs entries.  No upward
 *   projection runs and V is not read.
 * deinfer_lowrank_up_glu_silu: h = silu(t_gate V_gate) * (t_up V_up), the second stage of
 *   deinfer_lowrank_gateup_silu alone; t_gate / t_up as the t of deinfer_lowrank_up (read in
 *   place or copied first by the same rule, both together), both pairs share d_out.
 * Otherwise the contract of deinfer_lowrank_linear.
 */
int deinfer_lowrank_down_proj(const void *x, int64_t T, int64_t ldx,
                              const deinfer_factors_t *const *f, int n_pairs,
                              void *const *t_out, const int64_t *ldt,
                              void *ws, size_t ws_bytes, void *stream);
int deinfer_lowrank_up_glu_silu(const void *t_gate, int64_t ldtg, const void *t_up, int64_t ldtu,
                                int64_t T, const deinfer_factors_t *fgate,
                                const deinfer_factors_t *fup, void *h, int64_t ldh,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * First sub-layer of a non-GLU MLP (Table 2 lists GLU-based and non-GLU models; Sec. 4.1
 * "activation computation" after the upward projection):
 *   y = act((x U) V + bias),   bias: device, d_out values of the pair's dtype, may be NULL
 *   (PACKED pairs: 16-byte aligned), broadcast over the token rows;
 *   act: DEINFER_ACT_NONE, DEINFER_ACT_RELU max(z, 0), DEINFER_ACT_GELU z * Phi(z) (erf form).
 * Sum, bias and activation are evaluated in fp32 on the accumulators and rounded once.  The
 * paper prints neither activation nor a bias; these are the textbook definitions.  Otherwise
 * the contract of deinfer_lowrank_linear (a pair of rank 0 gives y = act(bias)).
 */
enum { DEINFER_ACT_NONE = 0, DEINFER_ACT_RELU = 1, DEINFER_ACT_GELU = 2 };
int deinfer_lowrank_linear_act(const void *x, int64_t T, int64_t ldx, const deinfer_factors_t *f,
                               const void *bias, int act, void *y, int64_t ldy,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * Paged low-rank cache and static graphs (Sec. 4.2, "Integrating Paged Cache and CUDA Graph").  The low-rank cache (k_low_rank, v_low_rank)
 * lives in a pool of fixed-size physical blocks; a block table names, per sequence, the blocks it
 * owns.  Before attention the blocks are squeezed into a compact buffer at a fixed address, the
 * buffer is multiplied by the upward matrix (deinfer_lowrank_up with T = the buffer's token
 * capacity, so the launch never changes) and, for keys, the rotary embedding is applied in
 * place.  The kernels take what changes between steps from device memory: the sequence
 * "preparation stage (host) -> copy of the plan and the positions to the device -> replay of a
 * captured graph of deinfer_kv_compact_copy, deinfer_lowrank_up, deinfer_rope_inplace" is valid.
 *
 * deinfer_kv_compact_plan (host only, preparation stage): walks the sequences in table order and
 * their blocks in logical order; the d-th block of the walk goes to buffer block d.  It writes
 *   plan   (host, DEINFER_KV_PLAN_WORDS(plan_capacity_runs) int32): [0] number of runs, [1] number
 *          of blocks, [2..3] zero, then (source block, destination block, length) per run, a run
 *          being a maximal stretch of the walk whose physical ids increase by one (it may pass
 *          from one sequence into the next);
 *   remap  (host, n_seqs x remap_pitch, may be NULL): the "remapping index list", remap[s][i] =
 *          buffer block of logical block i of sequence s, -1 beyond the sequence's blocks;
 *   positions (host, buffer_blocks * block_tokens, may be NULL): position inside its sequence of
 *          every token slot of the buffer (0 for unused blocks), the input of the rotary kernel.
 * block_table: host, n_seqs x table_pitch int32; n_blocks: host, blocks held per sequence.
 * Errors: a block id outside [0, n_pool_blocks), more blocks than the buffer or the tables hold,
 * more runs than plan_capacity_runs.
 *
 * deinfer_kv_compact_copy (device, graph replay stage): copies the runs of `plan` (DEVICE copy of
 * the host plan) from `pool` (n_pool_blocks x block_bytes, device, 16-byte aligned, block_bytes a
 * multiple of 16) into `buffer` (buffer_blocks x block_bytes).  Buffer blocks beyond plan[1] are
 * left alone.  Runs that point outside the pool or the buffer are skipped.  Asynchronous on
 * `stream`, no allocation; the launch shape depends only on buffer_blocks and block_bytes.
 */
#define DEINFER_KV_PLAN_WORDS(capacity_runs) (4 + 3 * (size_t)(capacity_runs))
int deinfer_kv_compact_plan(const int32_t *block_table, int64_t n_seqs, int64_t table_pitch,
                            const int32_t *n_blocks, int64_t n_pool_blocks, int64_t buffer_blocks,
                            int64_t block_tokens, int32_t *plan, int64_t plan_capacity_runs,
                            int32_t *remap, int64_t remap_pitch, int32_t *positions);
int deinfer_kv_compact_copy(const void *pool, int64_t n_pool_blocks, int64_t block_bytes,
                            const int32_t *plan, int64_t plan_capacity_runs,
                            void *buffer, int64_t buffer_blocks, void *stream);

/*
 * Rotary position embedding in place (Sec. 4.2 applies it to the rebuilt keys; the paper prints
 * no formula, this is the one of LLaMA-type models): x is T x (n_heads * head_dim), pitch ldx,
 * device, dtype DEINFER_BF16, DEINFER_F16 or DEINFER_F32; inside every head the elements i and i + head_dim/2
 * (i < head_dim/2) are replaced by
 *   x_i cos(a) - x_{i + D/2} sin(a),   x_{i + D/2} cos(a) + x_i sin(a),   a = pos * theta^(-2 i / D),
 * pos = positions[token] (device, int32).  Angles in double precision, products in fp32, one
 * rounding to the storage type.  Asynchronous on `stream`, no allocation.
 */
int deinfer_rope_inplace(void *x, int64_t T, int64_t ldx, int64_t n_heads, int64_t head_dim,
                         const int32_t *positions, double theta, int dtype, void *stream);

/*
 * Upward projection of keys with the rotary embedding applied on the way out (Sec. 4.2 rebuilds
 * the keys from k_low_rank and then rotates them; here the rotation is the last step of the
 * product's kernel, so the rebuilt keys cross HBM once instead of three times):
 *   deinfer_rope_table:      table[t][i] = cos(a_ti), table[t][head_dim/2 + i] = sin(a_ti),
 *                            a_ti = positions[t] * theta^(-2 i / head_dim), i < head_dim/2;
 *                            positions: device int32 [T]; table: device fp32 [T][head_dim],
 *                            16-byte aligned, owned by the caller (angles in double precision).
 *   deinfer_lowrank_up_rope: y = rope(t V) with the angles of `table`: the contract of
 *                            deinfer_lowrank_up, then that of deinfer_rope_inplace with
 *                            n_heads = d_out / head_dim (head_dim must divide d_out).  The
 *                            product is rounded to the storage type, rotated in fp32 and rounded
 *                            again, exactly as the two separate calls do.
 * PACKED pairs with head_dim = 128, d_out % 128 == 0, T > 128, y 16-byte aligned and
 * ldy % 8 == 0 rotate inside the product's kernel; every other case writes the product and
 * rotates it in place with a second launch.  The table depends only on the positions: one table
 * serves every layer of a step, and as device memory it may change between replays of a graph.
 * Asynchronous on `stream`, no allocation.
 */
int deinfer_rope_table(const int32_t *positions, int64_t T, int64_t head_dim, double theta,
                       float *table, void *stream);
int deinfer_lowrank_up_rope(const void *t, int64_t T, int64_t ldt, const deinfer_factors_t *f,
                            const float *table, int64_t head_dim, void *y, int64_t ldy,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * MLP second sub-layer (Sec. 4.1): y = (h U_d) V_d with d_in = FFN width.
 * Same contract as deinfer_lowrank_linear.
 */
int deinfer_lowrank_down(const void *h, int64_t T, int64_t ldh, const deinfer_factors_t *fdown,
                         void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DEINFER_H */
