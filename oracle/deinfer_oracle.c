/*
 * CPU oracle for the low-rank (decomposed) linear layer  y = (x . U) . V.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition of
 * what the GPU library computes.  It shares no code, header, table or helper
 * with the HIP path and must never be linked into, or called from, the product
 * library; only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may use it.
 *
 * What is computed (DeInfer paper, Sec. 2.1, Eq. 1 and Sec. 4.1):
 *   a weight W[d_in x d_out] is replaced by a factor pair  W ~= A . B  with
 *   A[d_in x r] (the "downward projection") and B[r x d_out] (the "upward
 *   projection").  The layer output is two chained matrix products, first
 *   t = x . A (rank space), then y = t . B.  Here A is called U and B is
 *   called V, row-vector convention, everything row-major with explicit
 *   leading dimensions.
 *
 * All arithmetic is IEEE double.  Every output element is a plain sum in
 * increasing index order; the loops are ordered i-c-k ("axpy" form) which
 * keeps that summation order per element and only makes memory access
 * contiguous.  No blocking, no fusion, no reassociation.
 *
 * Pins (tests/test_oracle_pins.py, run without a GPU): numpy fp64 matmul, the
 * associativity invariant (xU)V == x(UV) with UV from a separate loop nest,
 * full-rank SVD reproducing W, Eckart-Young truncation error, integer-exact
 * brute force, closed-form special cases (r = 1, identity factors, one-hot x,
 * linearity, SiLU identities) and the numbers the paper prints in Table 1.
 * No function in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the row loops will use (for the benchmark's report) */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Rank from a parameter-reduction ratio.
 * A pair of factors with inner size k holds (m + n) * k parameters instead of
 * m * n (Sec. 2.1, text after Eq. 1).  Keeping a fraction (1 - rho) of the
 * m*n parameters therefore allows k = floor((1 - rho) * m * n / (m + n)).
 * Exact integer arithmetic on a rational keep = keep_num / keep_den.
 * ---------------------------------------------------------------------- */
int64_t oracle_rank_for_keep(int64_t m, int64_t n, int64_t keep_num, int64_t keep_den) {
  if (m <= 0 || n <= 0 || keep_num < 0 || keep_den <= 0) return -1;
  /* floor(keep_num * m * n / (keep_den * (m + n))) with 128-bit headroom */
  __int128 num = (__int128)keep_num * (__int128)m * (__int128)n;
  __int128 den = (__int128)keep_den * ((__int128)m + (__int128)n);
  return (int64_t)(num / den);
}

/* parameter count of a factor pair: (m + n) * k  (Sec. 2.1) */
int64_t oracle_param_count(int64_t m, int64_t n, int64_t k) { return (m + n) * k; }

/* ------------------------------------------------------------------------
 * Per-token communication volume of one Transformer block (Table 1), in
 * "values per token".  Only used to pin the paper's printed numbers; it is
 * not on the GPU path (one GPU, no collectives).
 *   unoptimised: reduce-sum after every factor pair, counted twice
 *                (attention 2*(2h + 2h_kv), MLP 2*(2m + h));
 *   low-rank   : all-gather of l_q+l_k+l_v and l_up+l_gate, reduce-sum
 *                (counted twice) of l_o and l_down.
 * out[0] = unoptimised total, out[1] = all-gather part, out[2] = reduce-sum
 * part (already doubled), out[3] = low-rank total.
 * ---------------------------------------------------------------------- */
void oracle_comm_volume(int64_t h, int64_t h_kv, int64_t m,
                        int64_t l_q, int64_t l_k, int64_t l_v, int64_t l_o,
                        int64_t l_gate, int64_t l_up, int64_t l_down, int64_t out[4]) {
  out[0] = 2 * (2 * h + 2 * h_kv) + 2 * (2 * m + h);
  out[1] = (l_q + l_k + l_v) + (l_up + l_gate);
  out[2] = 2 * l_o + 2 * l_down;
  out[3] = out[1] + out[2];
}

/* ------------------------------------------------------------------------
 * Stage 1: downward projection  t[i,k] = sum_c x[i,c] * U[c,k]
 * (Sec. 4.1, first matrix of a pair; Eq. 1 with A -> U).
 * ---------------------------------------------------------------------- */
void oracle_down_projection(const double *x, int64_t T, int64_t ldx,
                            const double *U, int64_t ldu, int64_t d_in, int64_t r,
                            double *t, int64_t ldt) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < T; ++i) {
    double *ti = t + i * ldt;
    for (int64_t k = 0; k < r; ++k) ti[k] = 0.0;
    for (int64_t c = 0; c < d_in; ++c) {
      const double xc = x[i * ldx + c];
      const double *Uc = U + c * ldu;
      for (int64_t k = 0; k < r; ++k) ti[k] += xc * Uc[k];
    }
  }
}

/* ------------------------------------------------------------------------
 * Stage 2: upward projection  y[i,j] = sum_k t[i,k] * V[k,j]
 * (Sec. 4.1, second matrix of a pair; Eq. 1 with B -> V).
 * ---------------------------------------------------------------------- */
void oracle_up_projection(const double *t, int64_t T, int64_t ldt,
                          const double *V, int64_t ldv, int64_t r, int64_t d_out,
                          double *y, int64_t ldy) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < T; ++i) {
    double *yi = y + i * ldy;
    for (int64_t j = 0; j < d_out; ++j) yi[j] = 0.0;
    for (int64_t k = 0; k < r; ++k) {
      const double tk = t[i * ldt + k];
      const double *Vk = V + k * ldv;
      for (int64_t j = 0; j < d_out; ++j) yi[j] += tk * Vk[j];
    }
  }
}

/* ------------------------------------------------------------------------
 * One decomposed projection: y = (x . U) . V.  r == 0 gives y == 0.
 * If t_out is not NULL it receives the rank-space intermediate t[T x r]
 * (leading dimension r) - for the K and V projections this is what the paper
 * stores as the low-rank KV cache (Sec. 2.1, Sec. 4.1).
 * Returns 0, or -1 if scratch memory could not be obtained.
 * ---------------------------------------------------------------------- */
int oracle_lowrank_linear(const double *x, int64_t T, int64_t ldx,
                          const double *U, int64_t ldu, const double *V, int64_t ldv,
                          int64_t d_in, int64_t r, int64_t d_out,
                          double *y, int64_t ldy, double *t_out) {
  if (T <= 0) return 0;
  double *t = t_out;
  if (!t) {
    t = (double *)malloc(sizeof(double) * (size_t)T * (size_t)(r > 0 ? r : 1));
    if (!t) return -1;
  }
  oracle_down_projection(x, T, ldx, U, ldu, d_in, r, t, r);
  oracle_up_projection(t, T, r, V, ldv, r, d_out, y, ldy);
  if (!t_out) free(t);
  return 0;
}

/* ------------------------------------------------------------------------
 * Attention first sub-layer: the three projections share x (Sec. 4.1: the
 * downward matrices of a sub-layer are concatenated; each low-rank result is
 * then multiplied by its own upward matrix).  Computed here pair by pair,
 * which is the same thing element by element.  Ranks and output widths may
 * differ per pair (Sec. 4.3: variadic ratios, GQA).
 * ---------------------------------------------------------------------- */
int oracle_lowrank_qkv(const double *x, int64_t T, int64_t ldx, int64_t d_in,
                       const double *Uq, int64_t lduq, const double *Vq, int64_t ldvq, int64_t rq, int64_t dq,
                       const double *Uk, int64_t lduk, const double *Vk, int64_t ldvk, int64_t rk, int64_t dk,
                       const double *Uv, int64_t lduv, const double *Vv, int64_t ldvv, int64_t rv, int64_t dv,
                       double *q, int64_t ldq, double *k, int64_t ldk, double *v, int64_t ldvout,
                       double *tk_out, double *tv_out) {
  int rc = 0;
  rc |= oracle_lowrank_linear(x, T, ldx, Uq, lduq, Vq, ldvq, d_in, rq, dq, q, ldq, NULL);
  rc |= oracle_lowrank_linear(x, T, ldx, Uk, lduk, Vk, ldvk, d_in, rk, dk, k, ldk, tk_out);
  rc |= oracle_lowrank_linear(x, T, ldx, Uv, lduv, Vv, ldvv, d_in, rv, dv, v, ldvout, tv_out);
  return rc;
}

/* SiLU in fp64: z * sigmoid(z) = z / (1 + exp(-z)) */
double oracle_silu(double z) { return z / (1.0 + exp(-z)); }

/* ------------------------------------------------------------------------
 * GLU-type MLP first sub-layer (Sec. 4.1 "activation computation"; Table 2
 * "GLU-based"):  h = silu((x Ug) Vg) * ((x Uu) Vu), element-wise product.
 * ---------------------------------------------------------------------- */
int oracle_lowrank_gateup_silu(const double *x, int64_t T, int64_t ldx, int64_t d_in,
                               const double *Ug, int64_t ldug, const double *Vg, int64_t ldvg, int64_t rg,
                               const double *Uu, int64_t lduu, const double *Vu, int64_t ldvu, int64_t ru,
                               int64_t d_ff, double *h, int64_t ldh) {
  if (T <= 0) return 0;
  size_t n = (size_t)T * (size_t)(d_ff > 0 ? d_ff : 1);
  double *g = (double *)malloc(sizeof(double) * n);
  double *u = (double *)malloc(sizeof(double) * n);
  if (!g || !u) { free(g); free(u); return -1; }
  int rc = 0;
  rc |= oracle_lowrank_linear(x, T, ldx, Ug, ldug, Vg, ldvg, d_in, rg, d_ff, g, d_ff, NULL);
  rc |= oracle_lowrank_linear(x, T, ldx, Uu, lduu, Vu, ldvu, d_in, ru, d_ff, u, d_ff, NULL);
  for (int64_t i = 0; i < T; ++i)
    for (int64_t j = 0; j < d_ff; ++j)
      h[i * ldh + j] = oracle_silu(g[i * d_ff + j]) * u[i * d_ff + j];
  free(g); free(u);
  return rc;
}

/* ------------------------------------------------------------------------
 * Second stage of the GLU sub-layer alone (Sec. 4.1 under tensor parallelism: the rank-space
 * results of gate and up are gathered from all ranks first, then every rank applies its column
 * shard of the upward matrices):  h = silu(t_g V_g) * (t_u V_u).
 * ---------------------------------------------------------------------- */
int oracle_up_glu_silu(const double *tg, int64_t ldtg, const double *Vg, int64_t ldvg, int64_t rg,
                       const double *tu, int64_t ldtu, const double *Vu, int64_t ldvu, int64_t ru,
                       int64_t T, int64_t d_ff, double *h, int64_t ldh) {
  if (T <= 0) return 0;
  size_t n = (size_t)T * (size_t)(d_ff > 0 ? d_ff : 1);
  double *g = (double *)malloc(sizeof(double) * n);
  double *u = (double *)malloc(sizeof(double) * n);
  if (!g || !u) { free(g); free(u); return -1; }
  oracle_up_projection(tg, T, ldtg, Vg, ldvg, rg, d_ff, g, d_ff);
  oracle_up_projection(tu, T, ldtu, Vu, ldvu, ru, d_ff, u, d_ff);
  for (int64_t i = 0; i < T; ++i)
    for (int64_t j = 0; j < d_ff; ++j)
      h[i * ldh + j] = oracle_silu(g[i * d_ff + j]) * u[i * d_ff + j];
  free(g); free(u);
  return 0;
}

/* ------------------------------------------------------------------------
 * Non-GLU MLP first sub-layer (Table 2 lists GLU-based and non-GLU models; Sec. 4.1
 * "activation computation" after the upward projection):
 *   y = act((x U) V + b),  b broadcast over the token rows (NULL = no bias),
 *   act 0: identity, 1: ReLU max(z, 0), 2: GELU z * Phi(z) with Phi the standard
 *   normal distribution function, written with erf.
 * The paper prints neither activation; these are the textbook definitions.
 * ---------------------------------------------------------------------- */
double oracle_relu(double z) { return z > 0.0 ? z : 0.0; }
double oracle_gelu(double z) { return 0.5 * z * (1.0 + erf(z / sqrt(2.0))); }

int oracle_lowrank_linear_act(const double *x, int64_t T, int64_t ldx,
                              const double *U, int64_t ldu, const double *V, int64_t ldv,
                              int64_t d_in, int64_t r, int64_t d_out,
                              const double *bias, int act, double *y, int64_t ldy) {
  if (act < 0 || act > 2) return -3;
  int rc = oracle_lowrank_linear(x, T, ldx, U, ldu, V, ldv, d_in, r, d_out, y, ldy, NULL);
  if (rc) return rc;
  for (int64_t i = 0; i < T; ++i)
    for (int64_t j = 0; j < d_out; ++j) {
      double z = y[i * ldy + j] + (bias ? bias[j] : 0.0);
      y[i * ldy + j] = act == 1 ? oracle_relu(z) : act == 2 ? oracle_gelu(z) : z;
    }
  return 0;
}

/* Second sub-layer of the MLP (and the O projection): a plain factor pair. */
int oracle_lowrank_down(const double *h, int64_t T, int64_t ldh,
                        const double *U, int64_t ldu, const double *V, int64_t ldv,
                        int64_t d_ff, int64_t r, int64_t d_out, double *y, int64_t ldy) {
  return oracle_lowrank_linear(h, T, ldh, U, ldu, V, ldv, d_ff, r, d_out, y, ldy, NULL);
}

/* ------------------------------------------------------------------------
 * Diagnostic only (never the parity reference): round a double to the nearest
 * bfloat16 value, ties to even, returned as a double.  Used by tests to
 * separate the expected mixed-precision error of a bf16 rank-space
 * intermediate from real bugs.
 * ---------------------------------------------------------------------- */
double oracle_round_to_bf16(double v) {
  if (v == 0.0 || isnan(v) || isinf(v)) return v;
  int e;
  double m = frexp(v, &e);          /* v = m * 2^e, 0.5 <= |m| < 1 */
  if (e < -125) return v;           /* below the normal bf16 range: leave alone */
  double scaled = ldexp(m, 8);      /* 8 significant bits: 128 <= |scaled| < 256 */
  double rounded = nearbyint(scaled); /* default rounding mode = ties to even */
  return ldexp(rounded, e - 8);
}

/* ------------------------------------------------------------------------
 * Offline factorisation helper used only by the oracle's own tests
 * (Sec. 2.1, Eq. 1): truncated SVD  W ~= A B,  A = U_k sqrt(S_k),
 * B = sqrt(S_k) V_k^T.  One-sided Jacobi (Hestenes) on the columns of a work
 * copy; fp64.  W is m x n row-major with m >= n required (callers transpose
 * otherwise).  sigma receives all n singular values in decreasing order.
 * A is m x k, B is k x n, both row-major and dense.
 * Returns the number of sweeps used, or -1 on allocation failure.
 * ---------------------------------------------------------------------- */
int oracle_svd_factor(const double *W, int64_t m, int64_t n, int64_t k,
                      double *A, double *B, double *sigma) {
  if (m < n || k > n || k < 0) return -2;
  double *G = (double *)malloc(sizeof(double) * (size_t)m * (size_t)n); /* becomes U*S */
  double *R = (double *)malloc(sizeof(double) * (size_t)n * (size_t)n); /* accumulates V */
  int64_t *ord = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
  if (!G || !R || !ord) { free(G); free(R); free(ord); return -1; }
  memcpy(G, W, sizeof(double) * (size_t)m * (size_t)n);
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) R[i * n + j] = (i == j) ? 1.0 : 0.0;

  int sweeps = 0;
  for (; sweeps < 60; ++sweeps) {
    double off = 0.0;
    for (int64_t p = 0; p < n - 1; ++p) {
      for (int64_t q = p + 1; q < n; ++q) {
        double alpha = 0.0, beta = 0.0, gamma = 0.0;
        for (int64_t i = 0; i < m; ++i) {
          double gp = G[i * n + p], gq = G[i * n + q];
          alpha += gp * gp; beta += gq * gq; gamma += gp * gq;
        }
        if (gamma == 0.0) continue;
        double rel = fabs(gamma) / sqrt(alpha * beta);
        if (rel > off) off = rel;
        if (rel < 1e-16) continue;
        double zeta = (beta - alpha) / (2.0 * gamma);
        double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        double c = 1.0 / sqrt(1.0 + tt * tt), s = c * tt;
        for (int64_t i = 0; i < m; ++i) {
          double gp = G[i * n + p], gq = G[i * n + q];
          G[i * n + p] = c * gp - s * gq;
          G[i * n + q] = s * gp + c * gq;
        }
        for (int64_t i = 0; i < n; ++i) {
          double rp = R[i * n + p], rq = R[i * n + q];
          R[i * n + p] = c * rp - s * rq;
          R[i * n + q] = s * rp + c * rq;
        }
      }
    }
    if (off < 1e-15) break;
  }
  /* column norms are the singular values; sort decreasing (selection sort) */
  for (int64_t j = 0; j < n; ++j) {
    double s2 = 0.0;
    for (int64_t i = 0; i < m; ++i) s2 += G[i * n + j] * G[i * n + j];
    sigma[j] = sqrt(s2);
    ord[j] = j;
  }
  for (int64_t a = 0; a < n; ++a) {
    int64_t best = a;
    for (int64_t b = a + 1; b < n; ++b) if (sigma[ord[b]] > sigma[ord[best]]) best = b;
    int64_t tmp = ord[a]; ord[a] = ord[best]; ord[best] = tmp;
  }
  for (int64_t a = 0; a < k; ++a) {
    int64_t j = ord[a];
    double s = sigma[j];
    double rs = sqrt(s);
    /* column a of A = u_j * sqrt(s) = G[:,j] / s * sqrt(s); row a of B = sqrt(s) * v_j^T */
    for (int64_t i = 0; i < m; ++i) A[i * k + a] = (s > 0.0) ? G[i * n + j] / rs : 0.0;
    for (int64_t i = 0; i < n; ++i) B[a * n + i] = rs * R[i * n + j];
  }
  /* hand back sigma sorted */
  {
    double *tmp = (double *)malloc(sizeof(double) * (size_t)n);
    if (tmp) {
      for (int64_t a = 0; a < n; ++a) tmp[a] = sigma[ord[a]];
      memcpy(sigma, tmp, sizeof(double) * (size_t)n);
      free(tmp);
    }
  }
  free(G); free(R); free(ord);
  return sweeps;
}
