"""Pins for the fp64 CPU oracle (no GPU needed).

Each test ties the oracle to something other than itself: an independent library
routine (numpy / scipy in fp64), a closed form, an invariant, brute force on tiny
inputs, or numbers the paper prints.  The cases use non-square, pairwise distinct
sizes so that a transposed operand, a swapped factor, a dropped term or an
off-by-one index fails at least one of them.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(1234)


def rnd(*shape):
    return RNG.standard_normal(shape)


def rel_err(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


# --------------------------------------------------------------------- whole result
@pytest.mark.parametrize("T,d_in,r,d_out", [(1, 7, 3, 5), (5, 33, 9, 17), (16, 512, 64, 512), (3, 40, 1, 11)])
def test_matches_numpy_fp64_matmul(T, d_in, r, d_out):
    x, U, V = rnd(T, d_in), rnd(d_in, r), rnd(r, d_out)
    y, t = oracle.lowrank_linear(x, U, V, return_t=True)
    assert rel_err(t, x @ U) < 1e-13
    assert rel_err(y, (x @ U) @ V) < 1e-13
    assert y.shape == (T, d_out) and t.shape == (T, r)


def test_stage_functions_match_numpy_and_compose():
    x, U, V = rnd(4, 19), rnd(19, 6), rnd(6, 23)
    t = oracle.down_projection(x, U)
    y = oracle.up_projection(t, V)
    assert rel_err(t, x @ U) < 1e-13 and rel_err(y, x @ U @ V) < 1e-13
    assert np.array_equal(y, oracle.lowrank_linear(x, U, V))


def test_leading_dimensions_are_honoured():
    # call the C entry point on sub-views with ld > width, against numpy on the views
    L = oracle.lib()
    T, d_in, r, d_out = 3, 10, 4, 6
    xb, Ub, Vb = rnd(T, d_in + 5), rnd(d_in, r + 3), rnd(r, d_out + 2)
    yb = np.full((T, d_out + 7), np.nan)
    p = lambda a: a.ctypes.data_as(oracle._dp)
    rc = L.oracle_lowrank_linear(p(xb), T, d_in + 5, p(Ub), r + 3, p(Vb), d_out + 2,
                                 d_in, r, d_out, p(yb), d_out + 7, None)
    assert rc == 0
    ref = xb[:, :d_in] @ Ub[:, :r] @ Vb[:, :d_out]
    assert rel_err(yb[:, :d_out], ref) < 1e-13
    assert np.all(np.isnan(yb[:, d_out:]))      # nothing written outside the logical width


# --------------------------------------------------------------------- associativity
def test_associativity_invariant_separate_loop_nest():
    # (xU)V == x(UV), with W = UV built by an independent pure-Python triple loop
    T, d_in, r, d_out = 3, 6, 4, 5
    x, U, V = rnd(T, d_in), rnd(d_in, r), rnd(r, d_out)
    W = [[math.fsum(U[c, k] * V[k, j] for k in range(r)) for j in range(d_out)] for c in range(d_in)]
    xw = np.array([[math.fsum(x[i, c] * W[c][j] for c in range(d_in)) for j in range(d_out)] for i in range(T)])
    assert rel_err(oracle.lowrank_linear(x, U, V), xw) < 1e-13


# --------------------------------------------------------------------- SVD (Sec. 2.1, Eq. 1)
@pytest.mark.parametrize("m,n", [(12, 8), (8, 12), (9, 9)])
def test_full_rank_svd_reproduces_W(m, n):
    W = rnd(m, n)
    k = min(m, n)
    A, B, s = oracle.svd_factor(W, k)
    assert A.shape == (m, k) and B.shape == (k, n)
    assert rel_err(A @ B, W) < 1e-12
    assert np.allclose(s, np.linalg.svd(W, compute_uv=False), rtol=1e-12, atol=1e-13)
    # symmetric sqrt(Sigma) split: column norms of A equal row norms of B equal sqrt(sigma)
    assert np.allclose(np.linalg.norm(A, axis=0), np.sqrt(s[:k]), rtol=1e-10)
    assert np.allclose(np.linalg.norm(B, axis=1), np.sqrt(s[:k]), rtol=1e-10)
    x = rnd(5, m)
    assert rel_err(oracle.lowrank_linear(x, A, B), x @ W) < 1e-12


def test_truncated_svd_eckart_young():
    W = rnd(14, 10)
    s = np.linalg.svd(W, compute_uv=False)
    for k in (1, 3, 7):
        A, B, _ = oracle.svd_factor(W, k)
        err2 = np.sum((W - A @ B) ** 2)
        assert abs(err2 - np.sum(s[k:] ** 2)) < 1e-10 * np.sum(s ** 2)
        assert oracle.param_count(14, 10, k) == (14 + 10) * k


# --------------------------------------------------------------------- rank rule and printed numbers
def test_rank_rule_against_printed_and_hand_worked_values():
    for line in open(os.path.join(GOLDEN, "benchmark_ranks.txt")):
        if line.startswith("#") or not line.strip():
            continue
        m, n, a, b, r = map(int, line.split())
        assert oracle.rank_for_keep(m, n, a, b) == r
        assert r == math.floor(Fraction(a, b) * m * n / (m + n))
        # the rule keeps at most the requested fraction and r + 1 would exceed it
        assert oracle.param_count(m, n, r) * b <= a * m * n < oracle.param_count(m, n, r + 1) * b


def test_rank_rule_degenerate_arguments():
    assert oracle.rank_for_keep(0, 5, 1, 2) == -1
    assert oracle.rank_for_keep(5, 5, 1, 0) == -1
    assert oracle.rank_for_keep(64, 64, 0, 1) == 0
    assert oracle.rank_for_keep(64, 64, 1, 1) == 32      # full budget on a square matrix: n/2


def _golden_table1():
    d = {}
    for line in open(os.path.join(GOLDEN, "paper_table1_comm_volume.txt")):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.split("=")
        d[k.strip()] = int(v)
    return d


def test_paper_table1_numbers():
    g = _golden_table1()
    lb, lk = g["l_big"], g["l_kv"]
    out = oracle.comm_volume(g["h"], g["h_kv"], g["m"], lb, lk, lk, lb, lb, lb, lb)
    assert out["unoptimized"] == g["unoptimized_total"]
    assert out["all_gather"] == g["deinfer_all_gather"]
    assert out["reduce_sum"] == 2 * g["deinfer_reduce_sum_each"]
    assert out["lowrank_total"] == g["deinfer_total"]
    assert int(100 * (1 - out["lowrank_total"] / out["unoptimized"])) == g["saving_percent"]
    # the footnote's ranks are a rank-fraction rule (60 % of the width), not the
    # parameter-fraction rule used for the benchmark ranks: 0.6*8192 = 4915.2, 0.6*1024 = 614.4
    assert abs(lb - 0.6 * g["h"]) < 1 and abs(lk - 0.6 * g["h_kv"]) < 1


# --------------------------------------------------------------------- integer-exact brute force
def test_integer_brute_force_exact():
    T, d_in, r, d_out = 3, 5, 4, 6
    x = si.small_ints(7, 1, T * d_in, -4, 4).reshape(T, d_in)
    U = si.small_ints(7, 2, d_in * r, -4, 4).reshape(d_in, r)
    V = si.small_ints(7, 3, r * d_out, -4, 4).reshape(r, d_out)
    y = oracle.lowrank_linear(x, U, V)
    for i, j in itertools.product(range(T), range(d_out)):
        exact = sum(int(x[i, c]) * int(U[c, k]) * int(V[k, j]) for c in range(d_in) for k in range(r))
        assert y[i, j] == exact


# --------------------------------------------------------------------- special cases
def test_rank_one_is_outer_product():
    x, u, v = rnd(4, 9), rnd(9, 1), rnd(1, 6)
    y = oracle.lowrank_linear(x, u, v)
    assert rel_err(y, (x @ u[:, 0])[:, None] * v[0][None, :]) < 1e-13


def test_identity_factors_and_zero_input():
    x, V, U = rnd(3, 7), rnd(7, 5), rnd(7, 4)
    assert np.array_equal(oracle.lowrank_linear(x, np.eye(7), V), oracle.up_projection(x, V))
    assert rel_err(oracle.lowrank_linear(x, np.eye(7), V), x @ V) < 1e-13
    assert rel_err(oracle.lowrank_linear(x, U, np.eye(4)), x @ U) < 1e-13
    assert np.all(oracle.lowrank_linear(np.zeros((3, 7)), U, rnd(4, 6)) == 0.0)


def test_one_hot_rows_select_rows_of_UV():
    U, V = rnd(6, 3), rnd(3, 5)
    y = oracle.lowrank_linear(np.eye(6), U, V)
    assert rel_err(y, U @ V) < 1e-13


def test_linearity_in_x():
    x1, x2, U, V = rnd(2, 8), rnd(2, 8), rnd(8, 3), rnd(3, 4)
    lhs = oracle.lowrank_linear(2.5 * x1 - 0.75 * x2, U, V)
    rhs = 2.5 * oracle.lowrank_linear(x1, U, V) - 0.75 * oracle.lowrank_linear(x2, U, V)
    assert rel_err(lhs, rhs) < 1e-12


def test_zero_rank_and_empty_batch():
    x = rnd(3, 5)
    y = oracle.lowrank_linear(x, np.zeros((5, 0)), np.zeros((0, 4)))
    assert y.shape == (3, 4) and np.all(y == 0)
    assert oracle.lowrank_linear(np.zeros((0, 5)), rnd(5, 2), rnd(2, 4)).shape == (0, 4)


def test_zero_padded_rank_rows_change_nothing():
    x, U, V = rnd(3, 6), rnd(6, 4), rnd(4, 5)
    Up = np.concatenate([U, np.zeros((6, 3))], axis=1)
    Vp = np.concatenate([V, rnd(3, 5)], axis=0)      # padded U columns are zero: V rows there are free
    assert rel_err(oracle.lowrank_linear(x, Up, Vp), oracle.lowrank_linear(x, U, V)) < 1e-14


# --------------------------------------------------------------------- SiLU and the GLU sub-layer
def test_silu_closed_forms():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-16          # sigmoid(1)
    for z in (-30.0, -3.2, -0.5, 0.1, 2.0, 17.0):
        assert abs(oracle.silu(z) - z * scipy.special.expit(z)) < 1e-15 * max(1.0, abs(z))
        assert abs(oracle.silu(z) - oracle.silu(-z) - z) < 1e-14 * max(1.0, abs(z))   # silu(z) - silu(-z) = z
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12
    assert -1e-14 < oracle.silu(-40.0) < 0.0


def test_gateup_silu_against_library_pieces():
    x = rnd(4, 10)
    Ug, Vg, Uu, Vu = rnd(10, 3), rnd(3, 7), rnd(10, 5), rnd(5, 7)    # different ranks per pair
    h = oracle.lowrank_gateup_silu(x, Ug, Vg, Uu, Vu)
    g, u = x @ Ug @ Vg, x @ Uu @ Vu
    assert rel_err(h, g * scipy.special.expit(g) * u) < 1e-13
    # swapping gate and up must change the result (guards against a swapped operand)
    assert rel_err(oracle.lowrank_gateup_silu(x, Uu, Vu, Ug, Vg), h) > 1e-3
    # zero gate -> zero output; constant gate path reduces to a scaled "up"
    assert np.all(oracle.lowrank_gateup_silu(x, 0 * Ug, Vg, Uu, Vu) == 0.0)


def test_down_is_plain_pair():
    h, U, V = rnd(3, 11), rnd(11, 4), rnd(4, 6)
    assert np.array_equal(oracle.lowrank_down(h, U, V), oracle.lowrank_linear(h, U, V))
    assert rel_err(oracle.lowrank_down(h, U, V), h @ U @ V) < 1e-13


# --------------------------------------------------------------------- QKV grouping (Sec. 4.1)
def test_qkv_equals_concatenated_down_projection():
    x = rnd(5, 12)
    Uq, Vq = rnd(12, 4), rnd(4, 12)
    Uk, Vk = rnd(12, 2), rnd(2, 6)      # GQA-like: narrower k/v with their own ranks
    Uv, Vv = rnd(12, 3), rnd(3, 6)
    q, k, v, tk, tv = oracle.lowrank_qkv(x, Uq, Vq, Uk, Vk, Uv, Vv, return_t=True)
    tcat = oracle.down_projection(x, np.concatenate([Uq, Uk, Uv], axis=1))
    # slicing the concatenated product gives each pair's t bit for bit (same summation order)
    assert np.array_equal(tcat[:, 4:6], tk) and np.array_equal(tcat[:, 6:9], tv)
    assert np.array_equal(oracle.up_projection(tcat[:, :4], Vq), q)
    assert rel_err(q, x @ Uq @ Vq) < 1e-13 and rel_err(k, x @ Uk @ Vk) < 1e-13 and rel_err(v, x @ Uv @ Vv) < 1e-13
    assert rel_err(tk, x @ Uk) < 1e-13 and rel_err(tv, x @ Uv) < 1e-13


# --------------------------------------------------------------------- bf16 diagnostic rounding
def test_round_to_bf16_matches_bit_twiddling():
    vals = np.concatenate([RNG.standard_normal(2000) * 3, [1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e38 / 4]])
    for v in vals.astype(np.float32):
        expect = si.bf16_bits_to_f32(si.f32_to_bf16_bits(np.array([v], dtype=np.float32)))[0]
        assert oracle.round_to_bf16(float(v)) == float(expect)
    # ties go to even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2 * 2.0 ** -7


# --------------------------------------------------------------------- planted mistakes must be caught
def test_pins_catch_planted_mistakes():
    """Mutants written here (never in the oracle): each must disagree with the oracle on the
    pin shapes, which shows the shapes above can tell such mistakes apart."""
    x, U, V = rnd(4, 6), rnd(6, 6), rnd(6, 6)       # square on purpose: transposes are shape-legal
    y = oracle.lowrank_linear(x, U, V)
    mutants = {
        "transposed U": x @ U.T @ V,
        "transposed V": x @ U @ V.T,
        "swapped factors": x @ V @ U,
        "dropped last rank term": x @ U[:, :-1] @ V[:-1],
        "dropped last input column": x[:, :-1] @ U[:-1] @ V,
    }
    for name, m in mutants.items():
        assert rel_err(m, y) > 1e-3, name


# --------------------------------------------------------------------- input generator sanity
def test_generator_is_seeded_and_counter_based():
    a = si.normal(3, 5, 1001)
    assert np.array_equal(a, si.normal(3, 5, 1001))
    assert np.array_equal(a[:500], si.normal(3, 5, 500))
    assert not np.array_equal(a, si.normal(4, 5, 1001)) and not np.array_equal(a, si.normal(3, 6, 1001))
    big = si.normal(0, 9, 400000)
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1.0) < 0.01
    t = si.make(0, 1, (8, 16), 0.02, "bf16")
    assert t.bits.dtype == np.uint16 and t.values.dtype == np.float32
    assert np.array_equal(si.f32_to_bf16_bits(t.values), t.bits)      # already representable


# --------------------------------------------------------------------- non-GLU sub-layer: bias and activation
def test_gelu_is_z_times_the_normal_distribution_function():
    import scipy.stats
    for z in (-6.0, -2.5, -1.0, -0.3, 0.0, 0.3, 1.0, 2.5, 6.0):
        assert math.isclose(oracle.gelu(z), z * scipy.stats.norm.cdf(z), rel_tol=1e-13, abs_tol=1e-16)
    # values from a table of the normal distribution: Phi(1) = 0.8413447, Phi(2) = 0.9772499
    assert abs(oracle.gelu(1.0) - 0.8413447) < 1e-7 and abs(oracle.gelu(-1.0) + 0.1586553) < 1e-7
    assert abs(oracle.gelu(2.0) - 1.9544998) < 1e-7
    assert oracle.gelu(0.0) == 0.0 and abs(oracle.gelu(40.0) - 40.0) < 1e-12 and abs(oracle.gelu(-40.0)) < 1e-12
    assert oracle.relu(-3.0) == 0.0 and oracle.relu(2.5) == 2.5 and oracle.relu(0.0) == 0.0


def test_linear_act_against_numpy_and_special_cases():
    x, U, V, b = rnd(5, 21), rnd(21, 4), rnd(4, 13), rnd(13)
    z = (x @ U) @ V
    assert rel_err(oracle.lowrank_linear_act(x, U, V), z) < 1e-13
    assert rel_err(oracle.lowrank_linear_act(x, U, V, b), z + b[None, :]) < 1e-13
    assert rel_err(oracle.lowrank_linear_act(x, U, V, b, oracle.ACT_RELU), np.maximum(z + b[None, :], 0.0)) < 1e-13
    g = oracle.lowrank_linear_act(x, U, V, b, oracle.ACT_GELU)
    want = (z + b) * 0.5 * (1.0 + scipy.special.erf((z + b) / math.sqrt(2.0)))
    assert rel_err(g, want) < 1e-13
    # the bias is added before the activation and runs along the output features, not the tokens
    only_b = oracle.lowrank_linear_act(x, U, np.zeros_like(V), b, oracle.ACT_RELU)
    assert np.array_equal(only_b, np.tile(np.maximum(b, 0.0), (5, 1)))
    # ReLU is positively homogeneous, GELU is not
    r1 = oracle.lowrank_linear_act(3.0 * x, U, V, 3.0 * b, oracle.ACT_RELU)
    assert rel_err(r1, 3.0 * oracle.lowrank_linear_act(x, U, V, b, oracle.ACT_RELU)) < 1e-13
    with pytest.raises(RuntimeError):
        oracle.lowrank_linear_act(x, U, V, b, 7)


def test_stage_two_of_the_glu_layer_alone():
    import scipy.special
    x, Ug, Vg, Uu, Vu = rnd(6, 17), rnd(17, 5), rnd(5, 11), rnd(17, 3), rnd(3, 11)
    tg, tu = x @ Ug, x @ Uu
    h = oracle.up_glu_silu(tg, Vg, tu, Vu)
    assert rel_err(h, oracle.lowrank_gateup_silu(x, Ug, Vg, Uu, Vu)) < 1e-13      # same thing, staged
    g, u = tg @ Vg, tu @ Vu
    assert rel_err(h, g * scipy.special.expit(g) * u) < 1e-13                      # silu(z) = z * logistic(z)
    # gate and up are not interchangeable
    assert rel_err(oracle.up_glu_silu(tu, Vu, tg, Vg), h) > 1e-3
