"""Pins for the paged-cache / rotary oracle (no GPU needed).

The scan and the copy are pinned against the definition of a block table (brute-force gather),
against structural invariants (cover, maximality, order) and against hand-made tables; the
rotary embedding against its defining properties (rotation, relative positions), against a case
worked out with table values of sine and cosine, and against complex multiplication.
"""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import paged_cache as pc


def test_hand_made_table():
    #  seq 0: blocks 5 6 7 | 2      seq 1: 3 4 | 9       seq 2: 10 11 (continues seq 1's last run)
    table = [[5, 6, 7, 2], [3, 4, 9, -1], [10, 11, -1, -1]]
    runs, remap = pc.contiguous_runs(table, [4, 3, 2])
    # 2, 3, 4 are consecutive ids across the sequence boundary: one run of three
    assert runs == [(5, 0, 3), (2, 3, 3), (9, 6, 3)]
    assert remap == [[0, 1, 2, 3], [4, 5, 6], [7, 8]]


def test_descending_and_repeated_ids_do_not_merge():
    runs, _ = pc.contiguous_runs([[4, 3, 2], [2, 2, 3]], [3, 3])
    assert runs == [(4, 0, 1), (3, 1, 1), (2, 2, 1), (2, 3, 1), (2, 4, 2)]


def test_empty_inputs():
    assert pc.contiguous_runs([], []) == ([], [])
    assert pc.contiguous_runs([[7, 8]], [0]) == ([], [[]])
    assert pc.copy_runs(np.zeros((3, 2)), [], 4).shape == (4, 2)


@pytest.mark.parametrize("seed,recycled", [(1, 0), (2, 10), (3, 64), (4, 200)])
def test_runs_reproduce_the_gather_definition(seed, recycled):
    prompt = [9, 1, 17, 4, 0, 30]
    decode = [5, 0, 2, 7, 3, 1]
    table, n_blocks = si.paged_block_tables(seed, prompt, decode, 256, recycled)
    runs, remap = pc.contiguous_runs(table, n_blocks)
    total = int(n_blocks.sum())
    # cover: destinations tile [0, total) in order, without gaps or overlap
    assert [r[1] for r in runs] == list(np.cumsum([0] + [r[2] for r in runs[:-1]]))
    assert sum(r[2] for r in runs) == total
    # maximal: two neighbouring runs are never mergeable
    for a, b in zip(runs, runs[1:]):
        assert a[0] + a[2] != b[0]
    # every block of every run is the block the table names
    walk = [int(table[s][i]) for s in range(len(n_blocks)) for i in range(n_blocks[s])]
    flat = [src + j for src, _, n in runs for j in range(n)]
    assert flat == walk
    # remap is the walk index
    assert list(itertools.chain.from_iterable(remap)) == list(range(total))
    # the copy equals the gather
    pool = np.arange(256 * 6, dtype=np.int64).reshape(256, 2, 3) * 7 + 1
    got = pc.copy_runs(pool, runs, total + 3)
    want = pc.gather_blocks(pool, table, n_blocks, total + 3)
    assert np.array_equal(got, want)
    assert np.all(got[total:] == 0)
    for s in range(len(n_blocks)):
        for i in range(n_blocks[s]):
            assert np.array_equal(got[remap[s][i]], pool[table[s][i]])


def test_prefill_blocks_form_long_runs_and_decode_blocks_short_ones():
    # the generator's structure shows in the scan: without recycled blocks every prompt is one run
    table, n_blocks = si.paged_block_tables(5, [12, 20, 7], [4, 4, 4], 128, recycled=0)
    runs, _ = pc.contiguous_runs(table, n_blocks)
    lengths = sorted(r[2] for r in runs)
    assert lengths[-3:] == [7, 12, 20]
    assert all(n == 1 for n in lengths[:-3])


def test_token_positions():
    pos = pc.token_positions([2, 1], 4, 4)
    assert list(pos) == [0, 1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3, 0, 0, 0, 0]


# ------------------------------------------------------------------------------- rotary embedding
def test_rope_worked_example():
    # head_dim 4, theta 10000, position 1: angles 1 and 0.01 rad.
    # cos 1 = 0.5403023, sin 1 = 0.8414710 (tables); cos 0.01 = 1 - 0.00005 + ..., sin 0.01 = 0.01 - 1.6667e-7
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    y = pc.rope(x, [1], 1, 4)
    c1, s1 = 0.5403023, 0.8414710
    c2, s2 = 0.99995000, 0.00999983
    want = [1 * c1 - 3 * s1, 2 * c2 - 4 * s2, 3 * c1 + 1 * s1, 4 * c2 + 2 * s2]
    assert np.allclose(y[0], want, atol=2e-6)
    assert np.allclose(y[0], [-1.9841107, 1.9599007, 2.4623779, 4.0197997], atol=2e-6)


def test_rope_position_zero_is_identity_and_quarter_turn():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 2 * 8))
    assert np.array_equal(pc.rope(x, [0, 0, 0], 2, 8), x)
    # theta = 1: every pair turns by pos radians; pos = pi/2 maps (a, b) -> (-b, a)
    y = pc.rope(x[:1], [np.pi / 2], 2, 8, theta=1.0)
    for h in range(2):
        a, b = x[0, 8 * h: 8 * h + 4], x[0, 8 * h + 4: 8 * h + 8]
        assert np.allclose(y[0, 8 * h: 8 * h + 4], -b, atol=1e-15)
        assert np.allclose(y[0, 8 * h + 4: 8 * h + 8], a, atol=1e-15)


def test_rope_is_complex_multiplication():
    rng = np.random.default_rng(1)
    D, H, T = 16, 3, 5
    x = rng.standard_normal((T, H * D))
    pos = np.array([0, 1, 7, 100, 4095])
    y = pc.rope(x, pos, H, D, theta=500000.0)
    freq = 500000.0 ** (-np.arange(D // 2) * 2.0 / D)
    for h in range(H):
        z = x[:, h * D: h * D + D // 2] + 1j * x[:, h * D + D // 2: (h + 1) * D]
        w = z * np.exp(1j * pos[:, None] * freq[None, :])
        assert np.allclose(y[:, h * D: h * D + D // 2], w.real, atol=1e-12)
        assert np.allclose(y[:, h * D + D // 2: (h + 1) * D], w.imag, atol=1e-12)


def test_rope_composes_and_keeps_relative_positions():
    rng = np.random.default_rng(2)
    D = 32
    q, k = rng.standard_normal((1, D)), rng.standard_normal((1, D))
    # rotating by m then by n equals rotating by m + n; norms of pairs are kept
    a = pc.rope(pc.rope(q, [13], 1, D), [29], 1, D)
    assert np.allclose(a, pc.rope(q, [42], 1, D), atol=1e-12)
    assert np.allclose(q[0, :16] ** 2 + q[0, 16:] ** 2, a[0, :16] ** 2 + a[0, 16:] ** 2, atol=1e-12)
    # the score of a rotated query and key depends on the distance of their positions only
    s1 = pc.rope(q, [105], 1, D) @ pc.rope(k, [100], 1, D).T
    s2 = pc.rope(q, [1005], 1, D) @ pc.rope(k, [1000], 1, D).T
    s3 = pc.rope(q, [5], 1, D) @ k.T
    assert np.allclose(s1, s2, atol=1e-10) and np.allclose(s1, s3, atol=1e-10)


def test_rope_heads_are_independent_and_pairing_is_half_apart():
    # a single non-zero element at index i of head h only reaches i and i +- D/2 of the same head
    D, H = 8, 3
    for h, i in itertools.product(range(H), range(D)):
        x = np.zeros((1, H * D)); x[0, h * D + i] = 1.0
        y = pc.rope(x, [3], H, D)
        nz = set(np.nonzero(np.abs(y[0]) > 1e-15)[0])
        assert nz <= {h * D + i, h * D + (i + D // 2) % D}


def test_rope_table_is_the_rotation_of_rope():
    """The table form of the angles: unit rows (cos^2 + sin^2 = 1), position 0 gives (1, 0), pair index 0
    turns by the position itself, and multiplying (x_i + j x_{i+D/2}) by (cos + j sin) of the table
    gives what `rope` gives."""
    H, D = 3, 16
    pos = np.array([0, 1, 7, 4097, 99999])
    tab = pc.rope_table(pos, D, theta=500000.0)
    half = D // 2
    assert tab.shape == (5, D)
    assert np.allclose(tab[:, :half] ** 2 + tab[:, half:] ** 2, 1.0, atol=1e-14)
    assert np.array_equal(tab[0], np.r_[np.ones(half), np.zeros(half)])
    assert np.allclose(tab[:, 0], np.cos(pos), atol=1e-9) and np.allclose(tab[:, half], np.sin(pos), atol=1e-9)
    # the last pair index turns by pos / theta^((D - 2) / D)
    assert np.allclose(tab[:, half - 1], np.cos(pos / 500000.0 ** ((D - 2) / D)), atol=1e-9)
    x = np.random.default_rng(5).standard_normal((5, H * D))
    z = x.reshape(5, H, D)[:, :, :half] + 1j * x.reshape(5, H, D)[:, :, half:]
    w = z * (tab[:, None, :half] + 1j * tab[:, None, half:])
    y = np.concatenate([w.real, w.imag], axis=2).reshape(5, H * D)
    assert np.allclose(y, pc.rope(x, pos, H, D, theta=500000.0), atol=1e-12)
