"""Host side of the paged-cache path (Sec. 4.2, preparation stage): the library's scan against the
oracle's, bit for bit; runs on the CPU (the plan function touches no device)."""
import ctypes

import numpy as np
import pytest

import paper_2604_17709_amd as dn
import synth_inputs as si
from oracle import paged_cache as pc

CASES = [
    # seed, prompt blocks, decode blocks, pool, recycled
    (1, [9, 1, 17, 4, 0, 30], [5, 0, 2, 7, 3, 1], 256, 0),
    (2, [9, 1, 17, 4, 0, 30], [5, 0, 2, 7, 3, 1], 256, 40),
    (3, [32] * 16, [1] * 16, 1024, 0),
    (4, [3, 3, 3], [40, 40, 40], 200, 200),
    (5, [0], [0], 4, 0),
]


@pytest.mark.parametrize("seed,prompt,decode,n_pool,recycled", CASES)
def test_plan_matches_the_oracle_scan(seed, prompt, decode, n_pool, recycled):
    table, n_blocks = si.paged_block_tables(seed, prompt, decode, n_pool, recycled)
    total = int(n_blocks.sum())
    bt = 16
    plan, remap, pos = dn.deinfer_kv_compact_plan(table, n_blocks, n_pool, total + 5, bt)
    runs, remap_o = pc.contiguous_runs(table, n_blocks)
    assert plan[0] == len(runs) and plan[1] == total and plan[2] == 0 and plan[3] == 0
    got = [tuple(int(v) for v in plan[4 + 3 * i: 7 + 3 * i]) for i in range(plan[0])]
    assert got == runs
    assert np.all(plan[4 + 3 * plan[0]:] == 0)
    for s in range(len(n_blocks)):
        assert list(remap[s, :n_blocks[s]]) == remap_o[s]
        assert np.all(remap[s, n_blocks[s]:] == -1)
    assert np.array_equal(pos, pc.token_positions(n_blocks, bt, total + 5))


def test_plan_of_hand_made_table():
    table = np.array([[5, 6, 7, 2], [3, 4, 9, -1], [10, 11, -1, -1]], dtype=np.int32)
    plan, remap, _ = dn.deinfer_kv_compact_plan(table, np.array([4, 3, 2], dtype=np.int32), 12, 9, 1)
    assert list(plan[:4 + 9]) == [3, 9, 0, 0, 5, 0, 3, 2, 3, 3, 9, 6, 3]
    assert remap.tolist() == [[0, 1, 2, 3], [4, 5, 6, -1], [7, 8, -1, -1]]


def test_plan_errors():
    L = dn.lib()
    ip = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    table = np.array([[0, 1, 2, 5]], dtype=np.int32)
    nb = np.array([4], dtype=np.int32)
    plan = np.zeros(4 + 3 * 8, dtype=np.int32)

    def call(n_pool=8, buf=8, cap=8, nbv=nb, tbl=table, pitch=4):
        return L.deinfer_kv_compact_plan(ip(tbl), 1, pitch, ip(nbv), n_pool, buf, 16, ip(plan), cap, None, 0, None)

    assert call() == dn.OK
    assert call(n_pool=5) == dn.ERR_INVALID_ARG and "outside the pool" in dn.last_error()
    assert call(buf=3) == dn.ERR_WORKSPACE and "compact buffer" in dn.last_error()
    assert call(cap=1) == dn.ERR_WORKSPACE and "runs" in dn.last_error()
    assert call(nbv=np.array([5], dtype=np.int32)) == dn.ERR_INVALID_ARG
    assert call(nbv=np.array([-1], dtype=np.int32)) == dn.ERR_INVALID_ARG
    assert call(tbl=np.array([[0, -3, 2, 5]], dtype=np.int32)) == dn.ERR_INVALID_ARG
    assert L.deinfer_kv_compact_plan(ip(table), 1, 4, ip(nb), 8, 8, 16, None, 8, None, 0, None) == dn.ERR_INVALID_ARG
    # no sequences: an empty plan
    assert L.deinfer_kv_compact_plan(None, 0, 0, None, 8, 8, 16, ip(plan), 8, None, 0, None) == dn.OK
    assert plan[0] == 0 and plan[1] == 0


def test_copy_and_rope_argument_validation():
    L = dn.lib()
    FAKE = 0x7f0000000000
    assert L.deinfer_kv_compact_copy(FAKE, 8, 100, FAKE, 4, FAKE, 8, None) == dn.ERR_MISALIGNED      # block_bytes % 16
    assert L.deinfer_kv_compact_copy(FAKE, 8, 0, FAKE, 4, FAKE, 8, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_kv_compact_copy(None, 8, 64, FAKE, 4, FAKE, 8, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_kv_compact_copy(FAKE + 8, 8, 64, FAKE, 4, FAKE, 8, None) == dn.ERR_MISALIGNED
    assert L.deinfer_kv_compact_copy(FAKE, 8, 64, FAKE, 4, FAKE, 0, None) == dn.OK                     # nothing to do
    assert L.deinfer_rope_inplace(FAKE, 4, 64, 2, 31, FAKE, 10000.0, dn.BF16, None) == dn.ERR_INVALID_ARG   # odd head_dim
    assert L.deinfer_rope_inplace(FAKE, 4, 60, 2, 32, FAKE, 10000.0, dn.BF16, None) == dn.ERR_INVALID_ARG   # ldx < width
    assert L.deinfer_rope_inplace(FAKE, 4, 64, 2, 32, FAKE, 0.0, dn.BF16, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_inplace(FAKE, 4, 64, 2, 32, FAKE, 10000.0, 9, None) == dn.ERR_UNSUPPORTED
    assert L.deinfer_rope_inplace(FAKE, 4, 64, 2, 32, None, 10000.0, dn.BF16, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_inplace(None, 0, 64, 2, 32, None, 10000.0, dn.BF16, None) == dn.OK
