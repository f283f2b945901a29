"""Paged low-rank cache -> compact buffer -> rebuilt keys with rotary embedding (Sec. 4.2), on the
GPU through the C-ABI, against the CPU oracle: byte-exact for the copy, within the bf16 / fp32
tolerance for the arithmetic, and replayed from one captured graph with changing block tables."""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from oracle import paged_cache as pc
from gpu_util import TOKEN_TILE_BOTH, TOL, max_err, pair, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dn():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_17709_amd as dn
    dn.lib()
    return dn


@pytest.fixture(autouse=True, params=[(0, 0), (256, 0), (128, 256), (TOKEN_TILE_BOTH, 0)], ids=["tiles-auto", "tiles-256", "tiles-128x256", "tiles-mixed"])
def token_tile(request, dn):
    """Every test runs with the workgroup tile of the T > 128 kernel chosen per launch (small shapes then
    take the 128 x 128 tile), with 256-token tiles forced, with 128 x 256 tiles forced, and with both
    shapes in one launch (the second half of the feature blocks as 128 x 256 tiles)."""
    dn.deinfer_set_prefill_token_tile(request.param[0])
    dn.deinfer_set_prefill_feature_tile(request.param[1])
    yield request.param
    dn.deinfer_set_prefill_token_tile(0)
    dn.deinfer_set_prefill_feature_tile(0)


def pool_bits(seed, n_pool, block_tokens, pitch):
    """Seeded bf16 bit patterns for a whole pool (finite values)."""
    t = si.make(seed, 7, (n_pool * block_tokens, pitch), 1.0, "bf16")
    return np.ascontiguousarray(t.bits).reshape(n_pool, block_tokens, pitch)


@pytest.mark.parametrize("seed,prompt,decode,n_pool,recycled,block_tokens,pitch", [
    (1, [9, 1, 17, 4, 0, 30], [5, 0, 2, 7, 3, 1], 128, 0, 16, 24),        # 768-byte blocks
    (2, [9, 1, 17, 4, 0, 30], [5, 0, 2, 7, 3, 1], 128, 40, 16, 512),      # exactly one 16 KiB piece
    (3, [20, 3, 11], [6, 6, 6], 96, 10, 16, 1640),                        # 52480 bytes: three pieces and a ragged fourth
    (4, [3, 3, 3], [40, 40, 40], 200, 200, 8, 104),                       # nothing contiguous: one run per block
    (5, [0], [0], 4, 0, 16, 64),                                          # no blocks at all
])
def test_compact_copy_matches_gather(dn, seed, prompt, decode, n_pool, recycled, block_tokens, pitch):
    import torch
    table, n_blocks = si.paged_block_tables(seed, prompt, decode, n_pool, recycled)
    total = int(n_blocks.sum())
    cap = total + 3
    bits = pool_bits(seed, n_pool, block_tokens, pitch)
    pool = torch.from_numpy(bits.view(np.int16)).cuda()
    buf = torch.full((cap, block_tokens, pitch), 0x1234, dtype=torch.int16, device="cuda")
    plan, remap, _ = dn.deinfer_kv_compact_plan(table, n_blocks, n_pool, cap, block_tokens)
    plan_d = torch.from_numpy(plan).cuda()
    dn.deinfer_kv_compact_copy(pool, block_tokens * pitch * 2, plan_d, buf)
    torch.cuda.synchronize()
    got = buf.cpu().numpy().view(np.uint16)
    want = pc.gather_blocks(bits, table, n_blocks, cap)
    assert np.array_equal(got[:total], want[:total])
    assert np.all(got[total:] == 0x1234)                      # blocks beyond the plan are left alone
    for s in range(len(n_blocks)):                            # the remapping list is the buffer's block table
        for i in range(n_blocks[s]):
            assert np.array_equal(got[remap[s, i]], bits[table[s, i]])


def test_copy_skips_runs_that_point_outside(dn):
    import torch
    n_pool, bt, pitch = 8, 4, 16
    bits = pool_bits(9, n_pool, bt, pitch)
    pool = torch.from_numpy(bits.view(np.int16)).cuda()
    buf = torch.full((6, bt, pitch), 0x1234, dtype=torch.int16, device="cuda")
    # runs: (2 -> 0, 2 blocks) fine, (7 -> 2, 2 blocks) second block is outside the pool, (-1 -> 4, 1) outside
    plan = np.array([3, 5, 0, 0, 2, 0, 2, 7, 2, 2, -1, 4, 1] + [0] * 9, dtype=np.int32)
    dn.deinfer_kv_compact_copy(pool, bt * pitch * 2, torch.from_numpy(plan).cuda(), buf)
    torch.cuda.synchronize()
    got = buf.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[0], bits[2]) and np.array_equal(got[1], bits[3]) and np.array_equal(got[2], bits[7])
    assert np.all(got[3:] == 0x1234)


@pytest.mark.parametrize("dtype,T,H,D,extra,theta", [
    ("bf16", 37, 3, 32, 0, 10000.0),
    ("bf16", 130, 8, 128, 8, 500000.0),
    ("bf16", 5, 2, 20, 3, 10000.0),          # half = 10: a full group of 8 pair indices and a ragged one, unaligned rows
    ("f32", 33, 2, 64, 4, 10000.0),
    ("f16", 130, 8, 128, 8, 10000.0),
    ("f16", 5, 2, 20, 3, 10000.0),
])
def test_rope_matches_oracle(dn, dtype, T, H, D, extra, theta):
    import torch
    x = si.make(21, 3, (T, H * D + extra), 1.0, dtype)
    pos = (si.small_ints(21, 4, T, 0, 100000)).astype(np.int32)
    pos[0] = 0
    xd = to_dev(x)
    before = xd.clone()
    dn.deinfer_rope_inplace(xd[:, :H * D], H, D, torch.from_numpy(pos).cuda(), theta)
    torch.cuda.synchronize()
    got = to_host(xd)
    ref = pc.rope(x.values[:, :H * D].astype(np.float64), pos, H, D, theta)
    assert max_err(got[:, :H * D], ref) <= TOL[dtype]
    assert np.array_equal(got[0, :H * D], x.values[0, :H * D].astype(np.float64))        # position 0: untouched values
    assert torch.equal(xd[:, H * D:], before[:, H * D:])                                 # columns beyond the heads: untouched


def _scatter_into_pool(torch, pool, rows, table, n_blocks, block_tokens):
    """Paged-cache emulator: token j of sequence s goes to block table[s][j // bt], slot j % bt."""
    start = 0
    for s in range(len(n_blocks)):
        for i in range(n_blocks[s]):
            pool[int(table[s, i])] = rows[start:start + block_tokens]
            start += block_tokens
    return start


@pytest.mark.parametrize("H,D,fused", [(4, 64, False), (2, 128, True), (4, 64, True)])
def test_rebuild_keys_from_paged_cache_under_one_graph(dn, H, D, fused):
    """Preparation stage on the host, then ONE captured graph (copy, upward projection at the
    buffer's capacity, rotary embedding) replayed for two different cache states and back."""
    import torch
    d_in, r, bt = 264, 96, 16
    d_out = H * D
    n_pool, cap_blocks = 64, 24
    cap_tokens = cap_blocks * bt                                   # 384 tokens: the large-T path
    states = [(11, [6, 2, 5], [3, 1, 2], 12), (12, [1, 9, 4, 2], [2, 0, 3, 1], 30)]
    _, U, V = si.make(50, 1, (1, 1), 1.0, "bf16"), si.make(50, 2, (d_in, r), 1.0 / np.sqrt(d_in), "bf16"), \
        si.make(50, 3, (r, d_out), 1.0 / np.sqrt(r), "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = dn.Workspace(dn.deinfer_workspace_bytes(cap_tokens, [p, p, p]))
    pool = torch.zeros((n_pool, bt, r), dtype=torch.bfloat16, device="cuda")
    buf = torch.zeros((cap_blocks * bt, r), dtype=torch.bfloat16, device="cuda")
    keys = torch.zeros((cap_tokens, d_out), dtype=torch.bfloat16, device="cuda")
    plan_d = torch.zeros(dn.KV_PLAN_HEADER + 3 * cap_blocks, dtype=torch.int32, device="cuda")
    pos_d = torch.zeros(cap_tokens, dtype=torch.int32, device="cuda")
    table_d = torch.zeros((cap_tokens, D), dtype=torch.float32, device="cuda")

    prepared = []
    for seed, prompt, decode, recycled in states:
        table, n_blocks = si.paged_block_tables(seed, prompt, decode, n_pool, recycled)
        n_tok = int(n_blocks.sum()) * bt
        x = si.make(seed, 1, (n_tok, d_in), 1.0, "bf16")
        tk = torch.zeros((n_tok, r), dtype=torch.bfloat16, device="cuda")
        dn.deinfer_lowrank_qkv(to_dev(x), p, p, p, ws, t_k=tk)     # the low-rank cache rows of these tokens
        plan, remap, pos = dn.deinfer_kv_compact_plan(table, n_blocks, n_pool, cap_blocks, bt)
        prepared.append((table, n_blocks, n_tok, x, tk, plan, pos))

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()

    def enqueue():
        dn.deinfer_kv_compact_copy(pool, bt * r * 2, plan_d, buf, stream=stream)
        if fused:      # fused = the table of angles and the projection that rotates (in its epilogue for heads of 128)
            dn.deinfer_rope_table(pos_d, D, 10000.0, table=table_d, stream=stream)
            dn.deinfer_lowrank_up_rope(buf, p, table_d, ws, out=keys, stream=stream)
        else:
            dn.deinfer_lowrank_up(buf, p, ws, out=keys, stream=stream)
            dn.deinfer_rope_inplace(keys, H, D, pos_d, 10000.0, stream=stream)

    results = []
    for step, idx in enumerate((0, 1, 0)):
        table, n_blocks, n_tok, x, tk, plan, pos = prepared[idx]
        # ---- preparation stage: anything goes (cache contents, plan and positions to the device)
        pool.zero_()
        assert _scatter_into_pool(torch, pool, tk, table, n_blocks, bt) == n_tok
        plan_d.copy_(torch.from_numpy(plan)); pos_d.copy_(torch.from_numpy(pos))
        torch.cuda.synchronize()
        if step == 0:
            with torch.cuda.stream(stream):
                enqueue()                                          # warm-up outside the capture
            stream.synchronize()
            with torch.cuda.graph(graph, stream=stream):
                enqueue()
        # ---- graph replay stage
        graph.replay()
        torch.cuda.synchronize()
        got = to_host(keys[:n_tok])
        results.append(keys[:n_tok].clone())
        # the compact buffer holds the walk: sequence after sequence, which is the order tk was made in
        assert torch.equal(buf[:n_tok], tk)
        ref_same_t = pc.rope(oracle.up_projection(to_host(tk), V.values.astype(np.float64)), pos[:n_tok], H, D)
        assert max_err(got, ref_same_t) <= TOL["bf16"]
        ref_full = pc.rope(oracle.lowrank_linear(x.values, U.values, V.values), pos[:n_tok], H, D)
        assert max_err(got, ref_full) <= TOL["bf16"]
    assert torch.equal(results[0], results[2])                     # same state, same graph: same bits


def test_rebuild_at_the_benchmark_size(dn):
    """The configuration bench.py times for the rebuild step (7B block, keep 0.8: r = 1638 for k,
    4096 key features in 32 heads of 128; 16 sequences of 32 blocks of 16 tokens; pool of 1024
    blocks, 128 of them recycled): copy compared byte for byte in full, the keys on sampled
    token rows (first / last rows, rows around block, tile and sequence borders)."""
    import torch
    r, d_kv, H, D, bt = 1638, 4096, 32, 128, 16
    pitch = 1640
    n_seqs, per_seq, n_pool = 16, 32, 1024
    cap_blocks = n_seqs * per_seq
    T = cap_blocks * bt
    table, n_blocks = si.paged_block_tables(1, [24] * n_seqs, [8] * n_seqs, n_pool, recycled=n_pool // 8)
    plan, remap, pos = dn.deinfer_kv_compact_plan(table, n_blocks, n_pool, cap_blocks, bt)
    runs, _ = pc.contiguous_runs(table, n_blocks)
    assert plan[0] == len(runs) and plan[1] == cap_blocks
    bits = pool_bits(1, n_pool, bt, pitch)
    bits[:, :, r:] = 0                                              # the padding columns of the cache rows are zero
    pool = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    V = si.make(1, 21, (r, d_kv), 0.02, "bf16")
    U = si.make(1, 20, (64, r), 0.02, "bf16")                       # not used by the upward projection
    p, keep = pair(dn, U, V, packed=True)
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [p]))
    buf = torch.zeros((T, pitch), dtype=torch.bfloat16, device="cuda")
    keys = torch.empty((T, d_kv), dtype=torch.bfloat16, device="cuda")
    dn.deinfer_kv_compact_copy(pool, bt * pitch * 2, torch.from_numpy(plan).cuda(), buf)
    dn.deinfer_lowrank_up(buf, p, ws, out=keys)
    dn.deinfer_rope_inplace(keys, H, D, torch.from_numpy(pos).cuda(), 10000.0)
    torch.cuda.synchronize()
    want = pc.gather_blocks(bits, table, n_blocks, cap_blocks)
    got = buf.view(torch.int16).cpu().numpy().view(np.uint16).reshape(cap_blocks, bt, pitch)
    assert np.array_equal(got, want)
    rows = {0, T - 1}
    for b in list(range(bt, T, 1024)) + list(range(128, T, 896)) + list(range(per_seq * bt, T, per_seq * bt)):
        rows.update((b - 1, b))
    rows = sorted(rows)
    t_rows = si.bf16_bits_to_f32(want.reshape(T, pitch)[rows][:, :r]).astype(np.float64)
    ref = pc.rope(oracle.up_projection(t_rows, V.values.astype(np.float64)), pos[rows], H, D)
    assert max_err(to_host(keys[rows]), ref) <= TOL["bf16"]
    # the same keys from the projection that rotates in its epilogue
    keys2 = torch.empty_like(keys)
    tab = dn.deinfer_rope_table(torch.from_numpy(pos).cuda(), D, 10000.0)
    dn.deinfer_lowrank_up_rope(buf, p, tab, ws, out=keys2)
    torch.cuda.synchronize()
    assert max_err(to_host(keys2[rows]), ref) <= TOL["bf16"]
    assert float((keys2.float() - keys.float()).abs().max()) <= 2.0 ** -7 * float(keys.float().abs().max())


@pytest.mark.parametrize("T,D,theta", [(1, 128, 10000.0), (300, 128, 500000.0), (77, 20, 10000.0)])
def test_rope_table_matches_oracle(dn, T, D, theta):
    import torch
    pos = (si.small_ints(23, 4, T, 0, 100000)).astype(np.int32)
    pos[0] = 0
    tab = dn.deinfer_rope_table(torch.from_numpy(pos).cuda(), D, theta)
    torch.cuda.synchronize()
    got = tab.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - pc.rope_table(pos, D, theta))) <= 2e-7        # fp32 rounding of values in [-1, 1]
    assert np.array_equal(got[0], np.r_[np.ones(D // 2), np.zeros(D // 2)])


@pytest.mark.parametrize("dtype,packed,T,r,H,D,extra", [
    ("bf16", True, 300, 72, 3, 128, 0),       # rotation inside the product's kernel: three token blocks, ragged tail
    ("bf16", True, 1024, 200, 32, 128, 64),   # 16 feature blocks of 256, output pitch wider than the keys
    ("bf16", True, 129, 8, 1, 128, 0),        # one head: a half-empty feature block
    ("f16", True, 257, 40, 5, 128, 8),
    ("bf16", True, 300, 72, 6, 64, 0),        # heads of 64: product, then rotation from the table
    ("bf16", True, 300, 72, 3, 128, 4),       # output rows not 16-byte aligned: same
    ("bf16", True, 64, 72, 3, 128, 0),        # T <= 128: same
    ("bf16", True, 7, 33, 2, 32, 0),
    ("f16", True, 100, 40, 4, 64, 0),
    ("f32", False, 150, 19, 2, 24, 3),        # row-major fp32 pairs
    ("bf16", False, 150, 19, 2, 128, 0),
])
def test_up_rope_matches_oracle(dn, dtype, packed, T, r, H, D, extra):
    """y = rope(t V) in one call, against the oracle's upward projection followed by its rotation,
    and against the two separate calls of the library (same roundings: close to the last bit)."""
    import torch
    d_out = H * D
    V = si.make(31, 1, (r, d_out), 0.25, dtype)
    U = si.make(31, 2, (16, r), 0.25, dtype)
    r8 = max(8, (r + 7) // 8 * 8)
    t = si.make(31, 3, (T, r8), 1.0, dtype)
    pos = (si.small_ints(31, 4, T, 0, 8192)).astype(np.int32)
    pos[0] = 0
    p, keep = pair(dn, U, V, packed=packed)
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [p]))
    td = to_dev(t)
    pos_d = torch.from_numpy(pos).cuda()
    tab = dn.deinfer_rope_table(pos_d, D, 10000.0)
    y = torch.full((T, d_out + extra), 3.0, dtype=td.dtype, device="cuda")
    dn.deinfer_lowrank_up_rope(td[:, :r], p, tab, ws, out=y[:, :d_out])
    torch.cuda.synchronize()
    ws.check()
    ref = pc.rope(oracle.up_projection(t.values[:, :r].astype(np.float64), V.values.astype(np.float64)), pos, H, D)
    got = to_host(y)
    assert max_err(got[:, :d_out], ref) <= TOL[dtype]
    assert np.all(got[:, d_out:] == 3.0)
    y2 = dn.deinfer_lowrank_up(td[:, :r], p, ws)
    dn.deinfer_rope_inplace(y2, H, D, pos_d, 10000.0)
    torch.cuda.synchronize()
    assert max_err(got[:, :d_out], to_host(y2)) <= (2.0 ** -7 if dtype == "bf16" else 2.0 ** -10 if dtype == "f16" else 1e-6)


def test_up_rope_of_a_rank_zero_pair_is_zero(dn):
    import torch
    p0 = dn.deinfer_pack_factors(dn.raw_pair(torch.zeros((64, 0), dtype=torch.bfloat16, device="cuda"),
                                             torch.zeros((0, 256), dtype=torch.bfloat16, device="cuda")))
    T = 200
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [p0]))
    tab = dn.deinfer_rope_table(torch.arange(T, dtype=torch.int32, device="cuda"), 128)
    y = torch.full((T, 256), 7.0, dtype=torch.bfloat16, device="cuda")
    dn.deinfer_lowrank_up_rope(torch.zeros((T, 8), dtype=torch.bfloat16, device="cuda"), p0, tab, ws, out=y)
    assert float(y.abs().max()) == 0.0
