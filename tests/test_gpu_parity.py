"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element,
on seeded inputs.  Gate: max|y - ref| / max|ref| <= 1e-2 for bf16 storage (fp32 accumulate,
bf16 rank-space intermediate on the packed path) and <= 1e-5 for fp32."""
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


def ws_for(dn, T, pairs):
    return dn.Workspace(dn.deinfer_workspace_bytes(T, pairs))


def gen(seed, T, d_in, r, d_out, dtype, stream0=1):
    x = si.make(seed, stream0, (T, d_in), 1.0, dtype)
    U = si.make(seed, stream0 + 1, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
    V = si.make(seed, stream0 + 2, (r, d_out), 1.0 / np.sqrt(max(r, 1)), dtype)
    return x, U, V


# ------------------------------------------------------------------ the small fp32 case
def test_single_linear_fp32(dn):
    x, U, V = si.single_linear_f32(seed=0)            # 16 x 512, r = 64, 512 outputs
    p, keep = pair(dn, U, V, packed=False)
    ws = ws_for(dn, 16, [p])
    y = dn.deinfer_lowrank_linear(to_dev(x), p, ws)
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(y), ref) <= TOL["f32"]


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("T,d_in,r,d_out", [(1, 7, 3, 5), (5, 33, 9, 17), (70, 130, 65, 129), (64, 64, 1, 64)])
def test_linear_raw_odd_shapes(dn, dtype, T, d_in, r, d_out):
    x, U, V = gen(3, T, d_in, r, d_out, dtype)
    p, keep = pair(dn, U, V, packed=False)
    ws = ws_for(dn, T, [p])
    y = dn.deinfer_lowrank_linear(to_dev(x), p, ws)
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(y), ref) <= TOL[dtype]
    y2 = dn.deinfer_lowrank_down(to_dev(x), p, ws)
    assert np.array_equal(to_host(y2), to_host(y))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_group_calls_raw(dn, dtype):
    import torch
    T, d_in = 37, 72
    x = si.make(5, 1, (T, d_in), 1.0, dtype)
    shapes = {"q": (24, 72), "k": (10, 40), "v": (13, 40), "g": (20, 100), "u": (28, 100)}
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(5, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(5, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), dtype)
        F[n], _k = pair(dn, U, V, packed=False)
        host[n] = (U.values, V.values, _k)
    xd = to_dev(x)
    ws = ws_for(dn, T, [F["q"], F["k"], F["v"]])
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tk = torch.zeros((T, 10), dtype=tdt, device="cuda")
    tv = torch.zeros((T, 13), dtype=tdt, device="cuda")
    q, k, v = dn.deinfer_lowrank_qkv(xd, F["q"], F["k"], F["v"], ws, t_k=tk, t_v=tv)
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x.values, *host["q"][:2], *host["k"][:2], *host["v"][:2], return_t=True)
    for got, ref in ((q, rq), (k, rk), (v, rv), (tk, rtk), (tv, rtv)):
        assert max_err(to_host(got), ref) <= TOL[dtype]
    ws2 = ws_for(dn, T, [F["g"], F["u"]])
    h = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws2)
    rh = oracle.lowrank_gateup_silu(x.values, *host["g"][:2], *host["u"][:2])
    assert max_err(to_host(h), rh) <= TOL[dtype]


# ------------------------------------------------------------------ packed bf16, decode-sized
DECODE_T = [1, 5, 16, 17, 33, 64, 100, 128]


@pytest.mark.parametrize("T", DECODE_T)
@pytest.mark.parametrize("d_in,r,d_out", [(96, 40, 72), (512, 130, 200), (2048, 96, 48)])
def test_linear_packed_decode(dn, T, d_in, r, d_out):
    x, U, V = gen(11, T, d_in, r, d_out, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p])
    xd = to_dev(x)
    y = dn.deinfer_lowrank_linear(xd, p, ws)
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(y), ref) <= TOL["bf16"]
    # same workspace, second call: the sync words must have been left clean; result is deterministic
    y2 = dn.deinfer_lowrank_linear(xd, p, ws)
    ws.check()
    assert np.array_equal(to_host(y2), to_host(y))


@pytest.mark.parametrize("T", [1, 8, 40, 128, 129, 300, 515])
def test_group_calls_packed(dn, T):
    import torch
    d_in = 256
    x = si.make(6, 1, (T, d_in), 1.0, "bf16")
    shapes = {"q": (70, 256), "k": (24, 64), "v": (40, 64), "g": (100, 600), "u": (90, 600), "d": (33, 120)}
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(6, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), "bf16")
        V = si.make(6, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), "bf16")
        F[n], _k = pair(dn, U, V, packed=True)
        host[n] = (U.values, V.values)
    xd = to_dev(x)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, [F["q"], F["k"], F["v"]]),
                          dn.deinfer_workspace_bytes(T, [F["g"], F["u"]])))
    tk = torch.zeros((T, 24), dtype=torch.bfloat16, device="cuda")
    tv = torch.zeros((T, 40), dtype=torch.bfloat16, device="cuda")
    q, k, v = dn.deinfer_lowrank_qkv(xd, F["q"], F["k"], F["v"], ws, t_k=tk, t_v=tv)
    h = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws)
    y = dn.deinfer_lowrank_down(xd, F["d"], ws)
    ws.check()
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x.values, *host["q"], *host["k"], *host["v"], return_t=True)
    for got, ref in ((q, rq), (k, rk), (v, rv), (tk, rtk), (tv, rtv)):
        assert max_err(to_host(got), ref) <= TOL["bf16"]
    assert max_err(to_host(h), oracle.lowrank_gateup_silu(x.values, *host["g"], *host["u"])) <= TOL["bf16"]
    assert max_err(to_host(y), oracle.lowrank_down(x.values, *host["d"])) <= TOL["bf16"]


@pytest.mark.parametrize("T", [17, 40, 100, 128, 300])
def test_qkv_with_a_rank_zero_pair_in_an_exactly_sized_workspace(dn, T):
    """k has rank 0: its output is zero-filled and q, v run as a group of two, which splits differently
    from the group of three the workspace was sized for; the workspace has exactly the queried size
    and a guard region behind it stays untouched."""
    import torch
    d_in = 512
    x = si.make(21, 1, (T, d_in), 1.0, "bf16")
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate({"q": (64, 4096), "v": (64, 4096)}.items()):
        U = si.make(21, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), "bf16")
        V = si.make(21, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), "bf16")
        F[n], _k = pair(dn, U, V, packed=True)
        host[n] = (U.values, V.values)
    k0 = dn.deinfer_pack_factors(dn.raw_pair(torch.zeros((d_in, 0), dtype=torch.bfloat16, device="cuda"),
                                             torch.zeros((0, 4096), dtype=torch.bfloat16, device="cuda")))
    need = dn.deinfer_workspace_bytes(T, [F["q"], k0, F["v"]])
    guard = 1 << 20
    buf = torch.full((need + guard,), 0x5A, dtype=torch.uint8, device="cuda")
    ws = dn.Workspace(need, buf=buf[:need])
    q, k, v = dn.deinfer_lowrank_qkv(to_dev(x), F["q"], k0, F["v"], ws)
    ws.check()
    assert bool((buf[need:] == 0x5A).all()), "the call wrote past the end of its workspace"
    assert float(k.abs().max()) == 0.0
    assert max_err(to_host(q), oracle.lowrank_linear(x.values, *host["q"])) <= TOL["bf16"]
    assert max_err(to_host(v), oracle.lowrank_linear(x.values, *host["v"])) <= TOL["bf16"]


@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("T", [3, 50])
def test_integer_inputs_are_bit_exact(dn, packed, T):
    # small integers: every product and partial sum is exact in bf16-in / fp32-accumulate
    # arithmetic (|t| <= 4*4*64 = 1024 needs 11 bits -> keep t exactly representable in bf16:
    # |x|,|U| <= 2, d_in = 32 -> |t| <= 128; |V| <= 2, r = 24 -> |y| <= 6144 < 2^24)
    d_in, r, d_out = 32, 24, 40
    x = si.store(si.small_ints(9, 1, T * d_in, -2, 2).reshape(T, d_in).astype(np.float32), "bf16")
    U = si.store(si.small_ints(9, 2, d_in * r, -2, 2).reshape(d_in, r).astype(np.float32), "bf16")
    V = si.store(si.small_ints(9, 3, r * d_out, -2, 2).reshape(r, d_out).astype(np.float32), "bf16")
    p, keep = pair(dn, U, V, packed=packed)
    ws = ws_for(dn, T, [p])
    y = to_host(dn.deinfer_lowrank_linear(to_dev(x), p, ws))
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    # the output is rounded once to bf16: compare against the oracle rounded the same way
    ref_b = si.bf16_bits_to_f32(si.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64).reshape(ref.shape)
    assert np.array_equal(y, ref_b)


def test_degenerate_cases(dn):
    import torch
    x, U, V = gen(2, 4, 64, 8, 32, "bf16")
    xd = to_dev(x)
    for packed in (False, True):
        # r == 0 -> exact zeros
        U0 = si.Tensor("bf16", np.zeros((64, 0), np.uint16), np.zeros((64, 0), np.float32))
        V0 = si.Tensor("bf16", np.zeros((0, 32), np.uint16), np.zeros((0, 32), np.float32))
        p0 = dn.raw_pair(torch.zeros((64, 0), dtype=torch.bfloat16, device="cuda"),
                         torch.zeros((0, 32), dtype=torch.bfloat16, device="cuda"))
        if packed:
            p0 = dn.deinfer_pack_factors(p0)
        ws = ws_for(dn, 4, [p0])
        y = torch.full((4, 32), 7.0, dtype=torch.bfloat16, device="cuda")
        dn.deinfer_lowrank_linear(xd, p0, ws, out=y)
        assert float(y.abs().max()) == 0.0
        # T == 0 -> no-op
        p, keep = pair(dn, U, V, packed=packed)
        out = dn.deinfer_lowrank_linear(xd[:0], p, ws_for(dn, 0, [p]))
        assert out.shape == (0, 32)
        # x == 0 -> 0 ; strided (ld > width) input and output views
        big_x = torch.zeros((4, 80), dtype=torch.bfloat16, device="cuda")
        big_x[:, :64] = xd
        big_y = torch.full((4, 48), 3.0, dtype=torch.bfloat16, device="cuda")
        ws = ws_for(dn, 4, [p])
        dn.deinfer_lowrank_linear(big_x[:, :64], p, ws, out=big_y[:, :32])
        ref = oracle.lowrank_linear(x.values, U.values, V.values)
        assert max_err(to_host(big_y[:, :32]), ref) <= TOL["bf16"]
        assert float((big_y[:, 32:] - 3.0).abs().max()) == 0.0      # nothing written past d_out
        z = dn.deinfer_lowrank_linear(torch.zeros_like(xd), p, ws)
        assert float(z.abs().max()) == 0.0


@pytest.mark.parametrize("T", [129, 300, 1000])
@pytest.mark.parametrize("d_in,r,d_out", [(256, 72, 136), (1096, 300, 520)])
def test_linear_packed_beyond_decode_size(dn, T, d_in, r, d_out):
    x, U, V = gen(12, T, d_in, r, d_out, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p])
    y = dn.deinfer_lowrank_linear(to_dev(x), p, ws)
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(y), ref) <= TOL["bf16"]


# ------------------------------------------------------------------ graph replay and determinism
@pytest.mark.parametrize("T", [8, 64, 300])
def test_graph_replay_matches_eager(dn, T):
    """The four calls of a block captured into one HIP graph: every replay (with eager work and
    synchronisations in between) must reproduce the eager result bit for bit, and that result
    must match the oracle."""
    import torch
    d_in, d_ff = 256, 520
    xq, Uq, Vq = gen(21, T, d_in, 72, d_in, "bf16", 1)
    _, Ug, Vg = gen(21, T, d_in, 100, d_ff, "bf16", 4)
    _, Uu, Vu = gen(21, T, d_in, 100, d_ff, "bf16", 8)
    pq, k1 = pair(dn, Uq, Vq, packed=True)
    pg, k2 = pair(dn, Ug, Vg, packed=True)
    pu, k3 = pair(dn, Uu, Vu, packed=True)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, [pq]), dn.deinfer_workspace_bytes(T, [pg, pu])))
    x = to_dev(xq)
    y = torch.empty((T, d_in), dtype=torch.bfloat16, device="cuda")
    h = torch.empty((T, d_ff), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.Stream()

    def run():
        dn.deinfer_lowrank_linear(x, pq, ws, out=y, stream=stream)
        dn.deinfer_lowrank_gateup_silu(x, pg, pu, ws, out=h, stream=stream)

    with torch.cuda.stream(stream):
        run()
    stream.synchronize()
    y0, h0 = to_host(y).copy(), to_host(h).copy()
    assert max_err(y0, oracle.lowrank_linear(xq.values, Uq.values, Vq.values)) <= TOL["bf16"]
    assert max_err(h0, oracle.lowrank_gateup_silu(xq.values, Ug.values, Vg.values, Uu.values, Vu.values)) <= TOL["bf16"]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        run()
    for it in range(3):
        y.zero_(); h.zero_()                               # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(to_host(y), y0), "replay %d: linear differs from the eager result" % it
        assert np.array_equal(to_host(h), h0), "replay %d: gate/up differs from the eager result" % it
    ws.check()


@pytest.mark.parametrize("T", [1, 48, 200])
def test_results_are_deterministic(dn, T):
    """Partial sums are added in a fixed order on every path: repeated calls give identical bits."""
    x, U, V = gen(23, T, 1096, 300, 520, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p])
    xd = to_dev(x)
    first = to_host(dn.deinfer_lowrank_linear(xd, p, ws)).copy()
    for _ in range(3):
        assert np.array_equal(to_host(dn.deinfer_lowrank_linear(xd, p, ws)), first)


# ------------------------------------------------------------------ 16 < T <= 32: one-launch stages
@pytest.mark.parametrize("T", [17, 20, 32])
def test_stream_stage_odd_shapes(dn, T):
    """Stages with at least 100 blocks of 32 features run as one launch with the k split inside the
    workgroup: a wide second stage (odd tile count, ragged last block) and a wide first stage
    (rank not a multiple of 32), plus the GLU pairing and the rank-space copy."""
    import torch
    # wide second stage: d_out = 3300 -> 207 tiles of 16 -> 104 blocks; k = r_pad = 128
    x, U, V = gen(31, T, 264, 100, 3300, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p])
    y = dn.deinfer_lowrank_linear(to_dev(x), p, ws)
    assert max_err(to_host(y), oracle.lowrank_linear(x.values, U.values, V.values)) <= TOL["bf16"]
    # GLU over the same width
    _, U2, V2 = gen(31, T, 264, 72, 3300, "bf16", 5)
    p2, keep2 = pair(dn, U2, V2, packed=True)
    ws2 = ws_for(dn, T, [p, p2])
    h = dn.deinfer_lowrank_gateup_silu(to_dev(x), p, p2, ws2)
    ref = oracle.lowrank_gateup_silu(x.values, U.values, V.values, U2.values, V2.values)
    assert max_err(to_host(h), ref) <= TOL["bf16"]
    # wide first stage: r = 3210 -> r_pad = 3232 -> 101 blocks; narrow second stage
    x3, U3, V3 = gen(32, T, 136, 3210, 72, "bf16")
    p3, keep3 = pair(dn, U3, V3, packed=True)
    ws3 = ws_for(dn, T, [p3, p3, p3])
    tk = torch.zeros((T, 3210), dtype=torch.bfloat16, device="cuda")
    q, k, v = dn.deinfer_lowrank_qkv(to_dev(x3), p3, p3, p3, ws3, t_k=tk)
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x3.values, U3.values, V3.values, U3.values, V3.values,
                                              U3.values, V3.values, return_t=True)
    assert max_err(to_host(q), rq) <= TOL["bf16"]
    assert max_err(to_host(v), rv) <= TOL["bf16"]
    assert max_err(to_host(tk), rtk) <= TOL["bf16"]


# ------------------------------------------------------------------ upward projection alone (low-rank KV cache)
@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("T", [5, 40, 128, 300, 2000])
def test_up_projection_alone(dn, packed, T):
    """y = t V on caller-provided rank-space rows (rank not a multiple of 8, padded pitch)."""
    import torch
    r, d_in, d_out = 204 + 6, 136, 520                 # r % 8 == 2
    _, U, V = gen(41, 4, d_in, r, d_out, "bf16")
    tt = si.make(41, 9, (T, r), 1.0, "bf16")
    p, keep = pair(dn, U, V, packed=packed)
    ws = ws_for(dn, T, [p])
    ld = 216                                            # r rounded up to 8; padding columns zero
    t_dev = torch.zeros((T, ld), dtype=torch.bfloat16, device="cuda")
    t_dev[:, :r] = to_dev(tt)
    y = dn.deinfer_lowrank_up(t_dev[:, :r], p, ws)
    ref = oracle.up_projection(tt.values, V.values)
    assert max_err(to_host(y), ref) <= TOL["bf16"]


@pytest.mark.parametrize("layout", ["odd", "aligned"])
@pytest.mark.parametrize("kind", ["plain", "rope", "glu"])
@pytest.mark.parametrize("T", [3, 40, 128, 300])
@pytest.mark.parametrize("r", [210, 77, 5])
def test_up_projection_reads_only_the_rank_columns(dn, T, kind, layout, r):
    """Packed pairs, rank-space rows that sit inside a wider buffer full of NaN: nothing but columns
    0 .. r - 1 enters the product.  "odd": an odd pitch and an address that is only element aligned
    (the rows are copied first); "aligned": 16-byte aligned rows with a pitch of whole 16-byte
    chunks (read in place up to 128 tokens, the kernels zero what they read beyond column r - 1)."""
    import torch
    d_in, d_out = 136, 512
    r2 = r + 9 if r > 8 else 3                          # the up pair of the GLU call: another rank, another residue
    _, U, V = gen(47, 4, d_in, r, d_out, "bf16")
    _, U2, V2 = gen(48, 4, d_in, r2, d_out, "bf16")
    tt = si.make(47, 9, (T, r), 1.0, "bf16")
    tu = si.make(48, 9, (T, r2), 1.0, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    p2, keep2 = pair(dn, U2, V2, packed=True)
    ws = ws_for(dn, T, [p, p2])
    def embedded(rows, width):
        if layout == "odd":
            buf = torch.full((T, width + 7), float("nan"), dtype=torch.bfloat16, device="cuda")
            view = buf[:, 3:3 + width]
            assert view.data_ptr() % 16 != 0 and view.stride(0) % 8 != 0
        else:
            buf = torch.full((T, (width + 7) // 8 * 8 + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
            view = buf[:, :width]
            assert view.data_ptr() % 16 == 0 and view.stride(0) % 8 == 0
        view.copy_(to_dev(rows))
        return view
    t_dev, u_dev = embedded(tt, r), embedded(tu, r2)
    if kind == "plain":
        y = dn.deinfer_lowrank_up(t_dev, p, ws)
        ref = oracle.up_projection(tt.values, V.values)
    elif kind == "rope":
        pos = torch.arange(T, dtype=torch.int32, device="cuda") * 3 + 1
        tab = dn.deinfer_rope_table(pos, 128)
        y = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
        dn.deinfer_lowrank_up_rope(t_dev, p, tab, ws, out=y)
        ref = pc.rope(oracle.up_projection(tt.values, V.values), pos.cpu().numpy(), d_out // 128, 128)
    else:
        y = dn.deinfer_lowrank_up_glu_silu(t_dev, u_dev, p, p2, ws)
        ref = oracle.up_glu_silu(tt.values, V.values, tu.values, V2.values)
    ws.check()
    got = to_host(y)
    assert np.isfinite(got).all()
    assert max_err(got, ref) <= TOL["bf16"]


def test_up_projection_reads_only_the_rank_columns_wide_layers(dn):
    """The same with the widths that take the other kernels of the 17 .. 128-token range: a GLU second
    stage in one launch (forced) and second stages with several k-ranges."""
    import torch
    T, r, r2, d_in, d_out = 96, 1638, 1003, 64, 4096
    _, U, V = gen(51, 4, d_in, r, d_out, "bf16")
    _, U2, V2 = gen(52, 4, d_in, r2, d_out, "bf16")
    tt = si.make(51, 9, (T, r), 1.0, "bf16")
    tu = si.make(52, 9, (T, r2), 1.0, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    p2, keep2 = pair(dn, U2, V2, packed=True)
    ws = ws_for(dn, T, [p, p2])
    def embedded(rows, width):
        buf = torch.full((T, (width + 7) // 8 * 8 + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
        buf[:, :width] = to_dev(rows)
        return buf[:, :width]
    t_dev, u_dev = embedded(tt, r), embedded(tu, r2)
    y = dn.deinfer_lowrank_up(t_dev, p, ws)
    assert max_err(to_host(y), oracle.up_projection(tt.values, V.values)) <= TOL["bf16"]
    ref = oracle.up_glu_silu(tt.values, V.values, tu.values, V2.values)
    for mode in (0, 1, -1):
        dn.deinfer_set_decode_glu_one_launch(mode)
        try:
            h = dn.deinfer_lowrank_up_glu_silu(t_dev, u_dev, p, p2, ws)
        finally:
            dn.deinfer_set_decode_glu_one_launch(0)
        got = to_host(h)
        assert np.isfinite(got).all() and max_err(got, ref) <= TOL["bf16"]
    ws.check()


@pytest.mark.parametrize("T", [8, 64, 300])
def test_keys_rebuilt_from_the_low_rank_cache(dn, T):
    """t_k written by the qkv call, then the upward projection alone on it: the same keys as
    the qkv call produced, to the bit where both run the same schedule, and within the
    tolerance of the oracle everywhere."""
    import torch
    d_in, r, d_out = 264, 96, 200
    x, U, V = gen(43, T, d_in, r, d_out, "bf16")
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p, p, p])
    tk = torch.zeros((T, r), dtype=torch.bfloat16, device="cuda")
    q, k, v = dn.deinfer_lowrank_qkv(to_dev(x), p, p, p, ws, t_k=tk)
    k2 = dn.deinfer_lowrank_up(tk, p, ws)
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(k2), ref) <= TOL["bf16"]
    assert max_err(to_host(k2), to_host(k).astype(np.float64)) <= 2.0 ** -7    # at most an output rounding apart


# ------------------------------------------------------------------ non-GLU sub-layer: bias and activation
@pytest.mark.parametrize("act", [0, 1, 2])
@pytest.mark.parametrize("kind,T,d_in,r,d_out", [
    ("f32", 16, 96, 24, 70),          # generic fp32 kernel
    ("raw", 9, 96, 24, 70),           # generic kernel, bf16 storage
    ("packed", 3, 264, 96, 200),      # T <= 16 kernel
    ("packed", 16, 128, 40, 3300),    # T <= 16, ragged last feature tile
    ("packed", 24, 264, 96, 3240),    # one-launch stage (>= 100 blocks of 32 features)
    ("packed", 24, 264, 96, 200),     # streaming kernel + reduce
    ("packed", 64, 520, 72, 1000),
    ("packed", 128, 264, 96, 136),
    ("packed", 300, 264, 96, 200),    # compute-bound kernel, ragged token block
    ("packed", 520, 128, 40, 777),    # ... output rows not 16-byte aligned (odd width)
])
def test_linear_with_bias_and_activation(dn, kind, T, d_in, r, d_out, act):
    import torch
    dtype = "f32" if kind == "f32" else "bf16"
    x, U, V = gen(61, T, d_in, r, d_out, dtype)
    b = si.make(61, 9, (1, d_out), 0.5, dtype)
    p, keep = pair(dn, U, V, packed=(kind == "packed"))
    ws = ws_for(dn, T, [p])
    bias = to_dev(b).reshape(-1)
    y = dn.deinfer_lowrank_linear_act(to_dev(x), p, ws, bias=bias, act=act)
    ref = oracle.lowrank_linear_act(x.values, U.values, V.values, b.values.reshape(-1), act)
    assert max_err(to_host(y), ref) <= TOL[dtype]
    # without bias and activation the call is the plain linear layer, bit for bit
    if act == 0:
        y0 = dn.deinfer_lowrank_linear_act(to_dev(x), p, ws)
        assert torch.equal(y0, dn.deinfer_lowrank_linear(to_dev(x), p, ws))


def test_bias_and_activation_with_an_empty_product(dn):
    import torch
    for packed in (False, True):
        x, U, V = gen(62, 5, 64, 8, 48, "bf16")
        b = si.make(62, 9, (1, 48), 1.0, "bf16")
        p, keep = pair(dn, U, V, packed=packed)
        p.desc.r = 0
        ws = ws_for(dn, 5, [p])
        y = dn.deinfer_lowrank_linear_act(to_dev(x), p, ws, bias=to_dev(b).reshape(-1), act=dn.ACT_RELU)
        want = np.tile(np.maximum(b.values.reshape(-1).astype(np.float64), 0.0), (5, 1))
        assert np.array_equal(to_host(y), want)


@pytest.mark.parametrize("T", [200, 600])
def test_first_stage_split_over_k(dn, T):
    """A few hundred tokens and a long d_in: the first stage of the compute-bound path is cut
    into k-parts and summed by the reduce kernel, which also writes the rank-space outputs."""
    import torch
    d_in = 1096                                   # 35 k-blocks: four parts, the last one shorter
    x = si.make(8, 1, (T, d_in), 1.0, "bf16")
    shapes = {"q": (70, 256), "k": (24, 64), "v": (41, 72), "g": (100, 600), "u": (90, 600)}
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(8, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), "bf16")
        V = si.make(8, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), "bf16")
        F[n], _k = pair(dn, U, V, packed=True)
        host[n] = (U.values, V.values)
    xd = to_dev(x)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, [F["q"], F["k"], F["v"]]),
                          dn.deinfer_workspace_bytes(T, [F["g"], F["u"]])))
    tk = torch.zeros((T, 24), dtype=torch.bfloat16, device="cuda")
    tv = torch.zeros((T, 48), dtype=torch.bfloat16, device="cuda")     # wider than r_v = 41: the rest stays zero
    q, k, v = dn.deinfer_lowrank_qkv(xd, F["q"], F["k"], F["v"], ws, t_k=tk, t_v=tv)
    h = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws)
    b = si.make(8, 30, (1, 600), 0.5, "bf16")
    a = dn.deinfer_lowrank_linear_act(xd, F["g"], ws, bias=to_dev(b).reshape(-1), act=dn.ACT_GELU)
    ws.check()
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x.values, *host["q"], *host["k"], *host["v"], return_t=True)
    for got, ref in ((q, rq), (k, rk), (v, rv), (tk, rtk), (tv[:, :41], rtv)):
        assert max_err(to_host(got), ref) <= TOL["bf16"]
    assert bool((tv[:, 41:] == 0).all())
    assert max_err(to_host(h), oracle.lowrank_gateup_silu(x.values, *host["g"], *host["u"])) <= TOL["bf16"]
    assert max_err(to_host(a), oracle.lowrank_linear_act(x.values, *host["g"], b.values.reshape(-1), oracle.ACT_GELU)) <= TOL["bf16"]
    # the keys rebuilt from t_k equal the keys of the qkv call up to the output rounding
    k2 = dn.deinfer_lowrank_up(tk, F["k"], ws)
    assert max_err(to_host(k2), to_host(k)) <= 2.0 ** -7


# ------------------------------------------------------------------ the two stages as separate calls
@pytest.mark.parametrize("kind", ["f32", "raw", "packed"])
@pytest.mark.parametrize("T", [1, 12, 24, 100, 300, 600])
def test_stages_as_separate_calls(dn, kind, T):
    """What one tensor-parallel rank runs: downward projections alone (rank-space results handed
    out), then the upward projections on rank-space rows; together they reproduce the fused calls."""
    import torch
    dtype = "f32" if kind == "f32" else "bf16"
    d_in = 1096 if kind == "packed" else 200
    x = si.make(9, 1, (T, d_in), 1.0, dtype)
    shapes = {"q": (70, 256), "k": (24, 64), "g": (100, 3300), "u": (90, 3300)}
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(9, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(9, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), dtype)
        F[n], _k = pair(dn, U, V, packed=(kind == "packed"))
        host[n] = (U.values, V.values)
    xd = to_dev(x)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, [F["q"], F["k"]]), dn.deinfer_workspace_bytes(T, [F["g"], F["u"]])))
    tq, tk = dn.deinfer_lowrank_down_proj(xd, [F["q"], F["k"]], ws)
    tg, tu = dn.deinfer_lowrank_down_proj(xd, [F["g"], F["u"]], ws)
    for got, n in ((tq, "q"), (tk, "k"), (tg, "g"), (tu, "u")):
        assert max_err(to_host(got), oracle.down_projection(x.values, host[n][0])) <= TOL[dtype]
    q = dn.deinfer_lowrank_up(tq, F["q"], ws)
    h = dn.deinfer_lowrank_up_glu_silu(tg, tu, F["g"], F["u"], ws)
    ws.check()
    # against the oracle fed the same rank-space rows, and end to end
    assert max_err(to_host(q), oracle.up_projection(to_host(tq), host["q"][1])) <= TOL[dtype]
    assert max_err(to_host(h), oracle.up_glu_silu(to_host(tg), host["g"][1], to_host(tu), host["u"][1])) <= TOL[dtype]
    assert max_err(to_host(q), oracle.lowrank_linear(x.values, *host["q"])) <= TOL[dtype]
    assert max_err(to_host(h), oracle.lowrank_gateup_silu(x.values, *host["g"], *host["u"])) <= TOL[dtype]
    if kind == "packed":
        # the staged GLU call sees bf16 rank-space rows, as the fused call does inside
        h_fused = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws)
        assert max_err(to_host(h), to_host(h_fused)) <= 2.0 ** -6


# ------------------------------------------------------------------ the one-launch second stage of the GLU call
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("T", [17, 32, 40, 64, 100, 128])
def test_glu_second_stage_in_one_launch(dn, dtype, T):
    """Both products of the GLU call in one workgroup (no partial sums), forced for small shapes that
    would not choose it: ragged widths (not a multiple of 32, of 8), different ranks for gate and up
    (neither a multiple of 32), fused and staged entry points, against the oracle; and against the
    split with partial sums that it replaces."""
    import torch
    d_in = 520
    shapes = {"g": (100, 1234), "u": (75, 1234)}
    x = si.make(33, 1, (T, d_in), 1.0, dtype)
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(33, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(33, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), dtype)
        F[n], _k = pair(dn, U, V, packed=True)
        host[n] = (U.values, V.values)
    xd = to_dev(x)
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [F["g"], F["u"]]))
    try:
        dn.deinfer_set_decode_glu_one_launch(-1)
        h_split = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws)
        dn.deinfer_set_decode_glu_one_launch(1)
        h = torch.full((T, 1240), 9.0, dtype=xd.dtype, device="cuda")       # pitch > width: nothing may be written past d_out
        dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws, out=h[:, :1234])
        tg, tu = dn.deinfer_lowrank_down_proj(xd, [F["g"], F["u"]], ws)
        h_staged = dn.deinfer_lowrank_up_glu_silu(tg, tu, F["g"], F["u"], ws)
        ws.check()
    finally:
        dn.deinfer_set_decode_glu_one_launch(0)
    ref = oracle.lowrank_gateup_silu(x.values, *host["g"], *host["u"])
    assert max_err(to_host(h[:, :1234]), ref) <= TOL[dtype]
    assert max_err(to_host(h_staged), ref) <= TOL[dtype]
    assert float((h[:, 1234:].float() - 9.0).abs().max()) == 0.0
    assert max_err(to_host(h[:, :1234]), to_host(h_split)) <= 2.0 ** -6
    assert max_err(to_host(h_staged), oracle.up_glu_silu(to_host(tg), host["g"][1], to_host(tu), host["u"][1])) <= TOL[dtype]


# ------------------------------------------------------------------ the two token tiles of the T > 128 kernel
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("T", [129, 700])
def test_token_tiles_give_identical_results(dn, dtype, T):
    """The three workgroup tiles (256 x 256, 128 x 256, 128 x 128) take the same sums in the same order: the outputs of every
    kind of call (grouped, GLU, bias + activation, rank-space outputs) agree bit for bit, and with
    the oracle within the tolerance.  T = 700: ragged last tile for both (188 and 60 rows)."""
    import torch
    d_in = 264
    x = si.make(61, 1, (T, d_in), 1.0, dtype)
    shapes = {"q": (70, 384), "k": (24, 128), "v": (41, 72), "g": (100, 600), "u": (90, 600)}
    F, host = {}, {}
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(61, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(61, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), dtype)
        F[n], _k = pair(dn, U, V, packed=True)
        host[n] = (U.values, V.values)
    xd = to_dev(x)
    b = si.make(61, 30, (1, 600), 0.5, dtype)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, [F["q"], F["k"], F["v"]]),
                          dn.deinfer_workspace_bytes(T, [F["g"], F["u"]])))
    res = {}
    for tile in (128, 129, 256, TOKEN_TILE_BOTH):  # 128: 128 x 128 tiles, 129: 128 x 256 tiles, the last: two shapes in one launch
        dn.deinfer_set_prefill_token_tile(128 if tile == 129 else tile)
        dn.deinfer_set_prefill_feature_tile(256 if tile == 129 else 128 if tile == 128 else 0)
        tk = torch.zeros((T, 24), dtype=xd.dtype, device="cuda")
        q, k, v = dn.deinfer_lowrank_qkv(xd, F["q"], F["k"], F["v"], ws, t_k=tk)
        h = dn.deinfer_lowrank_gateup_silu(xd, F["g"], F["u"], ws)
        a = dn.deinfer_lowrank_linear_act(xd, F["g"], ws, bias=to_dev(b).reshape(-1), act=dn.ACT_GELU)
        k2 = dn.deinfer_lowrank_up(tk, F["k"], ws)
        torch.cuda.synchronize()
        ws.check()
        res[tile] = [t.clone() for t in (q, k, v, tk, h, a, k2)]
    dn.deinfer_set_prefill_token_tile(0)
    dn.deinfer_set_prefill_feature_tile(0)
    for t128, t129, t256, t384 in zip(res[128], res[129], res[256], res[TOKEN_TILE_BOTH]):
        assert torch.equal(t128.view(torch.int16), t256.view(torch.int16))
        assert torch.equal(t129.view(torch.int16), t256.view(torch.int16))
        assert torch.equal(t384.view(torch.int16), t256.view(torch.int16))
    q, k, v, tk, h, a, k2 = res[128]
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x.values, *host["q"], *host["k"], *host["v"], return_t=True)
    for got, ref in ((q, rq), (k, rk), (v, rv), (tk, rtk)):
        assert max_err(to_host(got), ref) <= TOL[dtype]
    assert max_err(to_host(h), oracle.lowrank_gateup_silu(x.values, *host["g"], *host["u"])) <= TOL[dtype]
    assert max_err(to_host(a), oracle.lowrank_linear_act(x.values, *host["g"], b.values.reshape(-1), oracle.ACT_GELU)) <= TOL[dtype]


# ------------------------------------------------------------------ calls in flight on two streams
@pytest.mark.parametrize("T", [8, 64, 300])
def test_two_streams_with_their_own_workspaces(dn, T):
    """The library keeps no device state of its own between calls: two chains of calls enqueued on
    two streams at once, each with its own workspace, give the bits of the same calls run one
    after the other."""
    import torch
    d_in = 264
    shapes = {"q": (70, 384), "k": (24, 128), "v": (41, 72), "g": (100, 600), "u": (90, 600)}
    F = {}
    keep = []
    for i, (n, (r, d_out)) in enumerate(shapes.items()):
        U = si.make(71, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), "bf16")
        V = si.make(71, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), "bf16")
        F[n], k = pair(dn, U, V, packed=True)
        keep.append(k)
    xs = [to_dev(si.make(71, 1 + j, (T, d_in), 1.0, "bf16")) for j in range(2)]
    nbytes = max(dn.deinfer_workspace_bytes(T, [F["q"], F["k"], F["v"]]), dn.deinfer_workspace_bytes(T, [F["g"], F["u"]]))
    wss = [dn.Workspace(nbytes) for _ in range(2)]

    def chain(j, stream):
        out = []
        for rep in range(3):
            q, k, v = dn.deinfer_lowrank_qkv(xs[j], F["q"], F["k"], F["v"], wss[j], stream=stream)
            h = dn.deinfer_lowrank_gateup_silu(xs[j], F["g"], F["u"], wss[j], stream=stream)
            o = dn.deinfer_lowrank_linear(xs[j], F["q"], wss[j], stream=stream)
            out = [q, k, v, h, o]
        return out

    want = [chain(j, None) for j in range(2)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [None, None]
    for j in range(2):                      # outputs are allocated under the stream that fills them
        with torch.cuda.stream(streams[j]):
            got[j] = chain(j, streams[j])
    torch.cuda.synchronize()
    for j in range(2):
        wss[j].check()
        for a, b in zip(got[j], want[j]):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ------------------------------------------------------------------ MQA shapes, a rank per layer and per projection
@pytest.mark.parametrize("T", [4, 64, 300])
def test_mqa_shapes_and_per_layer_ranks(dn, T):
    """Multi-query attention (one key / value head of 128 features beside 8 query heads) and a
    different parameter reduction per layer and per projection (Sec. 4.3: q, k, v may carry
    different ratios; Table 2 lists per-model settings): ranks from the rule of Sec. 2.1 for six
    "layers", every call against the oracle."""
    hidden, head = 1024, 128
    x = si.make(81, 1, (T, hidden), 1.0, "bf16")
    xd = to_dev(x)
    for layer, (rq, rk, rv) in enumerate([(0.2, 0.2, 0.2), (0.4, 0.1, 0.3), (0.6, 0.5, 0.0), (0.8, 0.7, 0.9), (0.3, 0.95, 0.5), (0.5, 0.5, 0.5)]):
        F, host = [], []
        for i, (rho, d_out) in enumerate(((rq, hidden), (rk, head), (rv, head))):
            r = dn.deinfer_rank_for_ratio(hidden, d_out, rho)
            assert r == oracle.rank_for_keep(hidden, d_out, round((1.0 - rho) * 1000), 1000)
            U = si.make(81, 10 * layer + 2 * i + 2, (hidden, r), 1.0 / np.sqrt(hidden), "bf16")
            V = si.make(81, 10 * layer + 2 * i + 3, (r, d_out), 1.0 / np.sqrt(r), "bf16")
            p, _k = pair(dn, U, V, packed=True)
            F.append(p); host.append((U.values, V.values))
        ws = ws_for(dn, T, F)
        q, k, v = dn.deinfer_lowrank_qkv(xd, F[0], F[1], F[2], ws)
        rq_, rk_, rv_ = oracle.lowrank_qkv(x.values, *host[0], *host[1], *host[2])
        for got, ref in ((q, rq_), (k, rk_), (v, rv_)):
            assert max_err(to_host(got), ref) <= TOL["bf16"]


# ------------------------------------------------------------------ wide outputs: one k-range, no reduce launch
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("T", [40, 128])
def test_wide_outputs_stored_by_the_streaming_kernel(dn, dtype, T):
    """More than 128 groups of 128 output features leave one k-range per group: the streaming
    kernel of 32 < T <= 128 then rounds and stores the outputs itself (bias, activation, three
    outputs of different width, a pitch that rules out 8-byte stores, a ragged last group)."""
    import torch
    d_in = 72
    x = si.make(91, 1, (T, d_in), 1.0, dtype)
    xd = to_dev(x)
    # single pair with bias and GELU, 16530 outputs (129.1 groups), odd output pitch
    U = si.make(91, 2, (d_in, 40), 1.0 / np.sqrt(d_in), dtype)
    V = si.make(91, 3, (40, 16530), 1.0 / np.sqrt(40), dtype)
    b = si.make(91, 4, (1, 16530), 0.5, dtype)
    p, keep = pair(dn, U, V, packed=True)
    ws = ws_for(dn, T, [p])
    for pitch in (16536, 16531):
        y = torch.full((T, pitch), 3.0, dtype=xd.dtype, device="cuda")
        dn.deinfer_lowrank_linear_act(xd, p, ws, bias=to_dev(b).reshape(-1), act=dn.ACT_GELU, out=y[:, :16530])
        ref = oracle.lowrank_linear_act(x.values, U.values, V.values, b.values.reshape(-1), oracle.ACT_GELU)
        got = to_host(y)
        assert max_err(got[:, :16530], ref) <= TOL[dtype]
        assert np.all(got[:, 16530:] == 3.0)
    ws.check()
    # three pairs, 16900 outputs together
    F, host = [], []
    for i, (r, d_out) in enumerate(((24, 6000), (9, 5500), (33, 5400))):
        Ui = si.make(91, 10 + 2 * i, (d_in, r), 1.0 / np.sqrt(d_in), dtype)
        Vi = si.make(91, 11 + 2 * i, (r, d_out), 1.0 / np.sqrt(r), dtype)
        pi_, _k = pair(dn, Ui, Vi, packed=True)
        F.append(pi_); host.append((Ui.values, Vi.values))
    ws3 = ws_for(dn, T, F)
    q, k, v = dn.deinfer_lowrank_qkv(xd, F[0], F[1], F[2], ws3)
    ws3.check()
    for got, ref in zip((q, k, v), oracle.lowrank_qkv(x.values, *host[0], *host[1], *host[2])):
        assert max_err(to_host(got), ref) <= TOL[dtype]
