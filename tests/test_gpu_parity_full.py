"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(packed bf16 weights, one call per entry point, shared workspace).

The GPU runs every call at the real shape.  The oracle (fp64 loops) is evaluated on a
sample of token rows - rows are independent in every step of the path, so a row of the
output depends only on the same row of the input - always including the first and last row
and the rows on either side of the kernels' 16-token tile boundaries.  For the decode sizes
the activations are fully seeded; for the prefill sizes the sampled rows are the seeded ones
and the remaining rows are filled by torch's seeded generator (they are computed but not
compared).
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from gpu_util import TOL, max_err, to_dev, to_host

pytestmark = pytest.mark.gpu

_cache = {}


def block(dn, name, seed, dtype="bf16"):
    """Packed device weights + fp64 host weights of one benchmark block (cached per module)."""
    import torch
    key = (name, seed, dtype)
    if key not in _cache:
        _cache.clear()                          # one block at a time: bounded host / device memory
        shape = si.BLOCKS[name]
        proj = shape.projections()
        rho = 1.0 - shape.keep_num / shape.keep_den
        ranks = {p: dn.deinfer_rank_for_ratio(m, n, rho) for p, (m, n) in proj.items()}
        for p, (m, n) in proj.items():          # library rule == oracle rule
            assert ranks[p] == oracle.rank_for_keep(m, n, shape.keep_num, shape.keep_den)
        P, H = {}, {}
        for i, p in enumerate(si._ORDER):
            if p not in proj:
                continue
            m, n = proj[p]
            U = si.make(seed, 16 + 2 * i, (m, ranks[p]), shape.weight_std, dtype)
            V = si.make(seed, 17 + 2 * i, (ranks[p], n), shape.weight_std, dtype)
            P[p] = dn.deinfer_pack_factors(dn.raw_pair(to_dev(U), to_dev(V)))
            torch.cuda.synchronize()
            H[p] = (U.values.astype(np.float64), V.values.astype(np.float64))
        _cache[key] = (shape, proj, ranks, P, H)
    return _cache[key]


@pytest.fixture(scope="module")
def dn():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_17709_amd as dn
    dn.lib()
    yield dn
    _cache.clear()


def sample_rows(T, limit):
    """First and last row plus rows on either side of the kernels' token-tile borders (16 for the
    decode kernels, 128 / 256 for the prefill kernel), thinned to about `limit` rows."""
    step = 16 if T <= 128 else 128
    rows = {0, T - 1}
    for b in range(step, T, step):
        rows.update((b - 1, b))
    rows = sorted(r for r in rows if 0 <= r < T)
    if len(rows) > limit:                        # keep first/last and an even spread of borders
        idx = np.unique(np.round(np.linspace(0, len(rows) - 1, limit)).astype(int))
        rows = [rows[i] for i in idx]
    return rows


def activations(seed, stream, T, width, rows, dtype="bf16"):
    """Device tensor [T x width] whose `rows` are the seeded rows; returns (device, host rows)."""
    import torch
    sub = si.make_rows(seed, stream, rows, width, 1.0, dtype)
    if len(rows) == T:
        return to_dev(sub), sub.values.astype(np.float64)
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 * seed + stream)
    full = torch.randn((T, width), generator=g, device="cuda", dtype=torch.float32).to(torch.float16 if dtype == "f16" else torch.bfloat16)
    full[torch.tensor(rows, device="cuda")] = to_dev(sub)
    return full, sub.values.astype(np.float64)


def run_block(dn, name, T, seed, row_limit, dtype="bf16"):
    import torch
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    shape, proj, ranks, P, H = block(dn, name, seed, dtype)
    rows = list(range(T)) if T <= row_limit else sample_rows(T, row_limit)
    xd, xh = activations(seed, 1, T, shape.hidden, rows, dtype)
    ad, ah = activations(seed, 2, T, shape.hidden, rows, dtype)
    hd, hh = activations(seed, 3, T, shape.ffn, rows, dtype)
    nbytes = max(dn.deinfer_workspace_bytes(T, [P["q"], P["k"], P["v"]]),
                 dn.deinfer_workspace_bytes(T, [P["o"]]),
                 dn.deinfer_workspace_bytes(T, [P["gate"], P["up"]] if shape.glu else [P["gate"]]),
                 dn.deinfer_workspace_bytes(T, [P["down"]]))
    ws = dn.Workspace(nbytes)
    tk = torch.zeros((T, ranks["k"]), dtype=tdt, device="cuda")
    tv = torch.zeros((T, ranks["v"]), dtype=tdt, device="cuda")
    q, k, v = dn.deinfer_lowrank_qkv(xd, P["q"], P["k"], P["v"], ws, t_k=tk, t_v=tv)
    o = dn.deinfer_lowrank_linear(ad, P["o"], ws)
    if shape.glu:
        h = dn.deinfer_lowrank_gateup_silu(xd, P["gate"], P["up"], ws)
        y = dn.deinfer_lowrank_down(hd, P["down"], ws)
    else:       # non-GLU MLP: act(x U1 V1 + b1), then the second pair with its bias
        b1 = si.make(seed, 4, (1, shape.ffn), shape.weight_std, dtype)
        b2 = si.make(seed, 5, (1, shape.hidden), shape.weight_std, dtype)
        h = dn.deinfer_lowrank_linear_act(xd, P["gate"], ws, bias=to_dev(b1).reshape(-1), act=dn.ACT_RELU)
        y = dn.deinfer_lowrank_linear_act(hd, P["down"], ws, bias=to_dev(b2).reshape(-1), act=dn.ACT_NONE)
    ws.check()
    sel = torch.tensor(rows, device="cuda")
    rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(xh, *H["q"], *H["k"], *H["v"], return_t=True)
    refs = {"q": (q, rq), "k": (k, rk), "v": (v, rv), "t_k": (tk, rtk), "t_v": (tv, rtv),
            "o": (o, oracle.lowrank_linear(ah, *H["o"])),
            "h": (h, oracle.lowrank_gateup_silu(xh, *H["gate"], *H["up"]) if shape.glu else
                  oracle.lowrank_linear_act(xh, *H["gate"], b1.values.reshape(-1), oracle.ACT_RELU)),
            "y": (y, oracle.lowrank_down(hh, *H["down"]) if shape.glu else
                  oracle.lowrank_linear_act(hh, *H["down"], b2.values.reshape(-1), oracle.ACT_NONE))}
    errs = {n: max_err(to_host(got[sel]), ref) for n, (got, ref) in refs.items()}
    print(name, "T=%d" % T, "rows=%d" % len(rows), {n: "%.2e" % e for n, e in errs.items()}, flush=True)
    assert max(errs.values()) <= TOL[dtype], errs
    # invariants that hold at any size: finite everywhere, untouched rows stay plausible
    for t in (q, k, v, o, h, y):
        assert bool(torch.isfinite(t.float()).all())


@pytest.mark.parametrize("T", [1, 8, 32, 64])
def test_llama7b_keep80_decode(dn, T):
    run_block(dn, "llama7b_keep80", T, seed=1, row_limit=12)


def test_llama70b_keep40_decode_128(dn):
    run_block(dn, "llama70b_keep40", 128, seed=4, row_limit=8)


def test_llama70b_keep40_prefill_4096(dn):
    run_block(dn, "llama70b_keep40", 4096, seed=4, row_limit=8)


@pytest.mark.parametrize("name", ["llama7b_keep60", "llama7b_keep40"])
def test_llama7b_prefill_8192(dn, name):
    run_block(dn, name, 8192, seed=2, row_limit=10)


def test_llama13b_keep60_mixed_8256(dn):
    run_block(dn, "llama13b_keep60", 8256, seed=3, row_limit=10)


@pytest.mark.parametrize("T", [64, 4096])
def test_opt30b_keep60_non_glu(dn, T):
    run_block(dn, "opt30b_keep60", T, seed=5, row_limit=8)


@pytest.mark.parametrize("T", [8, 64, 512])
def test_llama7b_keep60_fp16(dn, T):
    """The same block with fp16 storage (weights, activations, outputs), fp32 sums."""
    run_block(dn, "llama7b_keep60", T, seed=6, row_limit=8, dtype="f16")


def test_llama7b_keep60_chunk_of_512_tokens(dn):
    """Between the decode sizes and the large prefill: the first stage runs split over k."""
    run_block(dn, "llama7b_keep60", 512, seed=2, row_limit=10)
