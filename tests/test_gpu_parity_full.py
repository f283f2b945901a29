"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(packed bf16 weights, one call per entry point, shared workspace).

The GPU runs every call at the real shape.  The oracle (fp64 loops) is evaluated on ALL token
rows for T <= 128 and on a sample of rows for the large sizes - rows are independent in every
step of the path, so a row of the output depends only on the same row of the input.  The sample
(sample_rows) holds the first and last row, the rows on either side of every border of the
kernels' 128- and 256-token tiles, one seeded random interior row of every 128-token block, rows
of every residue modulo 32 in both halves of 256-token tiles, and rows of the last 256 tokens
(the ragged tile).  For the decode sizes the activations are fully seeded; for the large sizes
the sampled rows are the seeded ones and the remaining rows are filled by torch's seeded
generator.  Those remaining rows are checked too: every row of every output is compared, to the
same bar, with fp32 products of the same inputs formed on the device by torch (an independent
routine; it stands in for the oracle only where the oracle is too slow to go).
Beside the gate max|y - ref| / max|ref| the stricter max(|y - ref| / max(|ref_ij|, rms ref)) is
printed (it is not a gate: near a zero of the reference it measures the reference, not the error).
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from gpu_util import TOL, max_err, to_dev, to_host

pytestmark = pytest.mark.gpu

_cache = {}


def block(dn, name, seed, dtype="bf16"):
    """Packed device weights, the raw device weights and fp64 host weights of one benchmark block
    (cached per module)."""
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
        P, H, D = {}, {}, {}
        for i, p in enumerate(si._ORDER):
            if p not in proj:
                continue
            m, n = proj[p]
            U = si.make(seed, 16 + 2 * i, (m, ranks[p]), shape.weight_std, dtype)
            V = si.make(seed, 17 + 2 * i, (ranks[p], n), shape.weight_std, dtype)
            D[p] = (to_dev(U), to_dev(V))
            P[p] = dn.deinfer_pack_factors(dn.raw_pair(*D[p]))
            torch.cuda.synchronize()
            H[p] = (U.values.astype(np.float64), V.values.astype(np.float64))
        _cache[key] = (shape, proj, ranks, P, H, D)
    return _cache[key]


@pytest.fixture(scope="module")
def dn():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_17709_amd as dn
    dn.lib()
    yield dn
    _cache.clear()


def sample_rows(T, seed):
    """Rows of a large call that the oracle evaluates (see the module text)."""
    rng = np.random.default_rng(seed)
    rows = {0, T - 1}
    for b in range(128, T, 128):                 # borders of the 128- and 256-token tiles
        rows.update((b - 1, b))
    for blk in range((T + 127) // 128):          # an interior row of every 128-token block
        rows.add(min(T - 1, blk * 128 + int(rng.integers(1, 127))))
    for res in range(32):                        # every residue modulo 32, both halves of a 256-token tile
        for half in (0, 1):
            r = 256 * int(rng.integers(0, max(1, T // 256))) + 128 * half + 32 * int(rng.integers(0, 4)) + res
            if r < T:
                rows.add(r)
    for r in rng.integers(max(0, T - 256), T, size=8):     # the last (ragged) tile
        rows.add(int(r))
    return sorted(rows)


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


def strict_err(y, ref):
    """max |y - ref| / max(|ref_ij|, rms ref): the stricter, printed metric."""
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 1.0
    return float(np.max(np.abs(y - ref) / np.maximum(np.abs(ref), max(rms, 1e-300)))) if ref.size else 0.0


def run_block(dn, name, T, seed, dtype="bf16"):
    import torch
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    shape, proj, ranks, P, H, D = block(dn, name, seed, dtype)
    rows = list(range(T)) if T <= 128 else sample_rows(T, seed)
    assert T < 4096 or len(rows) >= 128
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
    errs, strict = {}, {}
    for n, (got, ref) in refs.items():
        g = to_host(got[sel])
        errs[n] = max_err(g, ref)
        strict[n] = strict_err(g, ref)
    print(name, "T=%d" % T, "rows=%d" % len(rows), {n: "%.2e" % e for n, e in errs.items()},
          "strict", {n: "%.2e" % e for n, e in strict.items()}, flush=True)
    assert max(errs.values()) <= TOL[dtype], errs
    # invariants that hold at any size: finite everywhere
    for t in (q, k, v, o, h, y):
        assert bool(torch.isfinite(t.float()).all())
    if len(rows) == T:
        return
    # every row, also those the oracle did not evaluate, against fp32 products formed by torch on the device
    def lin(x_, p):
        return (x_.float() @ D[p][0].float()) @ D[p][1].float()
    def dev_err(got, ref):
        return float((got.float() - ref).abs().max() / ref.abs().max())
    all_rows = {"q": dev_err(q, lin(xd, "q")), "k": dev_err(k, lin(xd, "k")), "v": dev_err(v, lin(xd, "v")),
                "t_k": dev_err(tk, xd.float() @ D["k"][0].float()), "t_v": dev_err(tv, xd.float() @ D["v"][0].float()),
                "o": dev_err(o, lin(ad, "o"))}
    if shape.glu:
        all_rows["h"] = dev_err(h, torch.nn.functional.silu(lin(xd, "gate")) * lin(xd, "up"))
        all_rows["y"] = dev_err(y, lin(hd, "down"))
    else:
        all_rows["h"] = dev_err(h, torch.relu(lin(xd, "gate") + to_dev(b1).reshape(-1).float()))
        all_rows["y"] = dev_err(y, lin(hd, "down") + to_dev(b2).reshape(-1).float())
    print(name, "T=%d" % T, "all rows against torch fp32 on the device", {n: "%.2e" % e for n, e in all_rows.items()}, flush=True)
    assert max(all_rows.values()) <= TOL[dtype], all_rows


@pytest.mark.parametrize("T", [1, 8, 32, 64])
def test_llama7b_keep80_decode(dn, T):
    run_block(dn, "llama7b_keep80", T, seed=1)


def test_llama70b_keep40_decode_128(dn):
    run_block(dn, "llama70b_keep40", 128, seed=4)


def test_llama70b_keep40_prefill_4096(dn):
    run_block(dn, "llama70b_keep40", 4096, seed=4)


@pytest.mark.parametrize("name", ["llama7b_keep60", "llama7b_keep40"])
def test_llama7b_prefill_8192(dn, name):
    run_block(dn, name, 8192, seed=2)


def test_llama13b_keep60_mixed_8256(dn):
    run_block(dn, "llama13b_keep60", 8256, seed=3)


@pytest.mark.parametrize("T", [64, 4096])
def test_opt30b_keep60_non_glu(dn, T):
    run_block(dn, "opt30b_keep60", T, seed=5)


@pytest.mark.parametrize("T", [8, 64, 512])
def test_llama7b_keep60_fp16(dn, T):
    """The same block with fp16 storage (weights, activations, outputs), fp32 sums."""
    run_block(dn, "llama7b_keep60", T, seed=6, dtype="f16")


def test_llama7b_keep60_chunk_of_512_tokens(dn):
    """Between the decode sizes and the large prefill: the first stage runs split over k."""
    run_block(dn, "llama7b_keep60", 512, seed=2)
