"""Seeded random shapes through every entry point of the packed path, against the oracle.

The fixed cases elsewhere sit on the borders the kernels are known to have; these cases are
drawn without regard to them (token counts from all four schedules, widths and ranks that are
no multiple of any tile size), so that a border nobody thought of still gets hit.
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si
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


def draw(case):
    rng = np.random.default_rng(1000 + case)
    T = int(rng.choice([rng.integers(1, 17), rng.integers(17, 33), rng.integers(33, 129), rng.integers(129, 700)]))
    d_in = int(rng.integers(1, 190)) * 8
    wide = rng.random() < 0.25
    ranks = [int(rng.integers(1, 300)) for _ in range(3)]
    outs = [int(rng.integers(1, 900)) if not wide else int(rng.integers(3200, 3600)) for _ in range(3)]
    return T, d_in, ranks, outs


@pytest.mark.parametrize("dtype,case", [("bf16", c) for c in range(48)] + [("f16", c) for c in range(30)])
def test_random_shapes(dn, dtype, case):
    import torch
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    T, d_in, ranks, outs = draw(case)
    x = si.make(100 + case, 1, (T, d_in), 1.0, dtype)
    F, H = [], []
    for i in range(3):
        d_out = outs[0] if i == 1 and case % 3 == 1 else outs[i]        # gate / up share their width
        U = si.make(100 + case, 10 + 2 * i, (d_in, ranks[i]), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(100 + case, 11 + 2 * i, (ranks[i], d_out), 1.0 / np.sqrt(ranks[i]), dtype)
        p, _keep = pair(dn, U, V, packed=True)
        F.append(p); H.append((U.values, V.values))
    xd = to_dev(x)
    ws = dn.Workspace(max(dn.deinfer_workspace_bytes(T, F), dn.deinfer_workspace_bytes(T, F[:2]), dn.deinfer_workspace_bytes(T, F[:1]),
                          dn.deinfer_workspace_bytes(T, F[1:2])))
    kind = case % 3
    if kind == 0:          # three pairs, rank-space outputs, then the keys rebuilt from t_k
        pad8 = lambda r: (r + 7) // 8 * 8
        tk = torch.zeros((T, pad8(ranks[1])), dtype=tdt, device="cuda")[:, :ranks[1]]
        tv = torch.zeros((T, ranks[2] + 3), dtype=tdt, device="cuda")[:, :ranks[2]]
        q, k, v = dn.deinfer_lowrank_qkv(xd, F[0], F[1], F[2], ws, t_k=tk, t_v=tv)
        rq, rk, rv, rtk, rtv = oracle.lowrank_qkv(x.values, *H[0], *H[1], *H[2], return_t=True)
        for got, ref in ((q, rq), (k, rk), (v, rv), (tk, rtk), (tv, rtv)):
            assert max_err(to_host(got), ref) <= TOL[dtype]
        k2 = dn.deinfer_lowrank_up(tk, F[1], ws)
        assert max_err(to_host(k2), rk) <= TOL[dtype]
    elif kind == 1:        # GLU sub-layer, fused and staged
        h = dn.deinfer_lowrank_gateup_silu(xd, F[0], F[1], ws)
        ref = oracle.lowrank_gateup_silu(x.values, *H[0], *H[1])
        assert max_err(to_host(h), ref) <= TOL[dtype]
        tg, tu = dn.deinfer_lowrank_down_proj(xd, [F[0], F[1]], ws)
        h2 = dn.deinfer_lowrank_up_glu_silu(tg, tu, F[0], F[1], ws)
        assert max_err(to_host(h2), ref) <= TOL[dtype]
    else:                  # single pair: plain, and with bias and activation
        y = dn.deinfer_lowrank_linear(xd, F[0], ws)
        assert max_err(to_host(y), oracle.lowrank_linear(x.values, *H[0])) <= TOL[dtype]
        b = si.make(100 + case, 40, (1, outs[0]), 0.5, dtype)
        act = 1 + case % 2
        ya = dn.deinfer_lowrank_linear_act(xd, F[0], ws, bias=to_dev(b).reshape(-1), act=act)
        assert max_err(to_host(ya), oracle.lowrank_linear_act(x.values, *H[0], b.values.reshape(-1), act)) <= TOL[dtype]
    ws.check()


@pytest.mark.parametrize("dtype,case", [(d, c) for d in ("f32", "bf16", "f16") for c in range(8)])
def test_random_shapes_raw_layout(dn, dtype, case):
    """The same through the generic kernels (RAW pairs, any alignment, any width)."""
    import torch
    rng = np.random.default_rng(5000 + case)
    T, d_in = int(rng.integers(1, 150)), int(rng.integers(1, 300))
    ranks = [int(rng.integers(1, 90)) for _ in range(3)]
    outs = [int(rng.integers(1, 260)) for _ in range(3)]
    outs[1] = outs[0]
    x = si.make(200 + case, 1, (T, d_in), 1.0, dtype)
    F, H = [], []
    for i in range(3):
        U = si.make(200 + case, 10 + 2 * i, (d_in, ranks[i]), 1.0 / np.sqrt(d_in), dtype)
        V = si.make(200 + case, 11 + 2 * i, (ranks[i], outs[i]), 1.0 / np.sqrt(ranks[i]), dtype)
        p, _keep = pair(dn, U, V, packed=False)
        F.append(p); H.append((U.values, V.values))
    xd = to_dev(x)
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, F))
    q, k, v = dn.deinfer_lowrank_qkv(xd, F[0], F[1], F[2], ws)
    rq, rk, rv = oracle.lowrank_qkv(x.values, *H[0], *H[1], *H[2])
    for got, ref in ((q, rq), (k, rk), (v, rv)):
        assert max_err(to_host(got), ref) <= TOL[dtype]
    h = dn.deinfer_lowrank_gateup_silu(xd, F[0], F[1], ws)
    ref = oracle.lowrank_gateup_silu(x.values, *H[0], *H[1])
    assert max_err(to_host(h), ref) <= TOL[dtype]
    tg, tu = dn.deinfer_lowrank_down_proj(xd, [F[0], F[1]], ws)
    h2 = dn.deinfer_lowrank_up_glu_silu(tg, tu, F[0], F[1], ws)
    assert max_err(to_host(h2), ref) <= TOL[dtype]
    b = si.make(200 + case, 40, (1, outs[2]), 0.5, dtype)
    ya = dn.deinfer_lowrank_linear_act(xd, F[2], ws, bias=to_dev(b).reshape(-1), act=2)
    assert max_err(to_host(ya), oracle.lowrank_linear_act(x.values, *H[2], b.values.reshape(-1), 2)) <= TOL[dtype]
