"""Host-side tests of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments on the host before touching a device (no GPU needed, and no call
here ever reaches a kernel launch)."""
import ctypes
import os
import re

import pytest

import paper_2604_17709_amd as dn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000000        # 256-byte aligned, never dereferenced: every call below fails validation first


def make(d_in=64, d_out=48, r=16, dtype=dn.BF16, layout=dn.LAYOUT_RAW, U=FAKE, V=FAKE + 0x100000, ldu=None, ldv=None):
    f = dn.Factors()
    f.U, f.V = U, V
    f.d_in, f.d_out, f.r = d_in, d_out, r
    f.ldu = r if ldu is None else ldu
    f.ldv = d_out if ldv is None else ldv
    f.dtype, f.layout = dtype, layout
    return f


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in ("deinfer.h", "deinfer_testing.h"):          # the product surface and the test / measurement aids
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(deinfer_[a-z0-9_]+)\s*\(", header))
    assert {"deinfer_lowrank_linear", "deinfer_lowrank_qkv", "deinfer_lowrank_gateup_silu",
            "deinfer_lowrank_down", "deinfer_lowrank_up"} <= declared
    L = ctypes.CDLL(dn.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), name
    assert declared == set(dn.EXPORTS)
    assert dn.lib().deinfer_version() >= 1000


def test_rank_for_ratio_matches_golden_table():
    path = os.path.join(ROOT, "tests", "golden", "benchmark_ranks.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        m, n, a, b, r = map(int, line.split())
        assert dn.deinfer_rank_for_ratio(m, n, 1.0 - a / b) == r
    assert dn.deinfer_rank_for_ratio(64, 64, 0.0) == 32
    assert dn.deinfer_rank_for_ratio(64, 64, 1.0) == 0
    for bad in [(0, 4, 0.5), (4, -1, 0.5), (4, 4, 1.5), (4, 4, -0.1), (4, 4, float("nan"))]:
        with pytest.raises(dn.DeinferError) as e:
            dn.deinfer_rank_for_ratio(*bad)
        assert e.value.code == dn.ERR_INVALID_ARG
    assert dn.lib().deinfer_rank_for_ratio(4, 4, 0.5, None) == dn.ERR_INVALID_ARG


def _linear(f, x=FAKE + 0x200000, T=4, ldx=None, y=FAKE + 0x300000, ldy=None, ws=FAKE + 0x400000, ws_bytes=1 << 26):
    return dn.lib().deinfer_lowrank_linear(x, T, f.d_in if ldx is None else ldx, ctypes.byref(f),
                                           y, f.d_out if ldy is None else ldy, ws, ws_bytes, None)


def test_linear_argument_validation():
    L = dn.lib()
    assert L.deinfer_lowrank_linear(FAKE, 4, 64, None, FAKE, 48, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG
    assert "NULL" in dn.last_error()
    assert _linear(make(d_in=0)) == dn.ERR_INVALID_ARG
    assert _linear(make(r=-1)) == dn.ERR_INVALID_ARG
    assert _linear(make(dtype=7)) == dn.ERR_UNSUPPORTED
    assert _linear(make(layout=9)) == dn.ERR_UNSUPPORTED
    assert _linear(make(U=None)) == dn.ERR_INVALID_ARG
    assert _linear(make(ldu=8)) == dn.ERR_INVALID_ARG           # ldu < r
    assert _linear(make(ldv=8)) == dn.ERR_INVALID_ARG           # ldv < d_out
    assert _linear(make(), T=-1) == dn.ERR_INVALID_ARG
    assert _linear(make(), x=None) == dn.ERR_INVALID_ARG
    assert _linear(make(), y=None) == dn.ERR_INVALID_ARG
    assert _linear(make(), ldx=10) == dn.ERR_INVALID_ARG
    assert _linear(make(), ldy=10) == dn.ERR_INVALID_ARG
    assert _linear(make(), ws=None) == dn.ERR_WORKSPACE
    assert _linear(make(), ws_bytes=64) == dn.ERR_WORKSPACE
    assert "needed" in dn.last_error()
    assert _linear(make(), ws=FAKE + 0x400010) == dn.ERR_MISALIGNED
    assert _linear(make(U=FAKE + 1)) == dn.ERR_MISALIGNED
    assert _linear(make(dtype=dn.F32, layout=dn.LAYOUT_PACKED)) == dn.ERR_UNSUPPORTED   # packed holds 16-bit types only
    assert _linear(make(layout=dn.LAYOUT_PACKED), x=FAKE + 0x200002) == dn.ERR_MISALIGNED
    assert _linear(make(layout=dn.LAYOUT_PACKED, d_in=60), ldx=60) == dn.ERR_MISALIGNED   # d_in % 8
    assert _linear(make(layout=dn.LAYOUT_PACKED), ldx=68) == dn.ERR_MISALIGNED           # ldx % 8
    # T == 0 is a successful no-op (checked after the descriptor, before any pointer use)
    assert _linear(make(), T=0, x=None, y=None, ws=None, ws_bytes=0) == dn.OK


def _up(f, t=FAKE + 0x200000, T=4, ldt=None, y=FAKE + 0x300000, ldy=None, ws=FAKE + 0x400000, ws_bytes=1 << 26):
    return dn.lib().deinfer_lowrank_up(t, T, f.r if ldt is None else ldt, ctypes.byref(f),
                                       y, f.d_out if ldy is None else ldy, ws, ws_bytes, None)


def test_up_projection_argument_validation():
    L = dn.lib()
    assert L.deinfer_lowrank_up(FAKE, 4, 16, None, FAKE, 48, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG
    assert _up(make(), t=None) == dn.ERR_INVALID_ARG
    assert _up(make(), y=None) == dn.ERR_INVALID_ARG
    assert _up(make(), ldt=8) == dn.ERR_INVALID_ARG             # ldt < r
    assert "ldt" in dn.last_error()
    assert _up(make(), ldy=10) == dn.ERR_INVALID_ARG
    assert _up(make(V=None)) == dn.ERR_INVALID_ARG
    assert _up(make(), ws=None) == dn.ERR_WORKSPACE
    # the rank-space operand is narrower than d_in: a pitch between r and d_in is fine
    assert _up(make(d_in=64, r=16), T=0, ldt=16) == dn.OK
    # packed pairs: any pitch >= r and any element-aligned pointer is accepted (rows that are not whole
    # 16-byte chunks are copied, zero padded, into the workspace first); half an element is not
    pk = dict(layout=dn.LAYOUT_PACKED, r=12)
    assert _up(make(**pk), ldt=11) == dn.ERR_INVALID_ARG
    assert _up(make(**pk), ldt=16, t=FAKE + 0x200001) == dn.ERR_MISALIGNED
    assert _up(make(**pk), T=0, ldt=12, t=None, y=None, ws=None, ws_bytes=0) == dn.OK


def test_up_rope_argument_validation():
    """Errors of the rotating upward projection and of its table are found on the host, before any launch."""
    L = dn.lib()
    TAB = FAKE + 0x500000

    def up_rope(f, table=TAB, head_dim=16, T=4, t=FAKE + 0x200000, y=FAKE + 0x300000, ws=FAKE + 0x400000):
        return L.deinfer_lowrank_up_rope(t, T, f.r, ctypes.byref(f), table, head_dim, y, f.d_out, ws, 1 << 26, None)

    assert L.deinfer_lowrank_up_rope(FAKE, 4, 16, None, TAB, 16, FAKE, 48, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG
    assert up_rope(make(), head_dim=32) == dn.ERR_INVALID_ARG       # 32 does not divide d_out = 48
    assert "head_dim" in dn.last_error()
    assert up_rope(make(), head_dim=3) == dn.ERR_INVALID_ARG        # odd
    assert up_rope(make(), head_dim=0) == dn.ERR_INVALID_ARG
    assert up_rope(make(), table=None) == dn.ERR_INVALID_ARG
    assert up_rope(make(), table=TAB + 4) == dn.ERR_MISALIGNED
    assert up_rope(make(), t=None) == dn.ERR_INVALID_ARG            # then the contract of the plain upward projection
    assert up_rope(make(), ws=None) == dn.ERR_WORKSPACE
    assert up_rope(make(), T=0, table=None) == dn.OK
    assert L.deinfer_rope_table(FAKE, 4, 7, 10000.0, TAB, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_table(FAKE, -1, 8, 10000.0, TAB, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_table(FAKE, 4, 8, 0.0, TAB, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_table(None, 4, 8, 10000.0, TAB, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_rope_table(FAKE, 4, 8, 10000.0, TAB + 8, None) == dn.ERR_MISALIGNED
    assert L.deinfer_rope_table(None, 0, 8, 10000.0, None, None) == dn.OK


def test_probe_argument_validation():
    L = dn.lib()
    sink, big = FAKE + 0x500000, dn.PROBE_SINK_BYTES
    assert L.deinfer_probe_stream_read(None, 1 << 20, sink, big, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_probe_stream_read(FAKE, 1000, sink, big, None) == dn.ERR_INVALID_ARG      # not a multiple of 1024
    assert L.deinfer_probe_stream_read(FAKE, 0, sink, big, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_probe_stream_read(FAKE + 4, 1 << 20, sink, big, None) == dn.ERR_MISALIGNED
    assert L.deinfer_probe_stream_read(FAKE, 1 << 20, sink, 4096, None) == dn.ERR_WORKSPACE
    assert L.deinfer_probe_mfma_bf16(None, 8192, 10, sink, big, None, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_probe_mfma_bf16(FAKE, 4096, 10, sink, big, None, None) == dn.ERR_INVALID_ARG   # too few operand bytes
    assert L.deinfer_probe_mfma_bf16(FAKE, 8192, 0, sink, big, None, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_probe_mfma_bf16(FAKE, 8192, 10, sink + 8, big, None, None) == dn.ERR_MISALIGNED


def test_linear_act_argument_validation():
    L = dn.lib()
    f = make()
    args = lambda bias=FAKE + 0x500000, act=1, ff=f: (FAKE + 0x200000, 4, 64, ctypes.byref(ff), bias, act,
                                                      FAKE + 0x300000, 48, FAKE + 0x400000, 1 << 26, None)
    assert L.deinfer_lowrank_linear_act(*args(act=5)) == dn.ERR_UNSUPPORTED
    assert L.deinfer_lowrank_linear_act(*args(act=-1)) == dn.ERR_UNSUPPORTED
    assert L.deinfer_lowrank_linear_act(*args(bias=FAKE + 1)) == dn.ERR_MISALIGNED
    assert L.deinfer_lowrank_linear_act(*args(bias=FAKE + 8, ff=make(layout=dn.LAYOUT_PACKED))) == dn.ERR_MISALIGNED
    assert L.deinfer_lowrank_linear_act(FAKE, 4, 64, None, None, 0, FAKE, 48, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG
    # T == 0 stays a no-op
    assert L.deinfer_lowrank_linear_act(None, 0, 64, ctypes.byref(f), None, 1, None, 48, None, 0, None) == dn.OK


def test_staged_calls_argument_validation():
    L = dn.lib()
    f, g = make(), make(r=24)
    FPA = ctypes.POINTER(dn.Factors) * 2
    fa = FPA(ctypes.pointer(f), ctypes.pointer(g))
    ta = (ctypes.c_void_p * 2)(FAKE + 0x300000, FAKE + 0x310000)
    la = (ctypes.c_int64 * 2)(16, 24)
    dp = lambda n=2, t=ta, l=la, ws=FAKE + 0x400000: L.deinfer_lowrank_down_proj(FAKE + 0x200000, 4, 64, fa, n, t, l, ws, 1 << 26, None)
    assert dp(n=0) == dn.ERR_INVALID_ARG and dp(n=4) == dn.ERR_INVALID_ARG
    assert dp(t=(ctypes.c_void_p * 2)(FAKE + 0x300000, None)) == dn.ERR_INVALID_ARG        # every pair hands out its t
    assert dp(l=(ctypes.c_int64 * 2)(16, 20)) == dn.ERR_INVALID_ARG                         # ldt < r
    assert dp(ws=None) == dn.ERR_WORKSPACE
    assert L.deinfer_lowrank_down_proj(FAKE, 4, 64, None, 1, ta, la, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG
    up = lambda tg=FAKE + 0x200000, tu=FAKE + 0x210000, ldu=24, gg=g: L.deinfer_lowrank_up_glu_silu(
        tg, 16, tu, ldu, 4, ctypes.byref(f), ctypes.byref(gg), FAKE + 0x300000, 48, FAKE + 0x400000, 1 << 26, None)
    assert up(tu=None) == dn.ERR_INVALID_ARG
    assert up(ldu=20) == dn.ERR_INVALID_ARG
    assert up(gg=make(r=24, d_out=40)) == dn.ERR_INVALID_ARG                                # gate and up widths differ
    assert L.deinfer_lowrank_up_glu_silu(FAKE, 16, FAKE, 24, 4, None, ctypes.byref(g), FAKE, 48, FAKE, 1 << 20, None) == dn.ERR_INVALID_ARG


def test_group_calls_validate_shared_properties():
    L = dn.lib()
    fq, fk, fv = make(), make(d_out=16, r=8), make(d_out=16, r=8)
    args = lambda a, b, c: (FAKE, 4, 64, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                            FAKE, 48, FAKE, 16, FAKE, 16, None, 0, None, 0, FAKE, 1 << 26, None)
    assert L.deinfer_lowrank_qkv(*args(fq, fk, make(d_in=32, d_out=16, r=8))) == dn.ERR_INVALID_ARG
    assert "share" in dn.last_error()
    assert L.deinfer_lowrank_qkv(*args(fq, fk, make(d_out=16, r=8, dtype=dn.F32))) == dn.ERR_INVALID_ARG
    bad_t = (FAKE, 4, 64, ctypes.byref(fq), ctypes.byref(fk), ctypes.byref(fv),
             FAKE, 48, FAKE, 16, FAKE, 16, FAKE, 4, None, 0, FAKE, 1 << 26, None)     # ldtk < r_k
    assert L.deinfer_lowrank_qkv(*bad_t) == dn.ERR_INVALID_ARG
    g, u = make(d_out=96), make(d_out=80)
    assert L.deinfer_lowrank_gateup_silu(FAKE, 4, 64, ctypes.byref(g), ctypes.byref(u),
                                         FAKE, 96, FAKE, 1 << 26, None) == dn.ERR_INVALID_ARG
    assert "same output width" in dn.last_error()
    assert L.deinfer_lowrank_down(FAKE, 4, 64, None, FAKE, 48, FAKE, 1 << 26, None) == dn.ERR_INVALID_ARG


def test_pack_and_workspace_queries_are_host_only():
    L = dn.lib()
    n = ctypes.c_size_t(0)
    f = make(d_in=4096, d_out=4096, r=1638)
    assert L.deinfer_packed_bytes(ctypes.byref(f), ctypes.byref(n)) == dn.OK
    # r padded to 1664: U image 104 tiles x 128 k-blocks KiB, V image 256 tiles x 52 k-blocks KiB
    assert n.value == (104 * 128 + 256 * 52) * 1024
    assert L.deinfer_packed_bytes(ctypes.byref(f), None) == dn.ERR_INVALID_ARG
    assert L.deinfer_packed_bytes(None, ctypes.byref(n)) == dn.ERR_INVALID_ARG
    out = dn.Factors()
    assert L.deinfer_pack_factors(ctypes.byref(f), FAKE, 16, ctypes.byref(out), None) == dn.ERR_WORKSPACE
    assert L.deinfer_pack_factors(ctypes.byref(f), FAKE + 8, 1 << 30, ctypes.byref(out), None) == dn.ERR_MISALIGNED
    assert L.deinfer_pack_factors(ctypes.byref(make(dtype=dn.F32)), FAKE, 1 << 30, ctypes.byref(out), None) == dn.ERR_UNSUPPORTED
    assert L.deinfer_pack_factors(ctypes.byref(f), FAKE, 1 << 30, None, None) == dn.ERR_INVALID_ARG

    FP = ctypes.POINTER(dn.Factors)
    arr = (FP * 1)(ctypes.pointer(f))
    assert L.deinfer_workspace_bytes(8, arr, 1, ctypes.byref(n)) == dn.OK and n.value > 8192
    small = n.value
    assert L.deinfer_workspace_bytes(4096, arr, 1, ctypes.byref(n)) == dn.OK and n.value >= small
    assert L.deinfer_workspace_bytes(8, arr, 0, ctypes.byref(n)) == dn.ERR_INVALID_ARG
    assert L.deinfer_workspace_bytes(-1, arr, 1, ctypes.byref(n)) == dn.ERR_INVALID_ARG
    assert L.deinfer_workspace_bytes(8, None, 1, ctypes.byref(n)) == dn.ERR_INVALID_ARG
    assert L.deinfer_workspace_init(None, 1 << 20, None) == dn.ERR_WORKSPACE
    assert L.deinfer_workspace_init(FAKE, 16, None) == dn.ERR_WORKSPACE
    assert L.deinfer_workspace_init(FAKE + 4, 1 << 20, None) == dn.ERR_MISALIGNED
    assert L.deinfer_workspace_check(None, 1 << 20, None) == dn.ERR_WORKSPACE


def _ws_bytes(T, fs):
    L = dn.lib()
    FP = ctypes.POINTER(dn.Factors)
    arr = (FP * len(fs))(*[ctypes.pointer(f) for f in fs])
    n = ctypes.c_size_t(0)
    assert L.deinfer_workspace_bytes(T, arr, len(fs), ctypes.byref(n)) == dn.OK
    return n.value


def test_workspace_covers_the_group_that_runs_when_a_pair_has_rank_zero():
    """A pair of rank 0 is dropped before the dispatch (its output is zero-filled) and the remaining
    pairs are split afresh: fewer feature groups can admit more k-ranges, i.e. more partial sums, so
    the size of the group as given must cover the size of the group that runs."""
    P = dict(dtype=dn.BF16, layout=dn.LAYOUT_PACKED)
    # the shape of the report: the reduced group needs 4,202,496 bytes
    q = make(d_in=512, d_out=4096, r=64, **P)
    k0 = make(d_in=512, d_out=4096, r=0, **P)
    v = make(d_in=512, d_out=4096, r=64, **P)
    assert _ws_bytes(17, [q, k0, v]) >= _ws_bytes(17, [q, v]) >= 4202496
    import itertools
    import random
    rng = random.Random(7)
    worst = 0
    for _ in range(400):
        T = rng.choice([1, 8, 16, 17, 31, 32, 33, 64, 65, 100, 128, 129, 300, 700])
        d_in = 8 * rng.randint(4, 600)
        fs = [make(d_in=d_in, d_out=rng.choice([64, 1024, 4096, 11008]), r=rng.choice([0, 0, 16, 64, 364, 1638]), **P)
              for _ in range(rng.randint(2, 3))]
        full = _ws_bytes(T, fs)
        for m in range(1, len(fs) + 1):
            for sub in itertools.combinations(fs, m):
                if all(f.r > 0 for f in sub) and all(f.r == 0 for f in fs if not any(f is g for g in sub)):
                    worst = max(worst, _ws_bytes(T, list(sub)) - full)
    assert worst <= 0


def test_static_scratch_entry_point_validates_on_the_host():
    L = dn.lib()
    f = make(d_in=4096, d_out=4096, r=1638, layout=dn.LAYOUT_PACKED)
    assert L.deinfer_lowrank_linear_static(FAKE, 4, 4096, None, FAKE, 4096, None) == dn.ERR_INVALID_ARG
    assert L.deinfer_lowrank_linear_static(FAKE, -1, 4096, ctypes.byref(f), FAKE, 4096, None) == dn.ERR_INVALID_ARG
    # more scratch than the static array holds: refused before anything touches a device
    assert _ws_bytes(1 << 16, [f]) > dn.STATIC_SCRATCH_BYTES
    assert L.deinfer_lowrank_linear_static(FAKE, 1 << 16, 4096, ctypes.byref(f), FAKE, 4096, None) == dn.ERR_WORKSPACE
    assert "static scratch" in dn.last_error()
    assert _ws_bytes(128, [f]) <= dn.STATIC_SCRATCH_BYTES          # decode-sized calls fit
    assert L.deinfer_lowrank_linear_static(FAKE, 0, 4096, ctypes.byref(f), FAKE, 4096, None) == dn.OK
    header = open(os.path.join(ROOT, "include", "deinfer.h")).read()
    assert "#define DEINFER_STATIC_SCRATCH_BYTES (32u << 20)" in header and dn.STATIC_SCRATCH_BYTES == 32 << 20


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(dn, "_lib", None)
    monkeypatch.setattr(dn, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        dn.lib()
