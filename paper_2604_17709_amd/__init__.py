"""Python binding of the gfx950 low-rank linear-layer library (``include/deinfer.h``).

Argument marshalling only: every function here turns torch tensors into device
pointers and sizes and calls the C entry point of the same name; all arithmetic runs
in the HIP kernels of ``libdeinfer.so``.  PyTorch is used for device memory and
streams.  There is no CPU fallback: if the shared library is missing the first call
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
# DEINFER_LIBRARY_PATH names another build of the library to load (e.g. the host-sanitized one of build.py)
LIB_PATH = os.environ.get("DEINFER_LIBRARY_PATH") or os.path.join(_HERE, "libdeinfer.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_UNSUPPORTED = -2
ERR_MISALIGNED = -3
ERR_WORKSPACE = -4
ERR_DEVICE = -5

F32 = 0
BF16 = 1
F16 = 2
LAYOUT_RAW = 0
LAYOUT_PACKED = 1
PROF_DECODE_DOWN, PROF_DECODE_REDUCE, PROF_DECODE_UP, PROF_PREFILL_DOWN, PROF_PREFILL_UP = 1, 2, 3, 4, 5
STATIC_SCRATCH_BYTES = 32 << 20   # DEINFER_STATIC_SCRATCH_BYTES
TOKEN_TILE_BOTH = 384         # deinfer_set_prefill_token_tile: both tile shapes in one launch (deinfer_testing.h)

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_sz = ctypes.c_size_t


class Factors(ctypes.Structure):
    """Mirror of ``deinfer_factors_t``."""
    _fields_ = [("U", _vp), ("V", _vp),
                ("d_in", _i64), ("d_out", _i64), ("r", _i64),
                ("ldu", _i64), ("ldv", _i64),
                ("dtype", ctypes.c_int32), ("layout", ctypes.c_int32),
                ("param_reduction", ctypes.c_double)]


class DeinferError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"deinfer error {code}: {text}")
        self.code = code


EXPORTS = [
    "deinfer_last_error", "deinfer_version", "deinfer_set_profile_events",
    "deinfer_set_prefill_token_tile", "deinfer_set_prefill_feature_tile", "deinfer_set_decode_glu_one_launch",
    "deinfer_rank_for_ratio", "deinfer_probe_stream_read", "deinfer_probe_mfma_bf16",
    "deinfer_packed_bytes", "deinfer_pack_factors",
    "deinfer_workspace_bytes", "deinfer_workspace_init", "deinfer_workspace_check",
    "deinfer_lowrank_linear", "deinfer_lowrank_linear_static", "deinfer_lowrank_qkv", "deinfer_lowrank_gateup_silu",
    "deinfer_lowrank_down", "deinfer_lowrank_up", "deinfer_lowrank_linear_act",
    "deinfer_lowrank_down_proj", "deinfer_lowrank_up_glu_silu",
    "deinfer_kv_compact_plan", "deinfer_kv_compact_copy", "deinfer_rope_inplace",
    "deinfer_rope_table", "deinfer_lowrank_up_rope",
]

_lib = None


def lib() -> ctypes.CDLL:
    """Load ``libdeinfer.so`` (built by ``python -m paper_2604_17709_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2604_17709_amd.build` (there is no fallback path)")
        # torch first: the library must bind to the HIP runtime that torch has loaded (its own copy), not
        # load a second one, or its calls see no device
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        FP = ctypes.POINTER(Factors)
        L.deinfer_last_error.restype = ctypes.c_char_p
        L.deinfer_version.restype = ctypes.c_int
        L.deinfer_set_prefill_token_tile.argtypes = [ctypes.c_int]
        L.deinfer_set_prefill_feature_tile.argtypes = [ctypes.c_int]
        L.deinfer_set_decode_glu_one_launch.argtypes = [ctypes.c_int]
        L.deinfer_set_profile_events.argtypes = [ctypes.c_int, _vp, _vp]
        L.deinfer_rank_for_ratio.argtypes = [_i64, _i64, ctypes.c_double, ctypes.POINTER(_i64)]
        L.deinfer_probe_stream_read.argtypes = [_vp, _sz, _vp, _sz, _vp]
        L.deinfer_probe_mfma_bf16.argtypes = [_vp, _sz, _i64, _vp, _sz, _vp, ctypes.POINTER(ctypes.c_double)]
        _ip = ctypes.POINTER(ctypes.c_int32)
        L.deinfer_kv_compact_plan.argtypes = [_ip, _i64, _i64, _ip, _i64, _i64, _i64, _ip, _i64, _ip, _i64, _ip]
        L.deinfer_kv_compact_copy.argtypes = [_vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp]
        L.deinfer_rope_inplace.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, ctypes.c_double, ctypes.c_int, _vp]
        L.deinfer_rope_table.argtypes = [_vp, _i64, _i64, ctypes.c_double, _vp, _vp]
        L.deinfer_lowrank_up_rope.argtypes = [_vp, _i64, _i64, FP, _vp, _i64, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_packed_bytes.argtypes = [FP, ctypes.POINTER(_sz)]
        L.deinfer_pack_factors.argtypes = [FP, _vp, _sz, FP, _vp]
        L.deinfer_workspace_bytes.argtypes = [_i64, ctypes.POINTER(FP), ctypes.c_int, ctypes.POINTER(_sz)]
        L.deinfer_workspace_init.argtypes = [_vp, _sz, _vp]
        L.deinfer_workspace_check.argtypes = [_vp, _sz, _vp]
        L.deinfer_lowrank_linear.argtypes = [_vp, _i64, _i64, FP, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_down.argtypes = [_vp, _i64, _i64, FP, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_linear_static.argtypes = [_vp, _i64, _i64, FP, _vp, _i64, _vp]
        L.deinfer_lowrank_up.argtypes = [_vp, _i64, _i64, FP, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_down_proj.argtypes = [_vp, _i64, _i64, ctypes.POINTER(FP), ctypes.c_int,
                                                ctypes.POINTER(_vp), ctypes.POINTER(_i64), _vp, _sz, _vp]
        L.deinfer_lowrank_up_glu_silu.argtypes = [_vp, _i64, _vp, _i64, _i64, FP, FP, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_linear_act.argtypes = [_vp, _i64, _i64, FP, _vp, ctypes.c_int, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_qkv.argtypes = [_vp, _i64, _i64, FP, FP, FP,
                                          _vp, _i64, _vp, _i64, _vp, _i64,
                                          _vp, _i64, _vp, _i64, _vp, _sz, _vp]
        L.deinfer_lowrank_gateup_silu.argtypes = [_vp, _i64, _i64, FP, FP, _vp, _i64, _vp, _sz, _vp]
        for name in EXPORTS:
            if name not in ("deinfer_last_error",):
                getattr(L, name).restype = ctypes.c_int
        L.deinfer_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def last_error() -> str:
    return lib().deinfer_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise DeinferError(rc, last_error())


# ------------------------------------------------------------------ host-only helpers
def deinfer_rank_for_ratio(m: int, n: int, param_reduction: float) -> int:
    r = _i64(0)
    _check(lib().deinfer_rank_for_ratio(m, n, float(param_reduction), ctypes.byref(r)))
    return int(r.value)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    h = int(stream.cuda_stream)
    return h if h else None


class Pair:
    """A factor pair on the device: the ctypes descriptor plus references that keep the
    tensors it points into alive."""

    def __init__(self, desc: Factors, keep: Sequence):
        self.desc = desc
        self._keep = list(keep)

    @property
    def d_in(self): return int(self.desc.d_in)
    @property
    def d_out(self): return int(self.desc.d_out)
    @property
    def r(self): return int(self.desc.r)
    @property
    def packed(self): return self.desc.layout == LAYOUT_PACKED


def raw_pair(U, V, param_reduction: float = 0.0) -> Pair:
    """Describe row-major device tensors U[d_in x r], V[r x d_out] (last stride 1)."""
    if U.dim() != 2 or V.dim() != 2 or U.shape[1] != V.shape[0]:
        raise ValueError("U must be [d_in x r] and V [r x d_out]")
    if U.dtype != V.dtype:
        raise TypeError("U and V must share a dtype")
    if (U.shape[1] and U.stride(1) != 1) or (V.shape[1] and V.stride(1) != 1):
        raise ValueError("U and V must be row-major")
    d = Factors()
    d.U, d.V = _ptr(U), _ptr(V)
    d.d_in, d.r, d.d_out = U.shape[0], U.shape[1], V.shape[1]
    d.ldu = U.stride(0) if U.shape[0] > 1 else max(U.shape[1], 1)
    d.ldv = V.stride(0) if V.shape[0] > 1 else max(V.shape[1], 1)
    d.dtype = _dtype_code(U)
    d.layout = LAYOUT_RAW
    d.param_reduction = float(param_reduction)
    return Pair(d, [U, V])


def deinfer_packed_bytes(pair: Pair) -> int:
    n = _sz(0)
    _check(lib().deinfer_packed_bytes(ctypes.byref(pair.desc), ctypes.byref(n)))
    return int(n.value)


def deinfer_pack_factors(pair: Pair, stream=None) -> Pair:
    """Re-lay a RAW bf16 pair into the packed MFMA-fragment format (device buffer owned
    by the returned Pair)."""
    import torch
    nbytes = deinfer_packed_bytes(pair)
    dev = pair._keep[0].device
    buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    out = Factors()
    _check(lib().deinfer_pack_factors(ctypes.byref(pair.desc), _ptr(buf), nbytes,
                                      ctypes.byref(out), _stream(stream)))
    return Pair(out, [buf])


class Workspace:
    """Caller-owned scratch for the library (rank-space intermediate + sync words)."""

    def __init__(self, nbytes: int, device="cuda", stream=None, buf=None):
        """buf: an existing uint8 device tensor of nbytes, 256-byte aligned, to use instead of a new one."""
        import torch
        self.nbytes = int(nbytes)
        self.buf = torch.empty(self.nbytes, dtype=torch.uint8, device=device) if buf is None else buf
        if self.buf.numel() < self.nbytes:
            raise ValueError("workspace buffer smaller than nbytes")
        _check(lib().deinfer_workspace_init(_ptr(self.buf), self.nbytes, _stream(stream)))

    @staticmethod
    def bytes_for(T: int, pairs: Sequence[Pair]) -> int:
        return deinfer_workspace_bytes(T, pairs)

    def check(self, stream=None) -> None:
        _check(lib().deinfer_workspace_check(_ptr(self.buf), self.nbytes, _stream(stream)))


def deinfer_workspace_bytes(T: int, pairs: Sequence[Pair]) -> int:
    FP = ctypes.POINTER(Factors)
    arr = (FP * len(pairs))(*[ctypes.pointer(p.desc) for p in pairs])
    n = _sz(0)
    _check(lib().deinfer_workspace_bytes(int(T), arr, len(pairs), ctypes.byref(n)))
    return int(n.value)


def _ld(t) -> int:
    # a single row keeps the pitch of the tensor it was cut from (it decides alignment checks)
    if t.shape[0] > 1 or int(t.stride(0)) >= int(t.shape[1]):
        return max(int(t.stride(0)), 1)
    return max(int(t.shape[1]), 1)


def _rows(x, what: str):
    if x.dim() != 2 or (x.shape[1] and x.stride(1) != 1):
        raise ValueError(f"{what} must be a row-major 2-D tensor")
    return int(x.shape[0])


# ------------------------------------------------------------------ the four entry points
def deinfer_lowrank_linear(x, pair: Pair, ws: Workspace, out=None, stream=None):
    """y = (x U) V."""
    import torch
    T = _rows(x, "x")
    if out is None:
        out = torch.empty((T, pair.d_out), dtype=x.dtype, device=x.device)
    _check(lib().deinfer_lowrank_linear(_ptr(x), T, _ld(x), ctypes.byref(pair.desc),
                                        _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


def deinfer_lowrank_linear_static(x, pair: Pair, out, stream=None):
    """y = (x U) V with the library's static device scratch: no workspace, nothing allocated (``out`` is the caller's)."""
    T = _rows(x, "x")
    _check(lib().deinfer_lowrank_linear_static(_ptr(x), T, _ld(x), ctypes.byref(pair.desc), _ptr(out), _ld(out), _stream(stream)))
    return out


def deinfer_lowrank_down(h, pair: Pair, ws: Workspace, out=None, stream=None):
    """y = (h U_d) V_d."""
    import torch
    T = _rows(h, "h")
    if out is None:
        out = torch.empty((T, pair.d_out), dtype=h.dtype, device=h.device)
    _check(lib().deinfer_lowrank_down(_ptr(h), T, _ld(h), ctypes.byref(pair.desc),
                                      _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


def deinfer_lowrank_down_proj(x, pairs, ws: Workspace, t_out=None, stream=None):
    """t_i = x U_i for 1 to 3 pairs that share x: the first stage alone.  Returns the list of t_i."""
    import torch
    T = _rows(x, "x")
    n = len(pairs)
    if t_out is None:       # pitch rounded up to 8 elements: rows that deinfer_lowrank_up reads in place where r % 8 == 0
        t_out = [torch.zeros((T, max((p.r + 7) // 8 * 8, 8)), dtype=x.dtype, device=x.device)[:, :p.r] for p in pairs]
    fa = (ctypes.POINTER(Factors) * n)(*[ctypes.pointer(p.desc) for p in pairs])
    ta = (_vp * n)(*[_ptr(t) for t in t_out])
    la = (_i64 * n)(*[_ld(t) for t in t_out])
    _check(lib().deinfer_lowrank_down_proj(_ptr(x), T, _ld(x), fa, n, ta, la, _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return list(t_out)


def deinfer_lowrank_up_glu_silu(t_gate, t_up, fgate: Pair, fup: Pair, ws: Workspace, out=None, stream=None):
    """h = silu(t_gate V_gate) * (t_up V_up): the second stage of the GLU sub-layer alone."""
    import torch
    T = _rows(t_gate, "t_gate")
    if _rows(t_up, "t_up") != T:
        raise ValueError("t_gate and t_up must have the same number of rows")
    if out is None:
        out = torch.empty((T, fgate.d_out), dtype=t_gate.dtype, device=t_gate.device)
    _check(lib().deinfer_lowrank_up_glu_silu(_ptr(t_gate), _ld(t_gate), _ptr(t_up), _ld(t_up), T,
                                             ctypes.byref(fgate.desc), ctypes.byref(fup.desc),
                                             _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def deinfer_lowrank_linear_act(x, pair: Pair, ws: Workspace, bias=None, act: int = ACT_NONE, out=None, stream=None):
    """y = act((x U) V + bias): first sub-layer of a non-GLU MLP."""
    import torch
    T = _rows(x, "x")
    if out is None:
        out = torch.empty((T, pair.d_out), dtype=x.dtype, device=x.device)
    _check(lib().deinfer_lowrank_linear_act(_ptr(x), T, _ld(x), ctypes.byref(pair.desc), _ptr(bias), int(act),
                                            _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


KV_PLAN_HEADER = 4


def deinfer_kv_compact_plan(block_table, n_blocks, n_pool_blocks: int, buffer_blocks: int, block_tokens: int,
                            capacity_runs: Optional[int] = None):
    """Preparation stage (host): scan the block tables for physically contiguous blocks.

    block_table: int32 numpy [n_seqs, pitch]; n_blocks: int32 numpy [n_seqs].  Returns numpy int32
    arrays (plan, remap, positions): plan = [n_runs, n_blocks, 0, 0, (src, dst, len) ...] of fixed
    size 4 + 3 * capacity_runs, remap = [n_seqs, pitch] (the new block table, -1 padded),
    positions = [buffer_blocks * block_tokens].
    """
    import numpy as np
    bt = np.ascontiguousarray(block_table, dtype=np.int32).reshape(len(n_blocks), -1)
    nb = np.ascontiguousarray(n_blocks, dtype=np.int32)
    n_seqs, pitch = bt.shape
    cap = int(buffer_blocks if capacity_runs is None else capacity_runs)
    plan = np.zeros(KV_PLAN_HEADER + 3 * cap, dtype=np.int32)
    remap = np.full((n_seqs, pitch), -1, dtype=np.int32)
    positions = np.zeros(int(buffer_blocks) * int(block_tokens), dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    _check(lib().deinfer_kv_compact_plan(ip(bt), n_seqs, pitch, ip(nb), int(n_pool_blocks), int(buffer_blocks),
                                         int(block_tokens), ip(plan), cap, ip(remap), pitch, ip(positions)))
    return plan, remap, positions


def deinfer_kv_compact_copy(pool, block_bytes: int, plan_dev, buffer, stream=None) -> None:
    """Graph-replay stage: copy the runs of the (device) plan from the block pool into the compact buffer."""
    pool_bytes = pool.numel() * pool.element_size()
    buf_bytes = buffer.numel() * buffer.element_size()
    cap = (plan_dev.numel() - KV_PLAN_HEADER) // 3
    _check(lib().deinfer_kv_compact_copy(_ptr(pool), pool_bytes // block_bytes, int(block_bytes), _ptr(plan_dev), cap,
                                         _ptr(buffer), buf_bytes // block_bytes, _stream(stream)))


def deinfer_rope_inplace(x, n_heads: int, head_dim: int, positions_dev, theta: float = 10000.0, stream=None) -> None:
    """Rotary position embedding in place on x [T, n_heads * head_dim] (pairs i, i + head_dim / 2)."""
    import torch
    dt = _dtype_code(x)
    _check(lib().deinfer_rope_inplace(_ptr(x), _rows(x, "x"), _ld(x), int(n_heads), int(head_dim), _ptr(positions_dev),
                                      float(theta), dt, _stream(stream)))


PROBE_SINK_BYTES = 1 << 20


def deinfer_set_prefill_token_tile(tokens: int) -> None:
    """Test and measurement aid: 0 = chosen per launch, 128 or 256 = forced token tile of the T > 128 kernel."""
    _check(lib().deinfer_set_prefill_token_tile(int(tokens)))


def deinfer_set_decode_glu_one_launch(mode: int) -> None:
    """Test and measurement aid: 0 = chosen per call, 1 = the one-launch GLU second stage forced, -1 = never."""
    _check(lib().deinfer_set_decode_glu_one_launch(int(mode)))


def deinfer_set_prefill_feature_tile(features: int) -> None:
    """Test and measurement aid: 0 = chosen per launch, 128 or 256 = forced feature extent of the 128-token tiles."""
    _check(lib().deinfer_set_prefill_feature_tile(int(features)))


def deinfer_probe_stream_read(buf, nbytes: int, sink, stream=None) -> None:
    """Measurement aid: one plain read of the first ``nbytes`` of ``buf`` (a multiple of 1024)."""
    _check(lib().deinfer_probe_stream_read(_ptr(buf), int(nbytes), _ptr(sink), sink.numel() * sink.element_size(),
                                           _stream(stream)))


def deinfer_probe_mfma_bf16(operands, n_rounds: int, sink, stream=None) -> float:
    """Measurement aid: back-to-back bf16 matrix products on register operands; returns the launch's flops."""
    fl = ctypes.c_double(0.0)
    _check(lib().deinfer_probe_mfma_bf16(_ptr(operands), operands.numel() * operands.element_size(), int(n_rounds),
                                         _ptr(sink), sink.numel() * sink.element_size(), _stream(stream),
                                         ctypes.byref(fl)))
    return float(fl.value)


def deinfer_lowrank_up(t, pair: Pair, ws: Workspace, out=None, stream=None):
    """y = t V: the upward projection alone (rebuilding keys / values from the low-rank cache)."""
    import torch
    T = _rows(t, "t")
    if out is None:
        out = torch.empty((T, pair.d_out), dtype=t.dtype, device=t.device)
    _check(lib().deinfer_lowrank_up(_ptr(t), T, _ld(t), ctypes.byref(pair.desc),
                                    _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


def deinfer_rope_table(positions_dev, head_dim: int, theta: float = 10000.0, table=None, stream=None):
    """cos | sin of the rotary angles per token: fp32 [T, head_dim] (cos in the first half of a row)."""
    import torch
    T = int(positions_dev.numel())
    if table is None:
        table = torch.empty((T, int(head_dim)), dtype=torch.float32, device=positions_dev.device)
    _check(lib().deinfer_rope_table(_ptr(positions_dev), T, int(head_dim), float(theta), _ptr(table), _stream(stream)))
    return table


def deinfer_lowrank_up_rope(t, pair: Pair, table, ws: Workspace, out=None, stream=None):
    """y = rope(t V): the upward projection of keys with the rotary embedding of ``table`` applied."""
    import torch
    T = _rows(t, "t")
    if table.dim() != 2 or table.shape[0] < T or not table.is_contiguous() or table.dtype != torch.float32:
        raise ValueError("table: contiguous float32 [>= T, head_dim] expected")
    if out is None:
        out = torch.empty((T, pair.d_out), dtype=t.dtype, device=t.device)
    _check(lib().deinfer_lowrank_up_rope(_ptr(t), T, _ld(t), ctypes.byref(pair.desc), _ptr(table), int(table.shape[1]),
                                         _ptr(out), _ld(out), _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out


def deinfer_lowrank_qkv(x, fq: Pair, fk: Pair, fv: Pair, ws: Workspace,
                        out=None, t_k=None, t_v=None, stream=None):
    """q, k, v = (x U_q) V_q, (x U_k) V_k, (x U_v) V_v; optional rank-space outputs t_k, t_v."""
    import torch
    T = _rows(x, "x")
    if out is None:
        out = tuple(torch.empty((T, p.d_out), dtype=x.dtype, device=x.device) for p in (fq, fk, fv))
    q, k, v = out
    _check(lib().deinfer_lowrank_qkv(
        _ptr(x), T, _ld(x), ctypes.byref(fq.desc), ctypes.byref(fk.desc), ctypes.byref(fv.desc),
        _ptr(q), _ld(q), _ptr(k), _ld(k), _ptr(v), _ld(v),
        _ptr(t_k), _ld(t_k) if t_k is not None else 0, _ptr(t_v), _ld(t_v) if t_v is not None else 0,
        _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return q, k, v


def deinfer_lowrank_gateup_silu(x, fgate: Pair, fup: Pair, ws: Workspace, out=None, stream=None):
    """h = silu((x U_g) V_g) * ((x U_u) V_u)."""
    import torch
    T = _rows(x, "x")
    if out is None:
        out = torch.empty((T, fgate.d_out), dtype=x.dtype, device=x.device)
    _check(lib().deinfer_lowrank_gateup_silu(_ptr(x), T, _ld(x), ctypes.byref(fgate.desc),
                                             ctypes.byref(fup.desc), _ptr(out), _ld(out),
                                             _ptr(ws.buf), ws.nbytes, _stream(stream)))
    return out
