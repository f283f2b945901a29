"""ctypes front-end of the fp64 CPU oracle (``deinfer_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU package never imports
this module and this module never imports the GPU package.

Every wrapper takes numpy arrays of any float type, upcasts them to float64
(exact for fp32 and bf16-valued inputs) and returns float64 results.  The
arithmetic itself lives in the C file; nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deinfer_oracle.c")
_SO = os.path.join(_HERE, "libdeinfer_oracle.so")

_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)


_SAN_SO = os.path.join(_HERE, "libdeinfer_oracle_san.so")


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (errors abort).  The
    process that loads it needs gcc's libasan preloaded; set DEINFER_ORACLE_SO to the returned path."""
    if (not os.path.exists(_SAN_SO)) or os.path.getmtime(_SAN_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-o", _SAN_SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SAN_SO


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over token rows). Returns the .so path.
    DEINFER_ORACLE_SO names a build to load instead (the sanitized one, see build_sanitized)."""
    if os.environ.get("DEINFER_ORACLE_SO"):
        return os.environ["DEINFER_ORACLE_SO"]
    if force or (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        L = _lib
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_rank_for_keep.restype = _i64
        L.oracle_rank_for_keep.argtypes = [_i64] * 4
        L.oracle_param_count.restype = _i64
        L.oracle_param_count.argtypes = [_i64] * 3
        L.oracle_comm_volume.restype = None
        L.oracle_comm_volume.argtypes = [_i64] * 10 + [ctypes.POINTER(_i64)]
        L.oracle_silu.restype = ctypes.c_double
        L.oracle_silu.argtypes = [ctypes.c_double]
        L.oracle_round_to_bf16.restype = ctypes.c_double
        L.oracle_round_to_bf16.argtypes = [ctypes.c_double]
        L.oracle_down_projection.restype = None
        L.oracle_down_projection.argtypes = [_dp, _i64, _i64, _dp, _i64, _i64, _i64, _dp, _i64]
        L.oracle_up_projection.restype = None
        L.oracle_up_projection.argtypes = [_dp, _i64, _i64, _dp, _i64, _i64, _i64, _dp, _i64]
        L.oracle_up_glu_silu.restype = ctypes.c_int
        L.oracle_up_glu_silu.argtypes = [_dp, _i64, _dp, _i64, _i64, _dp, _i64, _dp, _i64, _i64, _i64, _i64, _dp, _i64]
        L.oracle_relu.restype = ctypes.c_double
        L.oracle_relu.argtypes = [ctypes.c_double]
        L.oracle_gelu.restype = ctypes.c_double
        L.oracle_gelu.argtypes = [ctypes.c_double]
        L.oracle_lowrank_linear_act.restype = ctypes.c_int
        L.oracle_lowrank_linear_act.argtypes = [_dp, _i64, _i64, _dp, _i64, _dp, _i64, _i64, _i64, _i64,
                                                _dp, ctypes.c_int, _dp, _i64]
        L.oracle_lowrank_linear.restype = ctypes.c_int
        L.oracle_lowrank_linear.argtypes = [_dp, _i64, _i64, _dp, _i64, _dp, _i64,
                                            _i64, _i64, _i64, _dp, _i64, _dp]
        L.oracle_lowrank_qkv.restype = ctypes.c_int
        L.oracle_lowrank_qkv.argtypes = ([_dp, _i64, _i64, _i64]
                                         + [_dp, _i64, _dp, _i64, _i64, _i64] * 3
                                         + [_dp, _i64] * 3 + [_dp, _dp])
        L.oracle_lowrank_gateup_silu.restype = ctypes.c_int
        L.oracle_lowrank_gateup_silu.argtypes = ([_dp, _i64, _i64, _i64]
                                                 + [_dp, _i64, _dp, _i64, _i64] * 2
                                                 + [_i64, _dp, _i64])
        L.oracle_lowrank_down.restype = ctypes.c_int
        L.oracle_lowrank_down.argtypes = [_dp, _i64, _i64, _dp, _i64, _dp, _i64,
                                          _i64, _i64, _i64, _dp, _i64]
        L.oracle_svd_factor.restype = ctypes.c_int
        L.oracle_svd_factor.argtypes = [_dp, _i64, _i64, _i64, _dp, _dp, _dp]
    return _lib


def _f64(a) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.ndim != 2:
        raise ValueError("oracle wrappers take 2-D arrays")
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(_dp)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def rank_for_keep(m: int, n: int, keep_num: int, keep_den: int) -> int:
    """floor(keep * m * n / (m + n)) with keep = keep_num / keep_den (exact integers)."""
    return int(lib().oracle_rank_for_keep(m, n, keep_num, keep_den))


def param_count(m: int, n: int, k: int) -> int:
    return int(lib().oracle_param_count(m, n, k))


def comm_volume(h, h_kv, m, l_q, l_k, l_v, l_o, l_gate, l_up, l_down):
    out = (_i64 * 4)()
    lib().oracle_comm_volume(h, h_kv, m, l_q, l_k, l_v, l_o, l_gate, l_up, l_down, out)
    return {"unoptimized": out[0], "all_gather": out[1], "reduce_sum": out[2], "lowrank_total": out[3]}


def silu(z: float) -> float:
    return float(lib().oracle_silu(float(z)))


def round_to_bf16(v: float) -> float:
    return float(lib().oracle_round_to_bf16(float(v)))


def _check_pair(x, U, V):
    if x.shape[1] != U.shape[0] or U.shape[1] != V.shape[0]:
        raise ValueError(f"shape mismatch x{x.shape} U{U.shape} V{V.shape}")


def down_projection(x, U) -> np.ndarray:
    x, U = _f64(x), _f64(U)
    T, d_in = x.shape
    r = U.shape[1]
    t = np.empty((T, max(r, 0)), dtype=np.float64)
    if T and r:
        lib().oracle_down_projection(_p(x), T, d_in, _p(U), r, d_in, r, _p(t), r)
    return t


def up_projection(t, V) -> np.ndarray:
    t, V = _f64(t), _f64(V)
    T, r = t.shape
    d_out = V.shape[1]
    y = np.zeros((T, d_out), dtype=np.float64)
    if T and d_out:
        lib().oracle_up_projection(_p(t), T, max(r, 1), _p(V), d_out, r, d_out, _p(y), d_out)
    return y


def up_glu_silu(t_gate, V_gate, t_up, V_up) -> np.ndarray:
    """h = silu(t_gate V_gate) * (t_up V_up): the second stage of the GLU sub-layer alone."""
    tg, Vg, tu, Vu = _f64(t_gate), _f64(V_gate), _f64(t_up), _f64(V_up)
    T, rg = tg.shape
    ru = tu.shape[1]
    d_ff = Vg.shape[1]
    if Vg.shape[0] != rg or Vu.shape != (ru, d_ff) or tu.shape[0] != T:
        raise ValueError("shape mismatch")
    h = np.zeros((T, d_ff), dtype=np.float64)
    if T and d_ff:
        rc = lib().oracle_up_glu_silu(_p(tg), max(rg, 1), _p(Vg), d_ff, rg, _p(tu), max(ru, 1), _p(Vu), d_ff, ru,
                                      T, d_ff, _p(h), d_ff)
        if rc:
            raise MemoryError("oracle_up_glu_silu")
    return h


def lowrank_linear(x, U, V, return_t: bool = False):
    """y = (x U) V in fp64; optionally also the rank-space intermediate t = x U."""
    x, U, V = _f64(x), _f64(U), _f64(V)
    _check_pair(x, U, V)
    T, d_in = x.shape
    r, d_out = V.shape
    y = np.zeros((T, d_out), dtype=np.float64)
    t = np.zeros((T, r), dtype=np.float64) if return_t else None
    if T and d_out:
        rc = lib().oracle_lowrank_linear(_p(x), T, d_in, _p(U), max(r, 1), _p(V), d_out,
                                         d_in, r, d_out, _p(y), d_out,
                                         _p(t) if (t is not None and r) else None)
        if rc:
            raise MemoryError("oracle_lowrank_linear")
    return (y, t) if return_t else y


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def relu(z: float) -> float:
    return float(lib().oracle_relu(float(z)))


def gelu(z: float) -> float:
    return float(lib().oracle_gelu(float(z)))


def lowrank_linear_act(x, U, V, bias=None, act: int = ACT_NONE):
    """y = act((x U) V + bias) in fp64 (non-GLU MLP first sub-layer)."""
    x, U, V = _f64(x), _f64(U), _f64(V)
    _check_pair(x, U, V)
    T, d_in = x.shape
    r, d_out = V.shape
    b = None if bias is None else np.ascontiguousarray(np.asarray(bias, dtype=np.float64).reshape(d_out))
    y = np.zeros((T, d_out), dtype=np.float64)
    if T and d_out:
        rc = lib().oracle_lowrank_linear_act(_p(x), T, d_in, _p(U), max(r, 1), _p(V), d_out, d_in, r, d_out,
                                             _p(b) if b is not None else None, int(act), _p(y), d_out)
        if rc:
            raise RuntimeError("oracle_lowrank_linear_act: %d" % rc)
    return y


def lowrank_qkv(x, Uq, Vq, Uk, Vk, Uv, Vv, return_t: bool = False):
    x = _f64(x)
    Uq, Vq, Uk, Vk, Uv, Vv = map(_f64, (Uq, Vq, Uk, Vk, Uv, Vv))
    for U, V in ((Uq, Vq), (Uk, Vk), (Uv, Vv)):
        _check_pair(x, U, V)
    T, d_in = x.shape
    q = np.zeros((T, Vq.shape[1])); k = np.zeros((T, Vk.shape[1])); v = np.zeros((T, Vv.shape[1]))
    tk = np.zeros((T, Vk.shape[0])) if return_t else None
    tv = np.zeros((T, Vv.shape[0])) if return_t else None
    if T:
        rc = lib().oracle_lowrank_qkv(
            _p(x), T, d_in, d_in,
            _p(Uq), max(Uq.shape[1], 1), _p(Vq), max(Vq.shape[1], 1), Vq.shape[0], Vq.shape[1],
            _p(Uk), max(Uk.shape[1], 1), _p(Vk), max(Vk.shape[1], 1), Vk.shape[0], Vk.shape[1],
            _p(Uv), max(Uv.shape[1], 1), _p(Vv), max(Vv.shape[1], 1), Vv.shape[0], Vv.shape[1],
            _p(q), max(q.shape[1], 1), _p(k), max(k.shape[1], 1), _p(v), max(v.shape[1], 1),
            _p(tk) if (tk is not None and tk.size) else None,
            _p(tv) if (tv is not None and tv.size) else None)
        if rc:
            raise MemoryError("oracle_lowrank_qkv")
    return (q, k, v, tk, tv) if return_t else (q, k, v)


def lowrank_gateup_silu(x, Ug, Vg, Uu, Vu) -> np.ndarray:
    x, Ug, Vg, Uu, Vu = map(_f64, (x, Ug, Vg, Uu, Vu))
    _check_pair(x, Ug, Vg); _check_pair(x, Uu, Vu)
    if Vg.shape[1] != Vu.shape[1]:
        raise ValueError("gate and up must have the same output width")
    T, d_in = x.shape
    d_ff = Vg.shape[1]
    h = np.zeros((T, d_ff), dtype=np.float64)
    if T and d_ff:
        rc = lib().oracle_lowrank_gateup_silu(
            _p(x), T, d_in, d_in,
            _p(Ug), max(Ug.shape[1], 1), _p(Vg), d_ff, Vg.shape[0],
            _p(Uu), max(Uu.shape[1], 1), _p(Vu), d_ff, Vu.shape[0],
            d_ff, _p(h), d_ff)
        if rc:
            raise MemoryError("oracle_lowrank_gateup_silu")
    return h


def lowrank_down(h, U, V) -> np.ndarray:
    h, U, V = _f64(h), _f64(U), _f64(V)
    _check_pair(h, U, V)
    T, d_ff = h.shape
    r, d_out = V.shape
    y = np.zeros((T, d_out), dtype=np.float64)
    if T and d_out:
        rc = lib().oracle_lowrank_down(_p(h), T, d_ff, _p(U), max(r, 1), _p(V), d_out,
                                       d_ff, r, d_out, _p(y), d_out)
        if rc:
            raise MemoryError("oracle_lowrank_down")
    return y


def svd_factor(W, k: int):
    """Truncated-SVD factor pair (A, B, sigma) with the symmetric sqrt(Sigma) split."""
    W = _f64(W)
    m, n = W.shape
    if m < n:  # factor the transpose, then swap roles: W = (B'^T)(A'^T)
        A2, B2, s = svd_factor(W.T.copy(), k)
        return np.ascontiguousarray(B2.T), np.ascontiguousarray(A2.T), s
    A = np.zeros((m, k)); B = np.zeros((k, n)); s = np.zeros(n)
    rc = lib().oracle_svd_factor(_p(W), m, n, k, _p(A), _p(B), _p(s))
    if rc < 0:
        raise RuntimeError(f"oracle_svd_factor failed ({rc})")
    return A, B, s
