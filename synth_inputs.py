"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and bench.py.

This module holds NO arithmetic of the method (no matrix product, no activation,
no rank rule): only a counter-based random generator, the bf16 storage rounding
and the shape tables of the benchmark configurations.  Both sides of a parity
test draw their inputs here so that they see identical bit patterns.

Generator: splitmix64 over a 64-bit counter (stream id in the high bits) ->
two uniforms -> Box-Muller.  Values are produced in float64, scaled by the
requested standard deviation, rounded once to the storage type (float32, or
bfloat16 with round-to-nearest-even) and handed out both as the storage bit
pattern and as exact float32 values.

Shapes: Llama-7B / 13B / 70B decoder projections (hidden, FFN and GQA widths as
in the public model cards); activations ~ N(0, 1), weights ~ N(0, std 0.02)
for the bf16 configurations, N(0, std 1/sqrt(fan_in)) for the fp32 one.
"""
from __future__ import annotations

import os
from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    """Vectorised splitmix64 finaliser on uint64 counters (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _normal_chunk(base: np.uint64, s: int, e: int, out: np.ndarray) -> None:
    idx = np.arange(s, e, dtype=np.uint64)
    with np.errstate(over="ignore"):
        c0 = base + idx * np.uint64(2)
    a = _splitmix64(c0)
    b = _splitmix64(c0 + np.uint64(1))
    # 53-bit uniforms; u1 in (0, 1], u2 in [0, 1)
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    rad = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * np.pi) * u2
    out[2 * s:2 * e:2] = rad * np.cos(ang)
    out[2 * s + 1:2 * e:2] = rad * np.sin(ang)


def normal(seed: int, stream: int, n: int, std: float = 1.0, start: int = 0) -> np.ndarray:
    """n standard normals * std as float64: elements [start, start + n) of the stream
    (seed, stream); element i depends only on (seed, stream, i).  start must be even."""
    if start % 2:
        raise ValueError("start must be even (values are drawn in pairs)")
    n_pairs = (n + 1) // 2
    out = np.empty(2 * n_pairs, dtype=np.float64)
    chunk = 1 << 20
    base = ((np.uint64(seed & 0xFFFF) << np.uint64(48)) | (np.uint64(stream & 0xFFFF) << np.uint64(32))) \
        + np.uint64(start)
    spans = [(s, min(n_pairs, s + chunk)) for s in range(0, n_pairs, chunk)]
    if len(spans) > 2:      # numpy releases the GIL inside the ufuncs: chunks run in parallel
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(lambda se: _normal_chunk(base, se[0], se[1], out), spans))
    else:
        for s, e in spans:
            _normal_chunk(base, s, e, out)
    return out[:n] * std


def small_ints(seed: int, stream: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi] as float64 (for bit-exact brute-force cases)."""
    base = (np.uint64(seed & 0xFFFF) << np.uint64(48)) | (np.uint64(stream & 0xFFFF) << np.uint64(32))
    with np.errstate(over="ignore"):
        z = _splitmix64(base + np.arange(n, dtype=np.uint64))
    span = np.uint64(hi - lo + 1)
    return (z % span).astype(np.int64).astype(np.float64) + float(lo)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Tensor:
    """A generated tensor: ``bits`` is what goes to the GPU (float32 array, or uint16
    bf16 / fp16 patterns); ``values`` are the same numbers as exact float32."""
    dtype: str          # "f32" | "bf16" | "f16"
    bits: np.ndarray
    values: np.ndarray

    @property
    def shape(self):
        return self.values.shape


def make(seed: int, stream: int, shape: Tuple[int, int], std: float, dtype: str) -> Tensor:
    v = normal(seed, stream, shape[0] * shape[1], std).astype(np.float32).reshape(shape)
    return store(v, dtype)


def make_rows(seed: int, stream: int, rows, width: int, std: float, dtype: str) -> Tensor:
    """Selected rows of the (n_rows x width) tensor that make(seed, stream, ...) would draw
    (width must be even), without generating the other rows."""
    v = np.stack([normal(seed, stream, width, std, start=int(r) * width) for r in rows]).astype(np.float32)
    return store(v, dtype)


def store(v: np.ndarray, dtype: str) -> Tensor:
    """Round an array once to the storage type."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    if dtype == "f32":
        return Tensor("f32", v, v)
    if dtype == "bf16":
        b = f32_to_bf16_bits(v)
        return Tensor("bf16", b, bf16_bits_to_f32(b).reshape(v.shape))
    if dtype == "f16":
        h = v.astype(np.float16)                     # round to nearest even (storage rounding, no arithmetic of the method)
        return Tensor("f16", h.view(np.uint16), h.astype(np.float32))
    raise ValueError(dtype)


# ---------------------------------------------------------------------------
# Benchmark configurations (shapes only).  Each projection is (d_in, d_out).
# The rank of each pair is NOT decided here: callers obtain it from the side
# they are testing (the oracle's rule or the library's rule) and pass it in.
# ---------------------------------------------------------------------------
@dataclass
class BlockShape:
    name: str
    hidden: int
    ffn: int
    kv_width: int
    keep_num: int       # kept parameter fraction = keep_num / keep_den
    keep_den: int
    dtype: str = "bf16"
    weight_std: float = 0.02
    glu: bool = True    # False: non-GLU MLP, "gate" is its first layer (bias, activation), there is no "up"

    def projections(self) -> Dict[str, Tuple[int, int]]:
        p = {
            "q": (self.hidden, self.hidden), "k": (self.hidden, self.kv_width),
            "v": (self.hidden, self.kv_width), "o": (self.hidden, self.hidden),
            "gate": (self.hidden, self.ffn), "up": (self.hidden, self.ffn),
            "down": (self.ffn, self.hidden),
        }
        if not self.glu:
            del p["up"]
        return p


BLOCKS: Dict[str, BlockShape] = {
    # Llama-7B-shaped block, 20 % parameter reduction (decode T = 1, 8, 32, 64)
    "llama7b_keep80": BlockShape("llama7b_keep80", 4096, 11008, 4096, 4, 5),
    # same block at 40 % and 60 % reduction (prefill 4 x 2048 tokens)
    "llama7b_keep60": BlockShape("llama7b_keep60", 4096, 11008, 4096, 3, 5),
    "llama7b_keep40": BlockShape("llama7b_keep40", 4096, 11008, 4096, 2, 5),
    # Llama-13B-shaped, 40 % reduction (mixed 16 x 512 prefill + 64 decode tokens)
    "llama13b_keep60": BlockShape("llama13b_keep60", 5120, 13824, 5120, 3, 5),
    # Llama-70B-shaped GQA layer (8 kv heads -> k/v width 1024), 60 % reduction
    "llama70b_keep40": BlockShape("llama70b_keep40", 8192, 28672, 1024, 2, 5),
    # OPT-30B-shaped block (non-GLU MLP with ReLU and biases, full-width k/v), 40 % reduction
    "opt30b_keep60": BlockShape("opt30b_keep60", 7168, 28672, 7168, 3, 5, glu=False),
}

_ORDER = ["q", "k", "v", "o", "gate", "up", "down"]


def block_tensors(shape: BlockShape, ranks: Dict[str, int], T: int, seed: int,
                  names: List[str] | None = None) -> Dict[str, Tensor]:
    """Draw x, h_in (input of the down projection), a (input of the o projection) and the
    factor pairs U_<p>[d_in x r], V_<p>[r x d_out] of the requested projections.
    Stream ids are fixed per tensor so a subset draws the same numbers as the full set."""
    out: Dict[str, Tensor] = {}
    out["x"] = make(seed, 1, (T, shape.hidden), 1.0, shape.dtype)
    out["a"] = make(seed, 2, (T, shape.hidden), 1.0, shape.dtype)
    out["h_in"] = make(seed, 3, (T, shape.ffn), 1.0, shape.dtype)
    proj = shape.projections()
    if not shape.glu:      # biases of the two MLP layers
        out["b_gate"] = make(seed, 4, (1, shape.ffn), shape.weight_std, shape.dtype)
        out["b_down"] = make(seed, 5, (1, shape.hidden), shape.weight_std, shape.dtype)
    for i, p in enumerate(_ORDER):
        if p not in proj or (names is not None and p not in names):
            continue
        d_in, d_out = proj[p]
        r = ranks[p]
        out["U_" + p] = make(seed, 16 + 2 * i, (d_in, r), shape.weight_std, shape.dtype)
        out["V_" + p] = make(seed, 17 + 2 * i, (r, d_out), shape.weight_std, shape.dtype)
    return out


def single_linear_f32(seed: int = 0, T: int = 16, d_in: int = 512, r: int = 64, d_out: int = 512):
    """The small fp32 case: x ~ N(0,1), U ~ N(0, std 1/sqrt(d_in)), V ~ N(0, std 1/sqrt(r))."""
    x = make(seed, 1, (T, d_in), 1.0, "f32")
    U = make(seed, 2, (d_in, r), 1.0 / np.sqrt(d_in), "f32")
    V = make(seed, 3, (r, d_out), 1.0 / np.sqrt(r), "f32")
    return x, U, V


# ---------------------------------------------------------------------------------------------
# Block tables of a paged cache (inputs of the contiguous-block scan; no part of the scan itself)
def paged_block_tables(seed: int, prompt_blocks, decode_blocks, n_pool_blocks: int, recycled: int = 0):
    """Block tables as a paged-cache allocator leaves them after prefill and interleaved decoding.

    The allocator hands out physical block ids from a queue: first ``recycled`` ids in a seeded
    random order (blocks that earlier, finished sequences gave back), then the untouched ids in
    ascending order.  Every sequence first takes its ``prompt_blocks[s]`` blocks in one go
    (prefill: a physically contiguous run unless it falls into the recycled part), then the
    sequences take one block each, round after round, until sequence s holds
    ``prompt_blocks[s] + decode_blocks[s]`` blocks (decoding: neighbours in a sequence's table
    end up ``n_seqs`` apart or scattered).  Returns ``(table, n_blocks)``: int32
    ``[n_seqs, max_blocks]`` padded with -1, and int32 ``[n_seqs]``.
    """
    prompt_blocks = [int(v) for v in prompt_blocks]
    decode_blocks = [int(v) for v in decode_blocks]
    n_seqs = len(prompt_blocks)
    assert len(decode_blocks) == n_seqs
    total = sum(prompt_blocks) + sum(decode_blocks)
    assert 0 <= recycled <= n_pool_blocks and total <= n_pool_blocks
    # recycled ids: a seeded shuffle of a seeded choice of ids (sort by random keys)
    keys = _splitmix64(np.arange(n_pool_blocks, dtype=np.uint64) + (np.uint64(seed) << np.uint64(32)))
    chosen = np.sort(np.argsort(keys, kind="stable")[:recycled])
    keys2 = _splitmix64(chosen.astype(np.uint64) + (np.uint64(seed + 1) << np.uint64(32)))
    first = chosen[np.argsort(keys2, kind="stable")]
    mask = np.ones(n_pool_blocks, dtype=bool)
    mask[chosen] = False
    queue = np.concatenate([first, np.nonzero(mask)[0]]).astype(np.int64)
    n_blocks = np.array([p + d for p, d in zip(prompt_blocks, decode_blocks)], dtype=np.int32)
    table = np.full((n_seqs, max(1, int(n_blocks.max()) if n_seqs else 1)), -1, dtype=np.int32)
    head = 0
    fill = [0] * n_seqs
    for s in range(n_seqs):
        for _ in range(prompt_blocks[s]):
            table[s, fill[s]] = queue[head]; head += 1; fill[s] += 1
    for rnd_ in range(max(decode_blocks) if n_seqs else 0):
        for s in range(n_seqs):
            if rnd_ < decode_blocks[s]:
                table[s, fill[s]] = queue[head]; head += 1; fill[s] += 1
    return table, n_blocks
