"""CPU oracle for the paged-cache side of key/value reconstruction (Sec. 4.2) and for the
rotary position embedding applied to the rebuilt keys.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and nothing in the GPU package); it imports
nothing from the GPU package.  Plain Python loops and numpy in float64 / exact integers, written
for reading, not for speed.

What the paper fixes (Sec. 4.2): in a preparation stage a scan over the block tables finds the
logical blocks that are physically contiguous and derives a "remapping index list" that acts as
the block table of a compact buffer; in the graph-replay stage the contiguous pieces are copied
one after the other into that buffer, the compact low-rank cache is multiplied by the upward
matrix, and a rotary position embedding is applied in place where the model has one.

Readings (the paper gives no formulas here):
  * walk order = sequences in table order, logical blocks in order; the compact buffer receives
    the blocks in exactly that order, so buffer block d belongs to the d-th block of the walk;
  * a run is a maximal stretch of the walk whose physical ids increase by one; it may cross from
    one sequence into the next (both source and destination stay contiguous there);
  * whole blocks are copied, also the partly filled last block of a sequence;
  * the rotary embedding is the usual one of LLaMA-type models (the paper names it but prints no
    formula): within each head of width D the elements i and i + D/2 form a pair that is rotated
    by the angle pos * theta ** (-2 i / D).
"""
from __future__ import annotations

import numpy as np


def contiguous_runs(table, n_blocks):
    """Scan of the preparation stage.

    table: [n_seqs][>= n_blocks[s]] physical block ids; n_blocks: blocks per sequence.
    Returns (runs, remap): runs = list of (src_block, dst_block, length) in walk order;
    remap[s][i] = buffer block that holds logical block i of sequence s (a list per sequence).
    """
    runs = []
    remap = []
    d = 0                       # next free block of the compact buffer
    for s in range(len(n_blocks)):
        row = []
        for i in range(int(n_blocks[s])):
            p = int(table[s][i])
            if runs and runs[-1][0] + runs[-1][2] == p:
                runs[-1][2] += 1            # p continues the current run (destination is contiguous by construction)
            else:
                runs.append([p, d, 1])
            row.append(d)
            d += 1
        remap.append(row)
    return [tuple(r) for r in runs], remap


def copy_runs(pool, runs, buffer_blocks):
    """Graph-replay copy: pool [n_pool_blocks, ...] -> compact buffer [buffer_blocks, ...], run by run.
    Blocks of the buffer that no run writes keep the fill value 0."""
    pool = np.asarray(pool)
    buf = np.zeros((buffer_blocks,) + pool.shape[1:], dtype=pool.dtype)
    for src, dst, n in runs:
        for j in range(n):
            buf[dst + j] = pool[src + j]
    return buf


def gather_blocks(pool, table, n_blocks, buffer_blocks):
    """What the compact buffer must hold, straight from the definition of a block table:
    the d-th block of the walk is pool[table[s][i]]."""
    pool = np.asarray(pool)
    buf = np.zeros((buffer_blocks,) + pool.shape[1:], dtype=pool.dtype)
    d = 0
    for s in range(len(n_blocks)):
        for i in range(int(n_blocks[s])):
            buf[d] = pool[int(table[s][i])]
            d += 1
    return buf


def token_positions(n_blocks, block_tokens, buffer_blocks):
    """Position inside its sequence of every token slot of the compact buffer (0 for unused blocks)."""
    pos = np.zeros(buffer_blocks * block_tokens, dtype=np.int64)
    d = 0
    for s in range(len(n_blocks)):
        for i in range(int(n_blocks[s])):
            for j in range(block_tokens):
                pos[d * block_tokens + j] = i * block_tokens + j
            d += 1
    return pos


def rope(x, positions, n_heads, head_dim, theta=10000.0):
    """Rotary position embedding, float64.  x: [T, n_heads * head_dim]; positions: [T]."""
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    half = head_dim // 2
    assert head_dim % 2 == 0 and x.shape[1] == n_heads * head_dim
    y = np.empty_like(x)
    for t in range(T):
        for h in range(n_heads):
            base = h * head_dim
            for i in range(half):
                ang = float(positions[t]) * theta ** (-2.0 * i / head_dim)
                c, s = np.cos(ang), np.sin(ang)
                a, b = x[t, base + i], x[t, base + i + half]
                y[t, base + i] = a * c - b * s
                y[t, base + i + half] = b * c + a * s
    return y


def rope_table(positions, head_dim, theta=10000.0):
    """The angles of `rope` as a table, float64 [T, head_dim]: row t holds cos(a_ti) for i < D/2 and
    then sin(a_ti), a_ti = positions[t] * theta^(-2 i / D).  (The upward projection with a rotary
    epilogue takes its angles in this form.)"""
    half = head_dim // 2
    assert head_dim % 2 == 0
    tab = np.empty((len(positions), head_dim), dtype=np.float64)
    for t in range(len(positions)):
        for i in range(half):
            ang = float(positions[t]) * theta ** (-2.0 * i / head_dim)
            tab[t, i] = np.cos(ang)
            tab[t, half + i] = np.sin(ang)
    return tab
