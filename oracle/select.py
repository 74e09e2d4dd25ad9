"""Oracle: adaptive choice between per-sequence and per-document sharding.

TEST INFRASTRUCTURE ONLY.  Nothing here is used by the HIP path.

Paper Section 5.3 (Adaptive Sharding Selection): after the K/V all-gather, work out the
attention kernel's input shapes (number of query tokens and of key/value tokens) under both
shardings, estimate the kernel latency of each and take the faster one.  The estimate has three
steps: (1) the floating-point operations of the attention computation, with every document
chunk padded to a multiple of the kernel's tile size; (2) the achieved TFLOP/s for that shape,
looked up in a table collected by offline profiling; (3) latency = operations / achieved rate.

Readings where the paper leaves the detail open (shared with the C library by design):
  * a "chunk" is one segment of the sharding map (a maximal run of a rank's slots inside one
    chunk of one document); its shape is Q_len = its number of slots (padding slots included:
    the kernel processes them) and KV_len = seg_k_end - seg_k_begin, the keys its last row sees;
  * padding to the tile: the segment's rows are cut into row tiles of tile_q; the rows of a tile
    end at local row e = min((t+1)*tile_q, Q_len), and see KV_len - Q_len + e keys, which is
    rounded up to a multiple of tile_k; a tile counts tile_q * (that many) query-key pairs.
    A segment without a real row (KV_len = 0) counts nothing;
  * operations per pair: 4*D forward plus 10*D backward per query head;
  * the table is given on a grid of Q_len x KV_len; the rate of a shape is the bilinear
    interpolation in the two lengths, clamped to the grid's edges;
  * the ranks of a CP group run side by side, so the latency of a sharding is the MAXIMUM over
    ranks of the rank's summed segment latencies;
  * ties go to per-sequence sharding (the default the paper starts from).

All arithmetic is IEEE double in a fixed order so that the C library can match it exactly.

Pins (tests/test_oracle_select.py): hand-worked example under tests/golden/; closed form of the
padded pair count of a whole causal document; padded >= useful pairs; a flat table makes the
latency proportional to the padded operations; one document with 2*CP | L predicts the same
latency for both shardings.
"""
from __future__ import annotations

import numpy as np

from . import shard as _shard

PER_SEQ, PER_DOC = 1, 0     # the sharding modes' numbers (same as oracle.shard)


def padded_pairs(q_len: int, kv_len: int, tile_q: int, tile_k: int) -> int:
    """Query-key pairs the tiled kernel executes for one segment (see module docstring)."""
    if kv_len <= 0 or q_len <= 0:
        return 0
    total = 0
    n_tiles = -(-q_len // tile_q)
    for t in range(n_tiles):
        e = min((t + 1) * tile_q, q_len)
        vis = kv_len - q_len + e
        if vis <= 0:
            continue
        total += tile_q * (-(-vis // tile_k) * tile_k)
    return total


def lookup(q_grid, kv_grid, tflops, q_len: int, kv_len: int) -> float:
    """Bilinear interpolation of the profiled rate, clamped at the grid's edges."""
    def bracket(grid, x):
        n = len(grid)
        if x <= grid[0]:
            return 0, 0, 0.0
        if x >= grid[n - 1]:
            return n - 1, n - 1, 0.0
        i = 0
        while grid[i + 1] < x:
            i += 1
        return i, i + 1, float(x - grid[i]) / float(grid[i + 1] - grid[i])
    i0, i1, wq = bracket(q_grid, q_len)
    j0, j1, wk = bracket(kv_grid, kv_len)
    top = float(tflops[i0][j0]) * (1.0 - wk) + float(tflops[i0][j1]) * wk
    bot = float(tflops[i1][j0]) * (1.0 - wk) + float(tflops[i1][j1]) * wk
    return top * (1.0 - wq) + bot * wq


def rank_latency(doc_len, cp: int, rank: int, mode: int, hq: int, head_dim: int, tile_q: int, tile_k: int,
                 q_grid, kv_grid, tflops) -> float:
    """Predicted attention forward+backward latency (seconds) of one rank under one sharding."""
    sh = _shard.shard(doc_len, cp, rank, mode)
    cu_q, kb, ke = sh["cu_seqlens_q"], sh["seg_k_begin"], sh["seg_k_end"]
    flops_per_pair = 14.0 * float(head_dim) * float(hq)
    lat = 0.0
    for s in range(len(kb)):
        q_len = int(cu_q[s + 1] - cu_q[s])
        kv_len = int(ke[s] - kb[s])
        pairs = padded_pairs(q_len, kv_len, tile_q, tile_k)
        if pairs == 0:
            continue
        rate = lookup(q_grid, kv_grid, tflops, q_len, kv_len) * 1e12
        lat = lat + (float(pairs) * flops_per_pair) / rate
    return lat


def select(doc_len, cp: int, hq: int, head_dim: int, tile_q: int, tile_k: int, q_grid, kv_grid, tflops):
    """-> (mode, latency_per_seq, latency_per_doc): the sharding with the lower predicted latency."""
    lat = {}
    for mode in (PER_SEQ, PER_DOC):
        worst = 0.0
        for r in range(cp):
            x = rank_latency(doc_len, cp, r, mode, hq, head_dim, tile_q, tile_k, q_grid, kv_grid, tflops)
            if x > worst:
                worst = x
        lat[mode] = worst
    mode = PER_DOC if lat[PER_DOC] < lat[PER_SEQ] else PER_SEQ
    return mode, lat[PER_SEQ], lat[PER_DOC]
