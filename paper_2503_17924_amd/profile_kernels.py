"""Offline profiling for the adaptive sharding selection (paper Section 5.3): measures the
executed TFLOP/s of this library's attention forward+backward kernels on a grid of segment
shapes (Q_len, KV_len) and writes the table wlb_select_sharding reads.

A grid cell is measured on a synthetic rank whose local rows are N copies of one segment: N
documents of KV_len tokens, the rank holding the last Q_len rows of each (every row is real,
the rows of a segment see KV_len - Q_len + 1 .. KV_len keys).  N is chosen to fill the GPU.
The rate is counted on the padded pairs of the estimate (row tiles of 128, key tiles of 64).

Usage (on the GPU):  python -m paper_2503_17924_amd.profile_kernels [--out FILE]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_OUT = os.path.join(HERE, "kernel_profile_mi355x.json")
Q_GRID = [16, 64, 128, 256, 1024, 4096, 16384]
KV_GRID = [128, 1024, 8192, 32768, 131072]
TILE_Q, TILE_K = 128, 64


def padded_pairs(q_len: int, kv_len: int) -> int:
    total = 0
    for t in range(-(-q_len // TILE_Q)):
        e = min((t + 1) * TILE_Q, q_len)
        vis = kv_len - q_len + e
        if vis > 0:
            total += TILE_Q * (-(-vis // TILE_K) * TILE_K)
    return total


def time_rank(torch, B, q_idx, cu_k, total_tokens, hq, hkv, d, reps=3, seed=0):
    """Median milliseconds of (tile schedule + forward + backward) for one rank's rows."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    mk = lambda n, h: torch.randn((n, h, d), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    n_q = len(q_idx)
    q, do = mk(n_q, hq), mk(n_q, hq)
    k, v = mk(total_tokens, hkv), mk(total_tokens, hkv)
    attn = B.Attention(q_idx, cu_k, total_tokens, hq, hkv, d, 1.0 / float(np.sqrt(d)))
    o, lse = attn.forward(q, k, v)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    attn.backward(q, k, v, o, lse, do, dq, dk, dv)
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        attn.plan()
        attn.forward(q, k, v, o, lse)
        attn.backward(q, k, v, o, lse, do, dq, dk, dv)
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    return float(np.median(ts))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=DEFAULT_OUT)
    ap.add_argument("--hq", type=int, default=8)
    ap.add_argument("--hkv", type=int, default=1)
    ap.add_argument("--head-dim", type=int, default=128)
    args = ap.parse_args()
    import torch
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2503_17924_amd import binding as B
    B.lib()
    hq, hkv, d = args.hq, args.hkv, args.head_dim
    table = np.zeros((len(Q_GRID), len(KV_GRID)))
    for i, ql in enumerate(Q_GRID):
        for j, kv in enumerate(KV_GRID):
            if kv < ql:
                continue
            pp = padded_pairs(ql, kv)
            # enough segments for ~2e10 padded pairs per head, at least 1024 row tiles over all heads,
            # within 8M tokens of K/V
            n = max(1, min(int(2e10 // pp) + 1, (8 << 20) // kv))
            n = max(n, min(-(-1024 // (hq * -(-ql // TILE_Q))), (8 << 20) // kv))
            n = max(1, min(n, (1 << 20) // ql))             # Q / dO stay below the library's 4 GiB tensor limit
            cu_k = (np.arange(n + 1, dtype=np.int64) * kv).astype(np.int32)
            q_idx = (cu_k[1:, None] - ql + np.arange(ql, dtype=np.int32)[None, :]).reshape(-1).astype(np.int32)
            ms = time_rank(torch, B, q_idx, cu_k, n * kv, hq, hkv, d)
            table[i, j] = n * pp * 14.0 * d * hq / (ms * 1e-3) / 1e12
            print(f"Q_len {ql:6d} KV_len {kv:7d}  segments {n:6d}  {ms:8.3f} ms  {table[i, j]:8.1f} executed TFLOP/s", flush=True)
    # cells with KV_len < Q_len cannot occur (a row sees at least its own position): copy the nearest measured cell
    for i in range(len(Q_GRID)):
        for j in range(len(KV_GRID)):
            if table[i, j] == 0.0:
                jj = min(k for k in range(len(KV_GRID)) if table[i, k] > 0.0)
                table[i, j] = table[i, jj]
    out = {"device": torch.cuda.get_device_name(0), "hq": hq, "hkv": hkv, "head_dim": d, "tile_q": TILE_Q, "tile_k": TILE_K,
           "what": "executed (tile-padded) attention forward+backward TFLOP/s incl. tile schedule, per segment shape",
           "q_len": Q_GRID, "kv_len": KV_GRID, "tflops": [[round(float(x), 2) for x in row] for row in table]}
    with open(args.out, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", args.out)


def load(path: str = DEFAULT_OUT):
    """-> binding.KernelProfile from a table written by this script."""
    from paper_2503_17924_amd import binding as B
    with open(path) as f:
        t = json.load(f)
    return B.KernelProfile(t["q_len"], t["kv_len"], t["tflops"], t["tile_q"], t["tile_k"])


if __name__ == "__main__":
    main()
