"""Measured attention latency of the micro-batches the packers produce (an analogue of the paper's
packing comparison, Section 6.4 / Table 2, with this library's packer and kernels on a synthetic
long-tailed document pool).

The pool is streamed as Algorithm 1's dataloader (Section 4.3): documents in arrival order fill
windows of the context length, eight windows form one global batch.  Per global batch the
micro-batches are built three ways:
  fixed          each window is one micro-batch, as it arrived (the baseline of Section 3.2)
  greedy         wlb_packer_step with L_max = the window, no waiting queue
  greedy+queues  wlb_packer_step with L_max = 1.5 windows and two waiting queues (Section 4.2)
and every micro-batch runs tile schedule + forward + backward on the GPU (CP = 1).  Reported per
packer, averaged over the global batches: max/mean over the micro-batches of
  model      the packer's cost  a d^2 + b d  summed over the documents (Equation 2, Section 4.1)
  attention  the measured attention latency
  step       measured attention + b * tokens (the linear part is modelled, no such layers run here)
then the slowest micro-batch's latency (what a global batch waits for), also per token of the
global batch since the packers place different token counts per batch (left-over and waiting
documents move between batches), and the documents still held back when the stream ends,
and the a (picoseconds per token^2) that a least-squares fit of the measured latencies gives.

Usage (on the GPU):  python -m paper_2503_17924_amd.packing_report [--iterations 6]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
WINDOW = 131072
COST_A, COST_B = 6, 640000          # picoseconds per token^2 / per token


def arrival_windows(doc_len, window: int):
    """Documents in arrival order cut into sequences of `window` tokens; a document that crosses a
    boundary is split there and its rest starts the next sequence as a new document."""
    seqs, cur, used = [], [], 0
    for d in (int(x) for x in doc_len):
        while d > 0:
            take = min(d, window - used)
            cur.append(take)
            used += take
            d -= take
            if used == window:
                seqs.append(cur)
                cur, used = [], 0
    return seqs          # the unfinished tail is left out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iterations", type=int, default=6, help="global batches to measure")
    ap.add_argument("--reps", type=int, default=2)
    args = ap.parse_args()
    import torch
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2503_17924_amd import binding as B
    from paper_2503_17924_amd import profile_kernels as PK
    from paper_2503_17924_amd import workloads as wl
    w = wl.config(3)
    hq, hkv, d, n_mb = w.hq, w.hkv, w.head_dim, w.extra["n_microbatch"]
    seqs = arrival_windows(w.doc_len, WINDOW)
    batches = [sum(seqs[i:i + n_mb], []) for i in range(0, len(seqs) - n_mb + 1, n_mb)][:args.iterations]
    print(f"pool: {len(w.doc_len)} documents, {int(w.doc_len.sum())} tokens, {len(seqs)} windows of {WINDOW}; "
          f"{len(batches)} global batches of {n_mb} micro-batches measured; {hq}/{hkv} heads, head_dim {d}, CP=1; "
          f"cost model a={COST_A} b={COST_B} ps")

    cache = {}

    def attention_ms(docs):
        """Measured milliseconds of tile schedule + forward + backward for one packed micro-batch."""
        key = tuple(docs)
        if key not in cache:
            cu = np.concatenate([[0], np.cumsum(docs)]).astype(np.int32)
            t = int(cu[-1])
            cache[key] = PK.time_rank(torch, B, np.arange(t, dtype=np.int32), cu, t, hq, hkv, d, reps=args.reps)
        return cache[key]

    def fixed(_state, it, cur):
        return [seqs[it * n_mb + j] for j in range(n_mb)]

    def greedy(state, it, cur):
        ids = np.arange(state["next_id"], state["next_id"] + len(cur))
        state["next_id"] += len(cur)
        _, lens, mb, _, _ = state["packer"].step(ids, cur)
        return [[int(x) for x in lens[mb == j]] for j in range(n_mb)]

    packers = [
        ("fixed (arrival order)", fixed, lambda: {}),
        ("greedy, L_max = window", greedy, lambda: {"packer": B.Packer(n_mb, WINDOW, COST_A, COST_B), "next_id": 0}),
        ("greedy, L_max = 1.5 window, queues 64K/96K", greedy,
         lambda: {"packer": B.Packer(n_mb, WINDOW * 3 // 2, COST_A, COST_B, [WINDOW // 2, WINDOW * 3 // 4]), "next_id": 0}),
    ]
    imb = lambda xs: max(xs) / (sum(xs) / len(xs))
    fit_x, fit_y = [], []
    print(f"{'packer':44s} {'batches':>7s} {'model':>7s} {'attention':>9s} {'step':>7s}   slowest micro-batch (ms): attention / step, mean over batches; slowest step per token of the batch")
    for name, build, make_state in packers:
        state = make_state()
        rows = []
        for it, cur in enumerate(batches):
            mbs = build(state, it, cur)
            if any(len(m) == 0 for m in mbs):
                continue          # the queues are still filling: not every micro-batch has work yet
            model = [sum(COST_A * x * x + COST_B * x for x in m) for m in mbs]
            att = [attention_ms(m) for m in mbs]
            step = [a_ms + COST_B * sum(m) * 1e-9 for a_ms, m in zip(att, mbs)]
            rows.append((imb(model), imb(att), imb(step), max(att), max(step), float(sum(sum(m) for m in mbs))))
            for a_ms, m in zip(att, mbs):
                fit_x.append(float(sum(x * x for x in m)))
                fit_y.append(a_ms)
        r = np.mean(np.array(rows), axis=0)
        waiting = sum(state["packer"].pending()) if "packer" in state else 0
        print(f"{name:44s} {len(rows):7d} {r[0]:7.3f} {r[1]:9.3f} {r[2]:7.3f}   {r[3]:8.2f} / {r[4]:8.2f}   "
              f"{r[4] * 1e6 / r[5]:6.3f} ns per token; {waiting} documents still waiting", flush=True)
    x, y = np.array(fit_x), np.array(fit_y)
    a_fit = float((x * y).sum() / (x * x).sum()) * 1e9          # ms per token^2 -> ps per token^2
    print(f"least-squares fit of measured attention latency to a*sum(d^2): a = {a_fit:.2f} ps per token^2 "
          f"(the packers used a = {COST_A})")


if __name__ == "__main__":
    main()
