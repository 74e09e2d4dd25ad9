"""Predicted versus measured attention latency under per-sequence and per-document sharding, and
the choice wlb_select_sharding makes, on a set of synthetic 128K micro-batches (an analogue of the
paper's CP sharding case study, Section 6.4, with this library's kernels and profile table).

A sharding's measured latency is the maximum over the emulated CP ranks of (tile schedule +
forward + backward) for that rank's rows.  "optimal" is the faster of the two measured.

Usage (on the GPU):  python -m paper_2503_17924_amd.adaptive_report [--cp 8]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
T = 131072


def micro_batches(cp: int):
    rng = np.random.default_rng(11)
    def fill(lengths):
        lengths = [int(x) for x in lengths]
        out, s = [], 0
        for x in lengths:
            if s + x > T:
                break
            out.append(x); s += x
        if s < T:
            out.append(T - s)
        return np.array(out, dtype=np.int32)
    mixture = np.clip(np.rint(rng.lognormal(np.log(1024), 1.0, size=400)), 16, 8192)
    return {
        "one 112K document + short ones": fill([114688] + list(mixture)),
        "one 96K document + 1..64-token ones": fill([98304] + list(rng.integers(1, 65, size=2000))),
        "two 64K documents": fill([65536, 65536]),
        "eight 16K documents": fill([16384] * 8),
        "short documents (log-normal, median 1K)": fill(mixture),
        "2048 documents of 64 tokens": fill([64] * 2048),
        "512 documents of 256 tokens": fill([256] * 512),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cp", type=int, default=8)
    ap.add_argument("--profile", default=None)
    args = ap.parse_args()
    import torch
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2503_17924_amd import binding as B
    from paper_2503_17924_amd import profile_kernels as PK
    prof = PK.load(args.profile or PK.DEFAULT_OUT)
    cp, hq, hkv, d = args.cp, 8, 1, 128
    print(f"T={T} CP={cp} hq={hq} hkv={hkv} head_dim={d}; latencies in ms (max over ranks, schedule+fwd+bwd)")
    print(f"{'micro-batch':42s} {'pred seq':>9s} {'pred doc':>9s} {'meas seq':>9s} {'meas doc':>9s}  {'choice':>7s} {'optimal':>7s}  chosen/optimal")
    tot = {"seq": 0.0, "doc": 0.0, "chosen": 0.0, "optimal": 0.0}
    for name, doc_len in micro_batches(cp).items():
        mode, p_seq, p_doc = B.wlb_select_sharding(doc_len, cp, hq, d, prof)
        meas = {}
        for m in (B.SHARD_PER_SEQ, B.SHARD_PER_DOC_PADDED):
            worst = 0.0
            for r in range(cp):
                sh = B.wlb_shard(doc_len, cp, r, m)
                worst = max(worst, PK.time_rank(torch, B, sh["q_idx"], sh["cu_seqlens_k"], T, hq, hkv, d, reps=3, seed=r))
            meas[m] = worst
        best = min(meas, key=meas.get)
        nm = {B.SHARD_PER_SEQ: "per-seq", B.SHARD_PER_DOC_PADDED: "per-doc"}
        print(f"{name:42s} {p_seq*1e3:9.3f} {p_doc*1e3:9.3f} {meas[B.SHARD_PER_SEQ]:9.3f} {meas[B.SHARD_PER_DOC_PADDED]:9.3f}  "
              f"{nm[mode]:>7s} {nm[best]:>7s}  {meas[mode] / meas[best]:.3f}", flush=True)
        tot["seq"] += meas[B.SHARD_PER_SEQ]; tot["doc"] += meas[B.SHARD_PER_DOC_PADDED]
        tot["chosen"] += meas[mode]; tot["optimal"] += meas[best]
    print(f"sum over micro-batches: always per-seq {tot['seq']:.2f} ms, always per-doc {tot['doc']:.2f} ms, "
          f"adaptive {tot['chosen']:.2f} ms, optimal {tot['optimal']:.2f} ms")


if __name__ == "__main__":
    main()
