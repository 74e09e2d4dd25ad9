#!/usr/bin/env python3
"""Benchmark of the WLB-LLM hot path on one MI355X.

One step = one pass of the whole path over the 128K-context workload: the streaming packer on one
global batch of the document pool (host), then for each of the 8 emulated context-parallel ranks
the sharding map (host), the tile schedule, attention forward and attention backward (device).
Inputs (the packed sequence's K/V and every rank's Q / dO rows) are resident in HBM before timing
starts.

Prints ONE JSON line: useful attention TFLOP/s forward+backward (only in-document causal
query-key pairs are counted: 4*D flops forward and 10*D backward per pair and query head), the
roofline record of the dominant kernel, per-rank latency max/mean under per-document and
per-sequence sharding, the CPU oracle timed on a bounded sample of the same workload, and -- under
"other_workloads" -- the remaining measurements of the path: the other configurations' rates, the
small-document regime as HBM GB/s with its own roofline record, and the measured micro-batch
latency imbalance of fixed against workload-balanced packing.

During warm-up the share weights of the gang schedule are calibrated to the speeds of this GPU's XCDs
(binding.calibrate_gang_weights; --no-gang-calibration keeps the defaults).  With WLB_TRACE=1 in the
environment every rank's schedule (work-item costs, shares, splits) is described on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, published
COST_A, COST_B = 6, 640000    # packer cost model, picoseconds per token^2 / per token
WINDOW = 131072               # context window of the packing workload
# HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size), measured with
# rocprofv3 --pmc on this workload: profiles/hbm_traffic_c2_128k_cp8.txt
MEASURED_TRAFFIC_BYTES = {("c2_128k_cp8", "dkv_kernel"): int((4.214 + 0.246) * 2**30),
                          ("c2_128k_cp8", "dq_kernel"): int((3.010 + 0.077) * 2**30),
                          ("c2_128k_cp8", "fwd_kernel"): int((2.982 + 0.078) * 2**30)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload index (2 = the 128K CP=8 config)")
    ap.add_argument("--head-dim", type=int, default=0, choices=(0, 64, 128),
                    help="run the workload's documents and head counts at another head dimension (profiling the D=64 kernels)")
    ap.add_argument("--no-gang-calibration", action="store_true",
                    help="keep the default share weights of the gang schedule instead of measuring this GPU's XCDs "
                         "during warm-up (binding.calibrate_gang_weights: three rounds of two untimed steps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-seq", action="store_true", help="skip the per-sequence sharding comparison")
    ap.add_argument("--no-others", action="store_true", help="skip the other workloads (profiling runs)")
    ap.add_argument("--tiny-tail", action="store_true",
                    help="measure only the small-document (HBM-bound) regime: the 1..64-token documents of "
                         "config 4 as their own 32768-token sequence, CP=1 and CP=4, reported as GB/s")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def device_tensors(torch, seed, t, hq, hkv, d, device):
    """Q, K, V, dO of a packed sequence drawn on the GPU: i.i.d. N(0,1) rounded to bf16."""
    g = torch.Generator(device=device).manual_seed(seed)
    out = {}
    for name, h in (("q", hq), ("k", hkv), ("v", hkv), ("do", hq)):
        x = torch.empty((t, h, d), dtype=torch.bfloat16, device=device)
        for r0 in range(0, t, 32768):               # in pieces: no multi-GiB fp32 temporary
            n = min(32768, t - r0)
            x[r0:r0 + n] = torch.randn((n, h, d), device=device, generator=g, dtype=torch.float32).to(torch.bfloat16)
        out[name] = x
    return out


class RankState:
    """Everything one emulated CP rank keeps on the GPU."""

    def __init__(self, B, torch, doc_len, total_tokens, hq, hkv, d, scale, cp, full, rank, mode, device):
        self.rank, self.mode = rank, mode
        sh = B.wlb_shard(doc_len, cp, rank, mode)
        self.pairs = sh["useful_pairs"]
        qi = sh["q_idx"]
        self.n_q = len(qi)
        self.n_real = int((qi >= 0).sum())
        self.q_idx_host = torch.from_numpy(qi.copy()).pin_memory()
        self.attn = B.Attention(qi, sh["cu_seqlens_k"], total_tokens, hq, hkv, d, scale, device, visible_pairs=self.pairs)
        if cp == 1:
            self.q, self.do = full["q"], full["do"]
        else:
            rows = torch.from_numpy(np.maximum(qi, 0).astype(np.int64)).to(device)
            self.q = full["q"].index_select(0, rows).contiguous()
            self.do = full["do"].index_select(0, rows).contiguous()
        self.o = torch.empty_like(self.q)
        self.lse = torch.empty((hq, self.n_q), dtype=torch.float32, device=device)
        self.dq = torch.empty_like(self.q)
        self.dk = torch.empty_like(full["k"])
        self.dv = torch.empty_like(full["v"])

    def run(self, full, backward=True):
        self.attn.plan()
        self.attn.forward(self.q, full["k"], full["v"], self.o, self.lse)
        if backward:
            self.attn.backward(self.q, full["k"], full["v"], self.o, self.lse, self.do, self.dq, self.dk, self.dv)


def timed_ms(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def small_document_regime(B, torch, wl, steps, warmup, device):
    """HBM GB/s of schedule + forward + backward on the 1..64-token documents of config 4 as their own
    sequence, against the algorithmic byte count: Q, O, dO, dQ, LSE, delta per local row; K, V read by
    forward and backward and dK, dV written for every token, per rank."""
    w = wl.config(4)
    docs = w.doc_len[1:]                              # the 1..64-token documents that follow the long one
    T = int(docs.sum())
    hq, hkv, D = w.hq, w.hkv, w.head_dim
    full = device_tensors(torch, 1004, T, hq, hkv, D, device)
    out = {}
    for cp in (1, 4):
        states = [RankState(B, torch, docs, T, hq, hkv, D, w.scale, cp, full, r, B.SHARD_PER_DOC_PADDED, device)
                  for r in range(cp)]
        per_row = 2 * hq * D * 2 + 4 * hq                     # forward: Q, O, LSE
        per_row += 4 * hq * D * 2 + 4 * hq + 2 * 4 * hq       # backward: Q, O, dO read, dQ written, LSE read, delta written and read
        per_tok = 3 * 2 * hkv * D * 2                         # K, V read twice; dK, dV written
        nbytes = float(sum(st.n_real * per_row + T * per_tok for st in states))

        def run():
            for st in states:
                st.run(full)
        ms = timed_ms(torch, run, max(steps, 5), max(warmup, 2))
        out[f"cp{cp}"] = {"ms": round(ms, 4), "algorithmic_bytes": int(nbytes), "gb_per_s": round(nbytes / (ms * 1e-3) / 1e9, 1)}
    best = out["cp1"]
    return {"workload": "c4_tiny_document_tail", "tokens": T, "n_docs": int(len(docs)), "hq": hq, "hkv": hkv, "head_dim": D,
            "value": best["gb_per_s"], "unit": "GB/s", "ms_per_step": best["ms"],
            "roofline": {"bound": "hbm", "achieved": best["gb_per_s"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(best["gb_per_s"] / PEAK_HBM_GBS, 4), "traffic": None},
            "by_cp": out}


def other_config(B, torch, wl, idx, cp, steps, warmup, device):
    """Useful TFLOP/s of another configuration: every rank of `cp` in turn, schedule + forward + backward."""
    w = wl.config(idx)
    full = device_tensors(torch, 1000 + idx, w.total_tokens, w.hq, w.hkv, w.head_dim, device)
    states = [RankState(B, torch, w.doc_len, w.total_tokens, w.hq, w.hkv, w.head_dim, w.scale, cp, full, r,
                        B.SHARD_PER_DOC_PADDED, device) for r in range(cp)]

    def run():
        for st in states:
            st.run(full, w.backward)
    ms = timed_ms(torch, run, steps, warmup)
    pairs = sum(st.pairs for st in states)
    flops = (4.0 + (10.0 if w.backward else 0.0)) * w.head_dim * w.hq * pairs
    val = flops / (ms * 1e-3) / 1e12
    return {"workload": w.name, "cp_ranks_emulated": cp, "hq": w.hq, "hkv": w.hkv, "head_dim": w.head_dim,
            "tokens": w.total_tokens, "useful_pairs": int(pairs), "ms_per_step": round(ms, 3),
            "useful_tflops": round(val, 1), "pct_of_bf16_peak": round(100.0 * val / PEAK_BF16_TFLOPS, 2)}


def arrival_windows(doc_len, window):
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
    return seqs


def packing_latency(B, torch, wl, device, iterations=(2, 3)):
    """Config 3: the pool streamed in global batches of 8 windows.  Micro-batches are built as they arrive
    (fixed length) and by the streaming packer (variable length, L_max = 1.5 windows, two waiting queues);
    every micro-batch of the measured global batches runs schedule + forward + backward at CP = 1.
    Reported: max/mean over a global batch's micro-batches of the measured latency, averaged over the batches."""
    from paper_2503_17924_amd import profile_kernels as PK
    w = wl.config(3)
    n_mb = w.extra["n_microbatch"]
    seqs = arrival_windows(w.doc_len, WINDOW)
    batches = [sum(seqs[i:i + n_mb], []) for i in range(0, len(seqs) - n_mb + 1, n_mb)]
    packer = B.Packer(n_mb, WINDOW * 3 // 2, COST_A, COST_B, [WINDOW // 2, WINDOW * 3 // 4])
    next_id, step_us = 0, []
    cache = {}

    def attention_ms(docs):
        key = tuple(docs)
        if key not in cache:
            cu = np.concatenate([[0], np.cumsum(docs)]).astype(np.int32)
            t = int(cu[-1])
            cache[key] = PK.time_rank(torch, B, np.arange(t, dtype=np.int32), cu, t, w.hq, w.hkv, w.head_dim, reps=2)
        return cache[key]

    imb = lambda xs: max(xs) / (sum(xs) / len(xs))
    rows = {"fixed": [], "wlb": []}
    for it in range(max(iterations) + 1):
        cur = batches[it]
        ids = np.arange(next_id, next_id + len(cur))
        next_id += len(cur)
        t = time.perf_counter()
        _, lens, mb, _, _ = packer.step(ids, cur)
        step_us.append((time.perf_counter() - t) * 1e6)
        if it not in iterations:
            continue
        wlb = [[int(x) for x in lens[mb == j]] for j in range(n_mb)]
        fixed = [seqs[it * n_mb + j] for j in range(n_mb)]
        for name, mbs in (("fixed", fixed), ("wlb", wlb)):
            att = [attention_ms(m) if len(m) else 0.0 for m in mbs]
            step = [a + COST_B * sum(m) * 1e-9 for a, m in zip(att, mbs)]
            rows[name].append((imb(att), imb(step), max(att)))
    mean = lambda name, i: round(float(np.mean([r[i] for r in rows[name]])), 4)
    return {"workload": w.name, "global_batches_measured": list(iterations), "micro_batches": n_mb,
            "packer": "wlb_packer_step, L_max = 1.5 windows, queues at 64K and 96K tokens",
            "packer_step_us_per_global_batch": round(float(np.mean(step_us)), 1),
            "attention_latency_max_over_mean": {"fixed": mean("fixed", 0), "wlb": mean("wlb", 0)},
            "with_modelled_linear_part_max_over_mean": {"fixed": mean("fixed", 1), "wlb": mean("wlb", 1)},
            "slowest_micro_batch_attention_ms": {"fixed": mean("fixed", 2), "wlb": mean("wlb", 2)}}


def blas_threads():
    try:
        import threadpoolctl
        return int(max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1))
    except Exception:
        return None


def cpu_baseline(wl, w, tens, qi, D, hq):
    """The oracle as it stands, on the host cores: a bounded sample of the main workload (every 16th real
    query row of rank 0, forward + backward) gives `value`; configuration 0 is run in full beside it."""
    from oracle import attention as oat
    from oracle import shard as osh
    real = np.nonzero(qi >= 0)[0]
    stride = 16
    sample = real[::stride]
    f = {n: wl.bf16_bits_to_f64(tens[n]) for n in ("k", "v")}
    qs = wl.bf16_bits_to_f64(tens["q"][qi[sample]])
    dos = wl.bf16_bits_to_f64(tens["do"][qi[sample]])
    cu = np.concatenate([[0], np.cumsum(w.doc_len)]).astype(np.int64)
    spairs = oat.useful_pairs(qi[sample], cu)
    t0 = time.perf_counter()
    oat.attn_fwd(qs, f["k"], f["v"], qi[sample], cu, w.scale)
    if w.backward:
        oat.attn_bwd(qs, f["k"], f["v"], dos, qi[sample], cu, w.scale)
    cpu_s = time.perf_counter() - t0
    cpu_flops = (4.0 + (10.0 if w.backward else 0.0)) * D * hq * spairs
    threads = blas_threads()
    # configuration 0 in full: both ranks' sharding maps and forward (that configuration has no backward)
    w0 = wl.config(0)
    t0_tens = w0.tensors(names=("q", "k", "v"))
    f0 = {n: wl.bf16_bits_to_f64(t0_tens[n]) for n in ("q", "k", "v")}
    t0 = time.perf_counter()
    pairs0 = 0
    for r in range(w0.cp):
        sh = osh.shard(w0.doc_len, w0.cp, r, osh.PER_DOC_PADDED)
        rows = np.maximum(sh["q_idx"], 0)
        oat.attn_fwd(f0["q"][rows], f0["k"], f0["v"], sh["q_idx"], sh["cu_seqlens_k"], w0.scale)
        pairs0 += sh["useful_pairs"]
    c0_s = time.perf_counter() - t0
    return {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "useful TFLOP/s", "cores": int(threads or os.cpu_count()),
            "kind": "oracle", "seconds": round(cpu_s, 2), "os_cpu_count": os.cpu_count(), "blas_threads": threads,
            "sample": f"rank 0, every {stride}th real query row ({len(sample)} rows, {spairs} pairs), all heads, fwd+bwd",
            "full_config_0": {"workload": w0.name, "what": "sharding maps + forward of both ranks, whole configuration",
                              "seconds": round(c0_s, 3), "useful_pairs": int(pairs0),
                              "useful_tflops": round(4.0 * w0.head_dim * w0.hq * pairs0 / c0_s / 1e12, 6)}}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU (context-parallel ranks are emulated in turn); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_17924_amd import binding as B
    from paper_2503_17924_amd import workloads as wl

    B.lib()                       # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    device = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=device)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.tiny_tail:
        r = small_document_regime(B, torch, wl, args.steps, args.warmup, device)
        print(json.dumps({"metric": "HBM GB/s, small-document regime (schedule + attention fwd + bwd)", "value": r["value"],
                          "unit": "GB/s", "n_gpus": 1, "steps": max(args.steps, 5), "warmup": max(args.warmup, 2),
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                          "dtype": "bf16", "data": "synthetic",
                          "config": {k: r[k] for k in ("workload", "tokens", "n_docs", "hq", "hkv", "head_dim")},
                          "roofline": r["roofline"], "by_cp": r["by_cp"]}))
        return
    w = wl.config(args.config)
    if args.head_dim and args.head_dim != w.head_dim:
        w.head_dim, w.scale, w.name = args.head_dim, 1.0 / float(np.sqrt(args.head_dim)), f"{w.name}_d{args.head_dim}"
    if args.config == 3:
        raise SystemExit("config 3 (packing pool) is measured inside the default run; bench configs: 1, 2, 4, 5")
    D, hq = w.head_dim, w.hq

    t0 = time.time()
    tens = w.tensors()
    full = {n: B.bf16_bits_to_tensor(a, device) for n, a in tens.items()}
    modes = [B.SHARD_PER_DOC_PADDED] + ([] if (args.no_per_seq or w.cp == 1) else [B.SHARD_PER_SEQ])
    ranks = {m: [RankState(B, torch, w.doc_len, w.total_tokens, hq, w.hkv, D, w.scale, w.cp, full, r, m, device)
                 for r in range(w.cp)] for m in modes}
    # the packer's input: the document pool of config 3 streamed in global batches of 8 windows
    pool = wl.config(3)
    seqs = arrival_windows(pool.doc_len, WINDOW)
    n_mb = pool.extra["n_microbatch"]
    batches = [np.asarray(sum(seqs[i:i + n_mb], []), dtype=np.int32) for i in range(0, len(seqs) - n_mb + 1, n_mb)]
    packer = B.Packer(n_mb, WINDOW * 3 // 2, COST_A, COST_B, [WINDOW // 2, WINDOW * 3 // 4])
    pack_state = {"it": 0, "next_id": 0}
    setup_s = time.time() - t0

    host_us = {"pack": 0.0, "shard": 0.0}

    def step(states, record=None):
        t = time.perf_counter()
        cur = batches[pack_state["it"] % len(batches)]
        ids = np.arange(pack_state["next_id"], pack_state["next_id"] + len(cur))
        pack_state["it"] += 1
        pack_state["next_id"] += len(cur)
        packer.step(ids, cur)
        host_us["pack"] += (time.perf_counter() - t) * 1e6
        for st in states:
            t = time.perf_counter()
            sh = B.wlb_shard(w.doc_len, w.cp, st.rank, st.mode)
            host_us["shard"] += (time.perf_counter() - t) * 1e6
            st.q_idx_host.copy_(torch.from_numpy(sh["q_idx"]))
            st.attn.q_idx.copy_(st.q_idx_host, non_blocking=True)
            if record is not None:
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record()
            st.attn.plan()
            st.attn.forward(st.q, full["k"], full["v"], st.o, st.lse)
            if record is not None:
                e1.record()
            if w.backward:
                st.attn.backward(st.q, full["k"], full["v"], st.o, st.lse, st.do, st.dq, st.dk, st.dv)
            if record is not None:
                e2.record()
                record.append((e0, e1, e2))


    main_states = ranks[B.SHARD_PER_DOC_PADDED]
    if os.environ.get("WLB_TRACE") == "1":
        # the schedule of every rank (work-item costs, shares, splits) on stderr, for looking at it by eye
        for st in main_states:
            st.attn.plan()
            print(B.plan_report(st.attn, f"{w.name} rank {st.rank}"), file=sys.stderr)
    # Part of the warm-up: the XCDs of one GPU run the forward and dQ kernels at speeds that differ by several
    # percent, and the gang schedule can weight each XCD's share; the factors are measured on this workload's
    # own launches (the gangs' recorded clocks) and then stay fixed for the process.
    gang_factors = None
    if not args.no_gang_calibration:
        gang_factors = B.calibrate_gang_weights([st.attn for st in main_states], lambda: step(main_states))
    for _ in range(args.warmup):
        step(main_states)
    torch.cuda.synchronize()
    host_us = {"pack": 0.0, "shard": 0.0}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(main_states)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    host_us_timed = dict(host_us)          # later step() calls (per-rank latencies) keep adding to host_us

    pairs = sum(st.pairs for st in main_states)
    flops_fwd = 4.0 * D * hq * pairs
    flops_bwd = 10.0 * D * hq * pairs if w.backward else 0.0
    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12

    # ---- per-rank latency (events on the stream the library launches on), both shardings
    def rank_latency(states, reps=3):
        lat = np.zeros((reps, len(states), 2))
        for i in range(reps):
            rec = []
            step(states, rec)
            torch.cuda.synchronize()
            for j, (e0, e1, e2) in enumerate(rec):
                lat[i, j] = (e0.elapsed_time(e1), e1.elapsed_time(e2))
        return np.median(lat, axis=0)

    per_rank = {}
    for m in modes:
        lat = rank_latency(ranks[m])
        tot = lat.sum(axis=1)
        per_rank["per_document" if m == B.SHARD_PER_DOC_PADDED else "per_sequence"] = {
            "max_over_mean": float(tot.max() / tot.mean()), "fwd_ms": [round(x, 3) for x in lat[:, 0]],
            "bwd_ms": [round(x, 3) for x in lat[:, 1]],
            "pairs_max_over_mean": float(max(s.pairs for s in ranks[m]) / np.mean([s.pairs for s in ranks[m]]))}

    # ---- how evenly the gangs of the forward and dQ kernels finish (their workgroups leave start / end readings
    # of the 100 MHz real-time counter in the workspace): spread of the gangs' end times relative to the kernel's
    # duration, and mean end time of the first and the second half of the gangs (they get different shares)
    gang_balance = None
    lay0 = B.wlb_attn_plan_layout(main_states[0].attn.desc)
    if lay0.uses_gangs:
        G = hq // w.hkv
        acc = {"fwd": [], "dq": []}
        for st in main_states:
            clk = B.gang_clocks(st.attn).astype(np.int64)
            for k, name in enumerate(("fwd", "dq")):
                t0 = clk[k, :, 0].min()
                end = clk[k, :, 1] - t0
                b = np.arange(len(end))
                gang = ((b // 8) // G) * 8 + b % 8
                gend = np.array([end[gang == g].max() for g in range(lay0.row_gangs)], dtype=np.float64)
                half = lay0.row_gangs // 2
                acc[name].append(((gend.max() - gend.min()) / gend.max(), gend[:half].mean() / gend.max(), gend[half:].mean() / gend.max()))
        gang_balance = {name: {"end_time_spread_over_duration": round(float(np.mean([a[0] for a in v])), 4),
                               "worst_rank_spread": round(float(np.max([a[0] for a in v])), 4),
                               "mean_end_first_half_of_gangs": round(float(np.mean([a[1] for a in v])), 4),
                               "mean_end_second_half_of_gangs": round(float(np.mean([a[2] for a in v])), 4)}
                        for name, v in acc.items()}

    # ---- per-kernel timing on every rank: each kernel launched alone (the library's measurement flags),
    # timed with HIP events on the stream the library launches on (torch's current stream)
    def time_call(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.mean(ts))

    kern = {}

    def add(name, ms):
        kern.setdefault(name, []).append(ms)

    for st in main_states:
        add("plan_ms", time_call(lambda: st.attn.plan()))
        add("fwd_ms", time_call(lambda: st.attn.forward(st.q, full["k"], full["v"], st.o, st.lse)))
        if w.backward:
            bw = lambda fl: st.attn.backward(st.q, full["k"], full["v"], st.o, st.lse, st.do, st.dq, st.dk, st.dv,
                                             extra_flags=fl)
            add("delta_ms", time_call(lambda: bw(B.ATTN_BWD_SKIP_DQ | B.ATTN_BWD_SKIP_DKV)))
            add("dq_ms", time_call(lambda: bw(B.ATTN_BWD_SKIP_DELTA | B.ATTN_BWD_SKIP_DKV)))
            add("dkv_ms", time_call(lambda: bw(B.ATTN_BWD_SKIP_DELTA | B.ATTN_BWD_SKIP_DQ)))
    kern = {k: float(np.mean(v)) for k, v in kern.items()}
    # algorithmic flops per launch (mean over ranks): forward 4*D per pair and head; the dK/dV
    # kernel carries the score and dP recomputation plus dK and dV (8*D); the dQ kernel adds dQ (2*D)
    p0 = float(np.mean([st.pairs for st in main_states]))
    alg = {"fwd": 4.0 * D * hq * p0, "dkv": 8.0 * D * hq * p0, "dq": 2.0 * D * hq * p0}
    tfl = {k: alg[k] / (kern[k + "_ms"] * 1e-3) / 1e12 for k in alg if k + "_ms" in kern}
    dominant = max((k for k in tfl), key=lambda k: kern[k + "_ms"])
    traffic = MEASURED_TRAFFIC_BYTES.get((w.name, dominant + "_kernel"))
    # the dense bf16 MFMA rate this GPU sustains (a kernel of nothing but MFMAs on register operands):
    # lower for random operand values -- what attention sees -- than for all-ones
    ceiling = {"all_ones": round(B.mfma_ceiling(False), 1), "random": round(B.mfma_ceiling(True), 1)}
    # fp32 atomic-add rate (what a one-kernel backward would need for dQ): context for the 14*D executed flops
    atomics = {"private_tiles_tb_per_s": round(B.atomic_add_rate(False), 3), "shared_tiles_tb_per_s": round(B.atomic_add_rate(True), 3)}
    roofline = {"bound": "mfma", "kernel": dominant + "_kernel", "achieved": round(tfl[dominant], 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tfl[dominant] / PEAK_BF16_TFLOPS, 4),
                "measured_mfma_ceiling_tflops": ceiling,
                "frac_of_measured_ceiling_random_operands": round(tfl[dominant] / ceiling["random"], 4),
                "traffic": traffic, "launch_ms": round(kern[dominant + "_ms"], 4),
                "launch_ms_includes": {"dkv": "dkv_fixup_kernel (about 1 %)", "dq": "dq_merge_kernel (under 1 %)",
                                       "fwd": "fwd_merge_kernel (under 2 %)"}[dominant],
                "algorithmic_flops_per_launch": alg[dominant],
                "per_kernel_tflops": {k: round(v, 2) for k, v in tfl.items()},
                "per_kernel_ms_mean_over_ranks": {k: round(v, 4) for k, v in kern.items()}}

    # ---- the rest of the path's measurements, each a short run of its own
    others = None
    if not args.no_others and args.config == 2 and not args.head_dim:
        others = {"small_document_regime": small_document_regime(B, torch, wl, 10, 3, device),
                  "c1_32k_gqa_cp1": other_config(B, torch, wl, 1, 1, 10, 3, device),
                  "c4_straggler_cp1": other_config(B, torch, wl, 4, 1, 3, 1, device),
                  "c4_straggler_cp4": other_config(B, torch, wl, 4, 4, 3, 1, device),
                  "c5_64k_mha_cp2": other_config(B, torch, wl, 5, 2, 10, 3, device),
                  "c3_packing": packing_latency(B, torch, wl, device)}
    q_idx_rank0 = main_states[0].attn.q_idx.cpu().numpy()

    # ---- CPU oracle on a bounded sample of the same workload, and on configuration 0 in full
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, w, tens, q_idx_rank0, D, hq)

    out = {
        "metric": "useful attn TFLOP/s fwd+bwd (% bf16 MFMA peak); per-CP-rank latency max/mean",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "tokens": w.total_tokens, "cp_ranks_emulated": w.cp, "hq": hq, "hkv": w.hkv,
                   "head_dim": D, "n_docs": int(len(w.doc_len)), "longest_doc": int(w.doc_len.max()),
                   "sharding": "per_document_padded", "useful_pairs": int(pairs)},
        "pct_of_bf16_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "pct_of_measured_mfma_ceiling_random_operands": round(100.0 * value / ceiling["random"], 2),
        "per_rank_latency": per_rank, "gang_balance": gang_balance,
        "gang_xcd_speed_factors_measured_in_warmup": gang_factors, "atomic_add_rate": atomics,
        "host_us_per_step": {"pack": round(host_us_timed["pack"] / args.steps, 1),
                             "pack_what": "wlb_packer_step on one global batch (8 windows of 131072 tokens) of the config-3 pool",
                             "shard": round(host_us_timed["shard"] / args.steps, 1)},
        "roofline": roofline, "cpu_baseline": cpu, "other_workloads": others, "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
