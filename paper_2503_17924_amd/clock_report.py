"""Shader clock the GPU sustains while each attention kernel runs back to back, next to a pure MFMA stream.

The published dense bf16 MFMA peak (2.5 PFLOP/s) is the product of the unit count and the maximum
clock (2.4 GHz).  Under a sustained matrix load the GPU lowers its clock to stay inside its power
limit, by an amount that depends on what the kernel does besides MFMAs and on the operand bits.  This
report launches one kernel of the 128K-token configuration (rank 0 of the CP=8 per-document sharding)
over and over for a few seconds, reads the current shader clock from `rocm-smi --showclocks`
meanwhile, and prints per kernel: time per launch, sustained clock, executed TFLOP/s, and that rate
as a fraction of the MFMA peak at the sustained clock (unit count x that clock).

A second table puts the same kernels on a uniform problem -- 16384 rows that all see one document of 32768 keys,
no masking and no scheduling loss -- and gives the time per MFMA and SIMD (nanoseconds between two 32x32x16
MFMAs of one SIMD, 13.1 at the published peak) next to the value on the real workload: the distance between
the two is what masks, ragged tiles and the work schedule cost, the distance to the pure MFMA stream what
the kernels' own instruction streams cost.

Usage (on the GPU):  python -m paper_2503_17924_amd.clock_report
"""
from __future__ import annotations

import ctypes as C
import os
import re
import subprocess
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
PEAK_TFLOPS, PEAK_MHZ = 2500.0, 2400.0
N_SIMD, MFMA_FLOPS = 1024, 2 * 32 * 32 * 16


def shader_clock_mhz():
    """Current shader clock from rocm-smi, or None when the tool or the line is missing."""
    try:
        out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
    except (OSError, subprocess.TimeoutExpired):
        return None
    m = re.search(r"sclk clock level: \d+: \((\d+)Mhz\)", out)
    return int(m.group(1)) if m else None


def main():
    import torch
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2503_17924_amd import binding as B
    from paper_2503_17924_amd import workloads as wl
    dev = "cuda:0"
    w = wl.config(2)
    hq, hkv, d = w.hq, w.hkv, w.head_dim
    full = {n: B.bf16_bits_to_tensor(a, dev) for n, a in w.tensors().items()}
    sh = B.wlb_shard(w.doc_len, w.cp, 0, B.SHARD_PER_DOC_PADDED)
    qi = sh["q_idx"]
    rows = torch.from_numpy(np.maximum(qi, 0).astype(np.int64)).to(dev)
    q, do = full["q"].index_select(0, rows).contiguous(), full["do"].index_select(0, rows).contiguous()
    attn = B.Attention(qi, sh["cu_seqlens_k"], w.total_tokens, hq, hkv, d, w.scale, dev)
    o, lse = attn.forward(q, full["k"], full["v"])
    dq, dk, dv = attn.backward(q, full["k"], full["v"], o, lse, do)
    torch.cuda.synchronize()
    pairs = float(sh["useful_pairs"])
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    flops = C.c_double(0.0)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def mfma(random_operands):
        B._check(B.lib().wlb_calib_mfma(C.c_int32(random_operands), C.c_int32(4000), C.c_void_p(sink.data_ptr()),
                                        C.byref(flops), stream))
    mfma(1)
    torch.cuda.synchronize()
    # kernel, launch, executed flops per launch (recomputed products included), launches
    phases = [
        ("forward", lambda: attn.forward(q, full["k"], full["v"], o, lse), 4.0 * d * hq * pairs, 1000),
        ("dQ (+ delta pass)", lambda: attn.backward(q, full["k"], full["v"], o, lse, do, dq, dk, dv,
                                                     extra_flags=B.ATTN_BWD_SKIP_DKV), 6.0 * d * hq * pairs, 800),
        ("dK/dV (+ delta pass, fix-up)", lambda: attn.backward(q, full["k"], full["v"], o, lse, do, dq, dk, dv,
                                                                extra_flags=B.ATTN_BWD_SKIP_DQ), 8.0 * d * hq * pairs, 500),
        ("MFMA only, random operands", lambda: mfma(1), flops.value, 600),
        ("MFMA only, all-ones operands", lambda: mfma(0), flops.value, 600),
    ]
    ns_per_mfma = {}
    print(f"workload {w.name} rank 0: n_q {len(qi)}, {int(pairs)} visible pairs, heads {hq}/{hkv}, D {d}; idle clock {shader_clock_mhz()} MHz")
    print(f"{'kernel':30s} {'ms/launch':>10s} {'sclk MHz (4 readings)':>28s} {'executed TFLOP/s':>17s} {'of peak at 2.4 GHz':>19s} {'of peak at sclk':>16s}")
    for name, fn, fl, n in phases:
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        time.sleep(0.5)                       # the queue holds a few seconds of launches: sample while they run
        clk = [shader_clock_mhz() for _ in range(4)]
        busy = not e1.query()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / n
        tf = fl / (ms * 1e-3) / 1e12
        good = [c for c in clk if c]
        at = (f"{tf / (PEAK_TFLOPS * np.mean(good) / PEAK_MHZ):16.3f}" if good and busy else f"{'n/a':>16s}")
        print(f"{name:30s} {ms:10.3f} {str(clk):>28s} {tf:17.1f} {tf / PEAK_TFLOPS:19.3f} {at}")
        ns_per_mfma[name] = ms * 1e6 * N_SIMD / (fl / MFMA_FLOPS)
    print("executed flops: 4*D per visible pair and head forward, 6*D in the dQ kernel and 8*D in the dK/dV kernel (S and dP are")
    print("computed in both); the delta pass and the fix-up are included in the times.  'of peak at sclk' divides by 2.5 PFLOP/s x sclk / 2.4 GHz.")

    # ---- the same kernels on uniform, unmasked work
    del attn, q, do, o, lse, dq, dk, dv
    t_u, nq_u = 32768, 16384
    gen = torch.Generator(device=dev).manual_seed(0)
    mk = lambda n, h: torch.randn((n, h, d), device=dev, generator=gen, dtype=torch.float32).to(torch.bfloat16)
    q, do, k, v = mk(nq_u, hq), mk(nq_u, hq), mk(t_u, hkv), mk(t_u, hkv)
    attn = B.Attention(np.full(nq_u, t_u - 1, dtype=np.int32), np.array([0, t_u], dtype=np.int32), t_u, hq, hkv, d,
                       1.0 / float(np.sqrt(d)), dev)
    o, lse = attn.forward(q, k, v)
    dq, dk, dv = attn.backward(q, k, v, o, lse, do)
    torch.cuda.synchronize()

    def median_ms(fn, reps=7):
        out = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1))
        return float(np.median(out))
    pairs_u = float(nq_u) * t_u
    rows = [("forward", lambda: attn.forward(q, k, v, o, lse), 4.0),
            ("dQ (+ delta pass)", lambda: attn.backward(q, k, v, o, lse, do, dq, dk, dv, extra_flags=B.ATTN_BWD_SKIP_DKV), 6.0),
            ("dK/dV (+ delta pass, fix-up)", lambda: attn.backward(q, k, v, o, lse, do, dq, dk, dv, extra_flags=B.ATTN_BWD_SKIP_DQ), 8.0)]
    print()
    print(f"uniform problem: {nq_u} rows x one document of {t_u} keys, heads {hq}/{hkv}, D {d}; ns per MFMA and SIMD ({MFMA_FLOPS} flops per MFMA, {N_SIMD} SIMDs)")
    print(f"{'kernel':30s} {'ms/launch':>10s} {'executed TFLOP/s':>17s} {'ns per MFMA, uniform':>21s} {'ns per MFMA, ' + w.name:>27s}")
    for name, fn, mult in rows:
        fn()
        torch.cuda.synchronize()
        ms = median_ms(fn)
        fl = mult * d * hq * pairs_u
        print(f"{name:30s} {ms:10.3f} {fl / (ms * 1e-3) / 1e12:17.1f} {ms * 1e6 * N_SIMD / (fl / MFMA_FLOPS):21.1f} {ns_per_mfma[name]:27.1f}")
    for name in ("MFMA only, random operands", "MFMA only, all-ones operands"):
        print(f"{name:30s} {'':10s} {'':17s} {ns_per_mfma[name]:21.1f}")


if __name__ == "__main__":
    main()
