"""Shared plumbing of the GPU parity tests: run the HIP path and the oracle on the same
seeded inputs and compare with the acceptance bounds (errors relative to each tensor's
largest magnitude: max <= 2e-2, mean <= 2e-3; LSE absolute <= 1e-2)."""
import numpy as np

from oracle import attention as oat
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl

MAX_REL, MEAN_REL, LSE_ABS = 2e-2, 2e-3, 1e-2
SCALE_FLOOR = 1e-3


def check_close(name, got, ref, rows=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if rows is not None:
        got, ref = got[rows], ref[rows]
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    # Errors are relative to the tensor's largest magnitude.  A tensor that is exactly zero in
    # exact arithmetic (dQ when every document has one token: dS = dP - <dO, O> cancels) leaves
    # only the bf16 rounding of O behind, so the scale is floored at 1e-3 (inputs are N(0,1)).
    scale = max(np.abs(ref).max(), SCALE_FLOOR)
    err = np.abs(got - ref)
    mx, mean = err.max() / scale, err.mean() / scale
    assert mx <= MAX_REL, f"{name}: max err {mx:.3e} > {MAX_REL}"
    assert mean <= MEAN_REL, f"{name}: mean err {mean:.3e} > {MEAN_REL}"
    return mx, mean


def gather_rows(bits, q_idx):
    """Rows of a [T, H, D] bit tensor selected by q_idx; padding slots read row 0."""
    return np.ascontiguousarray(bits[np.maximum(np.asarray(q_idx), 0)])


class Case:
    """One rank's attention problem: bf16 bit tensors on the host, tensors on the GPU."""

    def __init__(self, tens, q_idx, cu_k, hq, hkv, d, scale, device="cuda:0"):
        import torch
        self.torch = torch
        self.q_idx = np.asarray(q_idx, dtype=np.int32)
        self.cu_k = np.asarray(cu_k, dtype=np.int32)
        self.scale = scale
        self.hq, self.hkv, self.d = hq, hkv, d
        self.t_kv = int(self.cu_k[-1])
        self.bits = {"q": gather_rows(tens["q"], self.q_idx), "k": tens["k"], "v": tens["v"]}
        if "do" in tens:
            self.bits["do"] = gather_rows(tens["do"], self.q_idx)
        self.dev = {n: B.bf16_bits_to_tensor(a, device) for n, a in self.bits.items()}
        self.attn = B.Attention(self.q_idx, self.cu_k, self.t_kv, hq, hkv, d, scale, device)
        self.flags = 0          # extra descriptor flags for every call (e.g. a forced work schedule)

    def f64(self, name):
        return wl.bf16_bits_to_f64(self.bits[name])

    def run_fwd(self):
        o, lse = self.attn.forward(self.dev["q"], self.dev["k"], self.dev["v"], extra_flags=self.flags)
        self.torch.cuda.synchronize()
        self.o, self.lse = o, lse
        return B.tensor_to_f64(o), B.tensor_to_f64(lse)

    def run_bwd(self):
        dq, dk, dv = self.attn.backward(self.dev["q"], self.dev["k"], self.dev["v"], self.o, self.lse,
                                        self.dev["do"], extra_flags=self.flags)
        self.torch.cuda.synchronize()
        return B.tensor_to_f64(dq), B.tensor_to_f64(dk), B.tensor_to_f64(dv)

    def oracle_fwd(self):
        return oat.attn_fwd(self.f64("q"), self.f64("k"), self.f64("v"), self.q_idx, self.cu_k, self.scale)

    def oracle_bwd(self):
        return oat.attn_bwd(self.f64("q"), self.f64("k"), self.f64("v"), self.f64("do"), self.q_idx, self.cu_k,
                            self.scale)

    def check_fwd(self, tag=""):
        o, lse = self.run_fwd()
        ro, rlse = self.oracle_fwd()
        real = self.q_idx >= 0
        stats = check_close(f"O{tag}", o, ro, rows=real)
        if (~real).any():
            assert (o[~real] == 0).all(), "padding rows of O must be zero"
            assert np.isneginf(lse[:, ~real]).all(), "padding rows of LSE must be -inf"
        if real.any():
            d = np.abs(lse[:, real] - rlse[:, real]).max()
            assert d <= LSE_ABS, f"LSE{tag}: abs err {d:.3e}"
        return stats

    def check_bwd(self, tag=""):
        dq, dk, dv = self.run_bwd()
        rdq, rdk, rdv = self.oracle_bwd()
        real = self.q_idx >= 0
        out = [check_close(f"dQ{tag}", dq, rdq, rows=real), check_close(f"dK{tag}", dk, rdk),
               check_close(f"dV{tag}", dv, rdv)]
        if (~real).any():
            assert (dq[~real] == 0).all(), "padding rows of dQ must be zero"
        return out
