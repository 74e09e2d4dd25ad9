"""Shared plumbing of the GPU parity tests: run the HIP path and the oracle on the same
seeded inputs and compare with the acceptance bounds (errors relative to each tensor's
largest magnitude: max <= 2e-2, mean <= 2e-3; LSE absolute <= 1e-2)."""
import numpy as np

from oracle import attention as oat
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl

MAX_REL, MEAN_REL, LSE_ABS = 2e-2, 2e-3, 1e-2
# Only for a tensor that is zero in exact arithmetic (the oracle's own value is below ZERO_EPS, i.e.
# nothing but its fp64 rounding): the error is then measured against SCALE_FLOOR instead.
SCALE_FLOOR, ZERO_EPS = 1e-3, 1e-9
GUARD_BYTES = 1 << 16        # sentinel margin on both sides of every buffer the library writes
GUARD_BYTE = 0xA5


def check_close(name, got, ref, rows=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if rows is not None:
        got, ref = got[rows], ref[rows]
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    # Errors are relative to the tensor's largest magnitude.  A tensor that is exactly zero in
    # exact arithmetic (dQ when every document has one token: dS = dP - <dO, O> cancels) leaves
    # only the bf16 rounding of O behind on the GPU; only then is the scale 1e-3 (inputs are N(0,1)).
    scale = np.abs(ref).max()
    if scale < ZERO_EPS:
        scale = SCALE_FLOOR
    err = np.abs(got - ref)
    mx, mean = err.max() / scale, err.mean() / scale
    assert mx <= MAX_REL, f"{name}: max err {mx:.3e} > {MAX_REL}"
    assert mean <= MEAN_REL, f"{name}: mean err {mean:.3e} > {MEAN_REL}"
    return mx, mean


def gather_rows(bits, q_idx):
    """Rows of a [T, H, D] bit tensor selected by q_idx; padding slots read row 0."""
    return np.ascontiguousarray(bits[np.maximum(np.asarray(q_idx), 0)])


class Guarded:
    """A device buffer the library writes, with sentinel-filled margins on both sides.  The payload
    starts as NaN bit patterns (0xFF bytes), so an element the library leaves unwritten shows up as
    non-finite; check() asserts on the host that no byte of either margin has changed."""

    def __init__(self, torch, shape, dtype, device, name):
        self.name = name
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        self.nbytes = n
        tail = (-n) % 256
        self.raw = torch.full((GUARD_BYTES + n + tail + GUARD_BYTES,), GUARD_BYTE, dtype=torch.uint8, device=device)
        body = self.raw[GUARD_BYTES:GUARD_BYTES + n]
        body.fill_(0xFF)
        self.t = body.view(dtype).view(shape)

    def check(self):
        lo = self.raw[:GUARD_BYTES]
        hi = self.raw[GUARD_BYTES + self.nbytes:]
        assert bool((lo == GUARD_BYTE).all()), f"{self.name}: bytes before the buffer were written"
        assert bool((hi == GUARD_BYTE).all()), f"{self.name}: bytes after the buffer were written"


class Case:
    """One rank's attention problem: bf16 bit tensors on the host, tensors on the GPU.  Every buffer
    the library writes (O, LSE, dQ, dK, dV, the workspace) sits between guard bands that are checked
    after each call."""

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
        n_q = len(self.q_idx)
        bf, f32, u8 = torch.bfloat16, torch.float32, torch.uint8
        self.guarded = {
            "o": Guarded(torch, (n_q, hq, d), bf, device, "O"), "lse": Guarded(torch, (hq, n_q), f32, device, "LSE"),
            "dq": Guarded(torch, (n_q, hq, d), bf, device, "dQ"), "dk": Guarded(torch, (self.t_kv, hkv, d), bf, device, "dK"),
            "dv": Guarded(torch, (self.t_kv, hkv, d), bf, device, "dV"),
            "ws": Guarded(torch, (self.attn.workspace.numel(),), u8, device, "workspace")}
        self.attn.workspace = self.guarded["ws"].t

    def check_guards(self):
        for g in self.guarded.values():
            g.check()

    def f64(self, name):
        return wl.bf16_bits_to_f64(self.bits[name])

    def run_fwd(self):
        g = self.guarded
        o, lse = self.attn.forward(self.dev["q"], self.dev["k"], self.dev["v"], g["o"].t, g["lse"].t, extra_flags=self.flags)
        self.torch.cuda.synchronize()
        self.check_guards()
        self.o, self.lse = o, lse
        return B.tensor_to_f64(o), B.tensor_to_f64(lse)

    def run_bwd(self):
        g = self.guarded
        dq, dk, dv = self.attn.backward(self.dev["q"], self.dev["k"], self.dev["v"], self.o, self.lse,
                                        self.dev["do"], g["dq"].t, g["dk"].t, g["dv"].t, extra_flags=self.flags)
        self.torch.cuda.synchronize()
        self.check_guards()
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
