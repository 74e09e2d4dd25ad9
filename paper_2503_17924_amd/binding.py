"""ctypes binding of libwlb.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/wlb.h).
Host calls take and return numpy arrays; device calls take torch tensors that
live on the GPU (torch is used for device memory and streams, nothing else) and
enqueue work on torch's current stream.  There is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# WLB_LIBRARY selects another build of the library (e.g. one made with different compiler flags)
LIB_PATH = os.environ.get("WLB_LIBRARY") or os.path.join(_HERE, "libwlb.so")

WLB_OK = 0
SHARD_PER_DOC_PADDED = 0
SHARD_PER_SEQ = 1
SHARD_PER_DOC_NOPAD = 2
ATTN_REUSE_PLAN = 1
ATTN_BWD_SKIP_DELTA = 2
ATTN_BWD_SKIP_DQ = 4
ATTN_BWD_SKIP_DKV = 8
ATTN_SCHEDULE_GANGS = 32
ATTN_SCHEDULE_ITEMS = 64
ATTN_NO_SHORT_PATH = 128

STATUS_NAMES = {0: "WLB_OK", 1: "WLB_ERR_INVALID_ARG", 2: "WLB_ERR_BUFFER_TOO_SMALL",
                3: "WLB_ERR_UNSUPPORTED", 4: "WLB_ERR_HIP"}

EXPORTS = ["wlb_last_error", "wlb_pack", "wlb_pack_optimal", "wlb_packer_create", "wlb_packer_destroy", "wlb_packer_step",
           "wlb_packer_pending", "wlb_calib_mfma", "wlb_calib_atomic_add", "wlb_predict_latency", "wlb_select_sharding", "wlb_shard_size", "wlb_shard", "wlb_attn_workspace_size",
           "wlb_attn_plan", "wlb_attn_plan_layout", "wlb_attn_set_gang_weights", "wlb_attn_get_gang_weights", "wlb_attn_fwd", "wlb_attn_fwd_static", "wlb_attn_bwd"]


class WlbError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class AttnDesc(C.Structure):
    _fields_ = [("n_q", C.c_int32), ("t_kv", C.c_int32), ("n_docs", C.c_int32), ("hq", C.c_int32),
                ("hkv", C.c_int32), ("head_dim", C.c_int32), ("scale", C.c_float), ("flags", C.c_int32),
                ("visible_pairs", C.c_int64)]


class PlanLayout(C.Structure):
    _fields_ = [("group_rows", C.c_int32), ("n_groups", C.c_int32), ("fwd_tile_rows", C.c_int32),
                ("n_fwd_tiles", C.c_int32), ("bwd_key_tile", C.c_int32), ("n_key_tiles", C.c_int32),
                ("off_row_lo", C.c_size_t), ("off_row_hi", C.c_size_t), ("off_group", C.c_size_t),
                ("off_group_real", C.c_size_t), ("off_fwd_order", C.c_size_t), ("off_fwd_cost", C.c_size_t), ("off_key_order", C.c_size_t),
                ("off_key_range", C.c_size_t), ("dkv_max_items", C.c_int32), ("dkv_max_partials", C.c_int32),
                ("off_key_ways", C.c_size_t), ("off_key_item_base", C.c_size_t), ("off_key_slot_base", C.c_size_t), ("off_dkv_counters", C.c_size_t),
                ("row_gangs", C.c_int32), ("uses_gangs", C.c_int32), ("off_fwd_prefix", C.c_size_t),
                ("n_blocks32", C.c_int32), ("off_block_hull", C.c_size_t), ("off_tile_short", C.c_size_t),
                ("off_gang_clock", C.c_size_t),
                ("plan_bytes", C.c_size_t)]


_lib = None


def lib():
    """Loads libwlb.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_17924_amd.build`")
        # torch ships its own HIP runtime; it must be in the process before libwlb.so is loaded
        # so that both resolve to the same one (streams and pointers cross between them)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.wlb_last_error.restype = C.c_char_p
        for name in EXPORTS[1:]:
            getattr(L, name).restype = C.c_int
        L.wlb_packer_destroy.restype = None
        L.wlb_packer_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _check(st: int):
    if st != WLB_OK:
        raise WlbError(st, lib().wlb_last_error().decode())


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _np_ptr(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


# ------------------------------------------------------------------------------- host calls
def wlb_pack(doc_len, n_microbatch: int, l_max: int, cost_a: int, cost_b: int):
    """-> (assign int32[n_docs], mb_len int64[N], mb_cost uint64[N])"""
    doc_len = _i32(doc_len)
    n = int(doc_len.shape[0])
    assign = np.empty(n, dtype=np.int32)
    mb_len = np.empty(max(n_microbatch, 1), dtype=np.int64)
    mb_cost = np.empty(max(n_microbatch, 1), dtype=np.uint64)
    _check(lib().wlb_pack(_np_ptr(doc_len, C.c_int32), C.c_int64(n), C.c_int32(n_microbatch), C.c_int64(l_max),
                          C.c_uint64(cost_a), C.c_uint64(cost_b), _np_ptr(assign, C.c_int32),
                          _np_ptr(mb_len, C.c_int64), _np_ptr(mb_cost, C.c_uint64)))
    return assign, mb_len[:n_microbatch], mb_cost[:n_microbatch]


def mfma_ceiling(random_operands: bool, n_iter: int = 4000, reps: int = 8) -> float:
    """Sustained dense bf16 MFMA TFLOP/s of the current GPU, measured with wlb_calib_mfma."""
    import torch
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    flops = C.c_double(0.0)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def launch():
        _check(lib().wlb_calib_mfma(C.c_int32(int(random_operands)), C.c_int32(n_iter), C.c_void_p(sink.data_ptr()),
                                    C.byref(flops), stream))
    for _ in range(reps):       # clocks settle over the first few milliseconds
        launch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return flops.value * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12


def atomic_add_rate(shared: bool, buf_mib: int = 256, n_iter: int = 200, reps: int = 3) -> float:
    """TB/s of fp32 data added to device memory by atomics, measured with wlb_calib_atomic_add."""
    import torch
    buf = torch.zeros(buf_mib << 18, dtype=torch.float32, device="cuda")
    done = C.c_double(0.0)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def launch():
        _check(lib().wlb_calib_atomic_add(C.c_int32(int(shared)), C.c_int32(n_iter), C.c_void_p(buf.data_ptr()),
                                          C.c_size_t(buf.numel() * 4), C.byref(done), stream))
    launch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return done.value * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12


def wlb_pack_optimal(doc_len, n_microbatch: int, l_max: int, cost_a: int, cost_b: int, node_limit: int = 0):
    """-> (assign, mb_len, mb_cost, optimal_cost, proven)"""
    doc_len = _i32(doc_len)
    assign = np.empty(len(doc_len), dtype=np.int32)
    mb_len = np.empty(n_microbatch, dtype=np.int64)
    mb_cost = np.empty(n_microbatch, dtype=np.uint64)
    opt, proven = C.c_uint64(0), C.c_int32(0)
    _check(lib().wlb_pack_optimal(_np_ptr(doc_len, C.c_int32), C.c_int64(len(doc_len)), C.c_int32(n_microbatch),
                                  C.c_int64(l_max), C.c_uint64(cost_a), C.c_uint64(cost_b), C.c_int64(node_limit),
                                  _np_ptr(assign, C.c_int32), _np_ptr(mb_len, C.c_int64), _np_ptr(mb_cost, C.c_uint64),
                                  C.byref(opt), C.byref(proven)))
    return assign, mb_len, mb_cost, opt.value, bool(proven.value)


class _KernelProfile(C.Structure):
    _fields_ = [("n_q", C.c_int32), ("n_kv", C.c_int32), ("q_len", C.POINTER(C.c_int32)),
                ("kv_len", C.POINTER(C.c_int32)), ("tflops", C.POINTER(C.c_double)),
                ("tile_q", C.c_int32), ("tile_k", C.c_int32)]


class KernelProfile:
    """The profiled-rate table wlb_predict_latency / wlb_select_sharding read (host arrays kept alive here)."""

    def __init__(self, q_grid, kv_grid, tflops, tile_q: int = 128, tile_k: int = 64):
        self.q = _i32(q_grid)
        self.kv = _i32(kv_grid)
        self.t = np.ascontiguousarray(tflops, dtype=np.float64)
        assert self.t.shape == (len(self.q), len(self.kv))
        self.c = _KernelProfile(len(self.q), len(self.kv), _np_ptr(self.q, C.c_int32), _np_ptr(self.kv, C.c_int32),
                                _np_ptr(self.t, C.c_double), tile_q, tile_k)


def wlb_predict_latency(doc_len, cp: int, mode: int, hq: int, head_dim: int, profile: KernelProfile):
    doc_len = _i32(doc_len)
    out = np.zeros(cp, dtype=np.float64)
    _check(lib().wlb_predict_latency(_np_ptr(doc_len, C.c_int32), C.c_int64(len(doc_len)), C.c_int32(cp), C.c_int32(mode),
                                     C.c_int32(hq), C.c_int32(head_dim), C.byref(profile.c), _np_ptr(out, C.c_double)))
    return out


def wlb_select_sharding(doc_len, cp: int, hq: int, head_dim: int, profile: KernelProfile):
    """-> (mode, predicted latency per-sequence, predicted latency per-document), seconds"""
    doc_len = _i32(doc_len)
    mode, a, b = C.c_int32(-1), C.c_double(0.0), C.c_double(0.0)
    _check(lib().wlb_select_sharding(_np_ptr(doc_len, C.c_int32), C.c_int64(len(doc_len)), C.c_int32(cp), C.c_int32(hq),
                                     C.c_int32(head_dim), C.byref(profile.c), C.byref(mode), C.byref(a), C.byref(b)))
    return mode.value, a.value, b.value


class Packer:
    """wlb_packer_create / wlb_packer_step / wlb_packer_pending / wlb_packer_destroy."""

    def __init__(self, n_microbatch: int, l_max: int, cost_a: int, cost_b: int, thresholds=()):
        th = np.ascontiguousarray(list(thresholds), dtype=np.int64)
        self.n = n_microbatch
        self._h = C.c_void_p(0)
        _check(lib().wlb_packer_create(C.c_int32(n_microbatch), C.c_int64(l_max), C.c_uint64(cost_a),
                                       C.c_uint64(cost_b), _np_ptr(th, C.c_int64) if len(th) else None,
                                       C.c_int32(len(th)), C.byref(self._h)))

    def pending(self):
        a, b = C.c_int64(0), C.c_int64(0)
        _check(lib().wlb_packer_pending(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def step(self, doc_id, doc_len):
        """-> (placed doc ids, their lengths, their micro-batch, mb_len, mb_cost)"""
        doc_len = _i32(doc_len)
        doc_id = np.ascontiguousarray(doc_id, dtype=np.int64)
        cap = sum(self.pending()) + len(doc_len)
        oid = np.empty(max(cap, 1), dtype=np.int64)
        olen = np.empty(max(cap, 1), dtype=np.int32)
        omb = np.empty(max(cap, 1), dtype=np.int32)
        mb_len = np.empty(self.n, dtype=np.int64)
        mb_cost = np.empty(self.n, dtype=np.uint64)
        n_out = C.c_int64(0)
        _check(lib().wlb_packer_step(self._h, _np_ptr(doc_len, C.c_int32), _np_ptr(doc_id, C.c_int64),
                                     C.c_int64(len(doc_len)), _np_ptr(oid, C.c_int64), _np_ptr(olen, C.c_int32),
                                     _np_ptr(omb, C.c_int32), C.c_int64(cap), C.byref(n_out),
                                     _np_ptr(mb_len, C.c_int64), _np_ptr(mb_cost, C.c_uint64)))
        k = n_out.value
        return oid[:k], olen[:k], omb[:k], mb_len, mb_cost

    def close(self):
        if self._h:
            lib().wlb_packer_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def wlb_shard_size(doc_len, cp: int, rank: int, mode: int):
    doc_len = _i32(doc_len)
    n_q, n_seg = C.c_int64(0), C.c_int64(0)
    _check(lib().wlb_shard_size(_np_ptr(doc_len, C.c_int32), C.c_int64(doc_len.shape[0]), C.c_int32(cp),
                                C.c_int32(rank), C.c_int32(mode), C.byref(n_q), C.byref(n_seg)))
    return n_q.value, n_seg.value


def wlb_shard(doc_len, cp: int, rank: int, mode: int):
    """-> dict(q_idx, cu_seqlens_q, seg_k_begin, seg_k_end, cu_seqlens_k, useful_pairs)"""
    doc_len = _i32(doc_len)
    n_q, n_seg = wlb_shard_size(doc_len, cp, rank, mode)
    n_docs = int(doc_len.shape[0])
    q_idx = np.empty(n_q, dtype=np.int32)
    cu_q = np.empty(n_seg + 1, dtype=np.int32)
    kb = np.empty(n_seg, dtype=np.int32)
    ke = np.empty(n_seg, dtype=np.int32)
    cu_k = np.empty(n_docs + 1, dtype=np.int32)
    pairs = C.c_int64(0)
    _check(lib().wlb_shard(_np_ptr(doc_len, C.c_int32), C.c_int64(n_docs), C.c_int32(cp), C.c_int32(rank),
                           C.c_int32(mode), _np_ptr(q_idx, C.c_int32), _np_ptr(cu_q, C.c_int32),
                           _np_ptr(kb, C.c_int32), _np_ptr(ke, C.c_int32), _np_ptr(cu_k, C.c_int32),
                           C.byref(pairs)))
    return dict(q_idx=q_idx, cu_seqlens_q=cu_q, seg_k_begin=kb, seg_k_end=ke, cu_seqlens_k=cu_k,
                useful_pairs=pairs.value)


# ----------------------------------------------------------------------------- device calls
def _desc(n_q, t_kv, n_docs, hq, hkv, head_dim, scale, flags=0, visible_pairs=0):
    return AttnDesc(int(n_q), int(t_kv), int(n_docs), int(hq), int(hkv), int(head_dim), float(scale), int(flags),
                    int(visible_pairs))


def wlb_attn_workspace_size(desc: AttnDesc):
    f, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().wlb_attn_workspace_size(C.byref(desc), C.byref(f), C.byref(b)))
    return f.value, b.value


def wlb_attn_plan_layout(desc: AttnDesc) -> PlanLayout:
    lay = PlanLayout()
    _check(lib().wlb_attn_plan_layout(C.byref(desc), C.byref(lay)))
    return lay


def _dev_ptr(t, dtype=None):
    import torch
    if t is None:
        return C.c_void_p(0)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("expected a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def wlb_attn_plan(desc, q_idx, cu_seqlens_k, workspace):
    import torch
    _check(lib().wlb_attn_plan(C.byref(desc), _dev_ptr(q_idx, torch.int32), _dev_ptr(cu_seqlens_k, torch.int32),
                               _dev_ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                               _stream()))


def wlb_attn_fwd(desc, q, k, v, q_idx, cu_seqlens_k, o, lse, workspace):
    import torch
    bf = torch.bfloat16
    _check(lib().wlb_attn_fwd(C.byref(desc), _dev_ptr(q, bf), _dev_ptr(k, bf), _dev_ptr(v, bf),
                              _dev_ptr(q_idx, torch.int32), _dev_ptr(cu_seqlens_k, torch.int32),
                              _dev_ptr(o, bf), _dev_ptr(lse, torch.float32), _dev_ptr(workspace),
                              C.c_size_t(workspace.numel() * workspace.element_size()), _stream()))


def wlb_attn_fwd_static(desc, q, k, v, q_idx, cu_seqlens_k, o, lse):
    import torch
    bf = torch.bfloat16
    _check(lib().wlb_attn_fwd_static(C.byref(desc), _dev_ptr(q, bf), _dev_ptr(k, bf), _dev_ptr(v, bf),
                                     _dev_ptr(q_idx, torch.int32), _dev_ptr(cu_seqlens_k, torch.int32),
                                     _dev_ptr(o, bf), _dev_ptr(lse, torch.float32), _stream()))


def wlb_attn_bwd(desc, q, k, v, o, lse, d_o, q_idx, cu_seqlens_k, dq, dk, dv, workspace):
    import torch
    bf = torch.bfloat16
    _check(lib().wlb_attn_bwd(C.byref(desc), _dev_ptr(q, bf), _dev_ptr(k, bf), _dev_ptr(v, bf), _dev_ptr(o, bf),
                              _dev_ptr(lse, torch.float32), _dev_ptr(d_o, bf), _dev_ptr(q_idx, torch.int32),
                              _dev_ptr(cu_seqlens_k, torch.int32), _dev_ptr(dq, bf), _dev_ptr(dk, bf),
                              _dev_ptr(dv, bf), _dev_ptr(workspace),
                              C.c_size_t(workspace.numel() * workspace.element_size()), _stream()))


# ------------------------------------------------------------------ convenience (allocation only)
class Attention:
    """Owns the output tensors and workspace for one (shape, mask); all arithmetic is in libwlb."""

    def __init__(self, q_idx, cu_seqlens_k, t_kv, hq, hkv, head_dim, scale, device="cuda:0", visible_pairs=0):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.q_idx = torch.as_tensor(np.ascontiguousarray(q_idx, dtype=np.int32)).to(self.device)
        self.cu_k = torch.as_tensor(np.ascontiguousarray(cu_seqlens_k, dtype=np.int32)).to(self.device)
        self.n_q = int(self.q_idx.numel())
        self.shape = (self.n_q, int(t_kv), int(self.cu_k.numel()) - 1, hq, hkv, head_dim, scale)
        self.visible_pairs = int(visible_pairs)     # wlb_shard's useful_pairs, if the caller has it (schedule choice only)
        self.desc = self.make_desc(0)
        self.desc_reuse = self.make_desc(ATTN_REUSE_PLAN)
        _, bwd_bytes = wlb_attn_workspace_size(self.desc)
        self.workspace = torch.empty(bwd_bytes, dtype=torch.uint8, device=self.device)
        self.planned = False

    def make_desc(self, flags):
        return _desc(*self.shape, flags=flags, visible_pairs=self.visible_pairs)

    def plan(self):
        wlb_attn_plan(self.desc, self.q_idx, self.cu_k, self.workspace)
        self.planned = True

    def forward(self, q, k, v, o=None, lse=None, extra_flags=0):
        torch = self.torch
        n_q, _, _, hq, _, d, _ = self.shape
        if o is None:
            o = torch.empty((n_q, hq, d), dtype=torch.bfloat16, device=self.device)
        if lse is None:
            lse = torch.empty((hq, n_q), dtype=torch.float32, device=self.device)
        desc = self.desc_reuse if self.planned else self.desc
        if extra_flags:
            desc = self.make_desc(desc.flags | extra_flags)
        wlb_attn_fwd(desc, q, k, v, self.q_idx, self.cu_k, o, lse, self.workspace)
        self.planned = True
        return o, lse

    def backward(self, q, k, v, o, lse, d_o, dq=None, dk=None, dv=None, extra_flags=0):
        torch = self.torch
        if dq is None:
            dq = torch.empty_like(q)
        if dk is None:
            dk = torch.empty_like(k)
        if dv is None:
            dv = torch.empty_like(v)
        desc = self.desc_reuse if self.planned else self.desc
        if extra_flags:
            desc = self.make_desc(desc.flags | extra_flags)
        wlb_attn_bwd(desc, q, k, v, o, lse, d_o, self.q_idx, self.cu_k, dq, dk, dv, self.workspace)
        self.planned = True
        return dq, dk, dv


def wlb_attn_set_gang_weights(kernel: int, weights=None):
    """weights: 16 integers [half of the launch][XCD], or None for the defaults."""
    if weights is None:
        _check(lib().wlb_attn_set_gang_weights(C.c_int32(kernel), None))
    else:
        w = _i32(np.asarray(weights).reshape(16))
        _check(lib().wlb_attn_set_gang_weights(C.c_int32(kernel), _np_ptr(w, C.c_int32)))


def plan_tables(attn: "Attention") -> dict:
    """The schedule the last wlb_attn_plan / forward / backward call of `attn` left in its workspace, as host
    arrays (reads the workspace: synchronises).  Keys: row_lo, row_hi [n_q]; group [n_groups][4] (hull and fully
    visible key range of each 64-row group); fwd_cost [n_fwd_tiles] (64-key tiles a query tile visits), fwd_order
    (heaviest first), fwd_prefix [n_fwd_tiles + 1] (running cost in that order, fixed cost per tile included);
    tile_short; key_range [n_key_tiles][2] (row groups a key tile is visible to), key_ways (items a key tile is
    split into), key_order, key_item_base; layout (the PlanLayout)."""
    lay = wlb_attn_plan_layout(attn.desc)
    ws = attn.workspace[:lay.plan_bytes].cpu().numpy()
    i32 = lambda off, n: ws[off:off + 4 * n].view(np.int32).copy()
    n_q = attn.shape[0]
    return {
        "layout": lay,
        "row_lo": i32(lay.off_row_lo, n_q), "row_hi": i32(lay.off_row_hi, n_q),
        "group": i32(lay.off_group, 4 * lay.n_groups).reshape(-1, 4),
        "fwd_cost": i32(lay.off_fwd_cost, lay.n_fwd_tiles), "fwd_order": i32(lay.off_fwd_order, lay.n_fwd_tiles),
        "fwd_prefix": ws[lay.off_fwd_prefix:lay.off_fwd_prefix + 8 * (lay.n_fwd_tiles + 1)].view(np.int64).copy(),
        "tile_short": i32(lay.off_tile_short, lay.n_fwd_tiles),
        "key_range": i32(lay.off_key_range, 2 * lay.n_key_tiles).reshape(-1, 2),
        "key_ways": i32(lay.off_key_ways, lay.n_key_tiles), "key_order": i32(lay.off_key_order, lay.n_key_tiles),
        "key_item_base": i32(lay.off_key_item_base, lay.n_key_tiles + 1),
    }


def plan_report(attn: "Attention", name: str = "") -> str:
    """A few lines of text about the schedule in `attn`'s workspace: what the work items cost and how they are
    spread (for looking at a schedule by eye; bench.py prints it when WLB_TRACE=1)."""
    t = plan_tables(attn)
    lay = t["layout"]
    n_q, t_kv, n_docs, hq, hkv, d = attn.shape[:6]
    cost = t["fwd_cost"][t["fwd_order"]].astype(np.int64)
    per = np.diff(t["fwd_prefix"])
    lines = [f"plan {name}: n_q {n_q} t_kv {t_kv} docs {n_docs} heads {hq}/{hkv} D {d}: "
             f"{lay.n_fwd_tiles} query tiles ({int(t['tile_short'].sum())} short-hull), {lay.n_key_tiles} key tiles, "
             f"{'gang' if lay.uses_gangs else 'item'} schedule for forward and dQ"]
    q = lambda a: "min %d  median %d  max %d  sum %d" % (a.min(), np.median(a), a.max(), a.sum()) if len(a) else "none"
    lines.append(f"  query tile cost (64-key tiles visited, heaviest first): {q(cost)}; first ten: {cost[:10].tolist()}")
    if lay.uses_gangs:
        w = wlb_attn_get_gang_weights(0).astype(np.int64).reshape(2, 8)
        ng = lay.row_gangs
        gw = np.array([w[0 if g < ng // 2 else 1][g % 8] for g in range(ng)])
        cum = np.concatenate([[0], np.cumsum(gw)])
        total = int(t["fwd_prefix"][-1]) * hkv
        begin = total * cum // cum[-1]
        share = np.diff(begin)
        lines.append(f"  forward work line: {total} units (tile cost + fixed part, x KV heads) over {ng} gangs of {hq // hkv} "
                     f"workgroups: share {q(share)}")
    else:
        lines.append(f"  forward / dQ items: {lay.n_fwd_tiles * hq} (tile, head), cost with fixed part {q(per)}")
    kr = t["key_range"]
    stages = (kr[:, 1] - kr[:, 0]).astype(np.int64) * (hq // hkv) // np.maximum(t["key_ways"], 1)
    lines.append(f"  dK/dV items: {int(t['key_item_base'][-1])} (key tile, KV head, head part); tiles split "
                 f"{dict(zip(*[x.tolist() for x in np.unique(t['key_ways'], return_counts=True)]))} ways; stages per item {q(stages)}")
    return "\n".join(lines)


def wlb_attn_get_gang_weights(kernel: int) -> np.ndarray:
    """The 16 weights in force for the forward (0) or dQ (1) gang kernel: [half of the launch][XCD]."""
    out = np.zeros(16, dtype=np.int32)
    _check(lib().wlb_attn_get_gang_weights(C.c_int32(kernel), _np_ptr(out, C.c_int32)))
    return out


def gang_clocks(attn: "Attention") -> np.ndarray:
    """The start / end real-time counter values (100 MHz ticks) the gang kernels' workgroups left in the workspace
    on their last launch: uint64 [2 (forward, dQ)][workgroups][2 (start, end)].  Reads the workspace (synchronises)."""
    lay = wlb_attn_plan_layout(attn.desc)
    n = lay.row_gangs * (attn.shape[3] // attn.shape[4])
    raw = attn.workspace[lay.off_gang_clock:lay.off_gang_clock + 2 * n * 2 * 8].cpu().numpy()
    return raw.view(np.uint64).reshape(2, n, 2)


def calibrate_gang_weights(attns, launch, rounds: int = 3, extra_flags: int = 0):
    """Sets the XCD part of the gang schedule's share weights from measurement on this GPU.

    The XCDs of one GPU run the forward and dQ kernels at speeds that differ by several percent (the same
    ones are slow in every launch, which ones differs from GPU to GPU), and a gang's workgroups all sit on
    one XCD (gang g on XCD g % 8).  `attns` are Attention objects whose problems use the gang schedule and
    `launch()` runs forward and backward of each of them once (the caller's own tensors; `extra_flags` are the
    descriptor flags those calls add, e.g. a forced schedule).  Per
    round: launch twice, read the gangs' recorded clocks, and scale each XCD's weight by mean end time /
    its gangs' median end time; the split between the halves of a launch keeps its default.  The weights
    hold for the process (wlb_attn_set_gang_weights(k, None) restores the defaults).  Returns
    {"fwd": [8 factors], "dq": [8 factors]} (relative speeds, mean 1), or None if no problem uses gangs."""
    import torch
    use = [a for a in attns if wlb_attn_plan_layout(a.make_desc(a.desc.flags | extra_flags)).uses_gangs]
    if not use:
        return None
    factor = np.ones((2, 8))
    default = []
    for kern in (0, 1):
        wlb_attn_set_gang_weights(kern, None)
        default.append(wlb_attn_get_gang_weights(kern).astype(np.float64).reshape(2, 8))
    for _ in range(rounds):
        launch()
        launch()
        torch.cuda.synchronize()
        ends = np.zeros((2, 8))
        for a in use:
            lay = wlb_attn_plan_layout(a.desc)
            group = a.shape[3] // a.shape[4]
            b = np.arange(lay.row_gangs * group)
            gang = ((b // 8) // group) * 8 + b % 8
            clk = gang_clocks(a).astype(np.int64)
            for kern in (0, 1):
                end = clk[kern, :, 1] - clk[kern, :, 0].min()
                gend = np.array([end[gang == i].max() for i in range(lay.row_gangs)], dtype=np.float64)
                xcd = np.arange(lay.row_gangs) % 8
                per = np.array([np.median(gend[xcd == x]) if (xcd == x).any() else gend.mean() for x in range(8)])
                ends[kern] += per / per.mean() / len(use)
        factor = factor / ends
        factor = np.clip(factor / factor.mean(axis=1, keepdims=True), 0.8, 1.25)
        for kern in (0, 1):
            w = default[kern] * factor[kern][None, :] * 10.0
            wlb_attn_set_gang_weights(kern, np.maximum(np.rint(w), 1).astype(np.int32).reshape(16))
    return {"fwd": [round(float(x), 4) for x in factor[0]], "dq": [round(float(x), 4) for x in factor[1]]}


def bf16_bits_to_tensor(bits: np.ndarray, device="cuda:0"):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device (a reinterpretation)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def tensor_to_f64(t) -> np.ndarray:
    """GPU tensor (bf16 or fp32) -> numpy float64 on the host."""
    return t.detach().to("cpu").double().numpy()
