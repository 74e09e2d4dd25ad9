"""wlb_attn_fwd_static: the forward for callers that cannot allocate.  Its scratch (the schedule
tables) is a fixed device array inside the library, shared by every call on the GPU and holding
the previous call's contents, so the test runs two calls in a row -- the second on a smaller input --
and checks each against wlb_attn_fwd, which keeps the same tables in a caller's workspace."""
import numpy as np
import pytest

from oracle import shard as osh
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl
from gpu_helpers import Guarded, check_close, LSE_ABS

pytestmark = pytest.mark.gpu


def _run_both(seed, docs, hq, hkv, d, cp, rank):
    import torch
    dev = "cuda:0"
    w, tens = wl.small_case(seed, docs, hq, hkv, d)
    sh = osh.shard(docs, cp, rank, osh.PER_DOC_PADDED)
    qi = sh["q_idx"]
    rows = np.maximum(qi, 0)
    q = B.bf16_bits_to_tensor(tens["q"][rows], dev)
    k, v = B.bf16_bits_to_tensor(tens["k"], dev), B.bf16_bits_to_tensor(tens["v"], dev)
    attn = B.Attention(qi, sh["cu_seqlens_k"], int(sh["cu_seqlens_k"][-1]), hq, hkv, d, w.scale, dev)
    n_q = len(qi)
    # the existing entry point, in the schedule the new one uses and in the one the library picks
    o_items, lse_items = attn.forward(q, k, v, extra_flags=B.ATTN_SCHEDULE_ITEMS)
    attn.planned = False
    o_auto, lse_auto = attn.forward(q, k, v)
    torch.cuda.synchronize()
    # the new one: outputs between guard bands, no workspace anywhere
    go = Guarded(torch, (n_q, hq, d), torch.bfloat16, dev, "O")
    gl = Guarded(torch, (hq, n_q), torch.float32, dev, "LSE")
    B.wlb_attn_fwd_static(attn.desc, q, k, v, attn.q_idx, attn.cu_k, go.t, gl.t)
    torch.cuda.synchronize()
    go.check()
    gl.check()
    assert torch.equal(go.t, o_items) and torch.equal(gl.t, lse_items), "same kernels, same schedule: bit for bit"
    real = qi >= 0
    check_close("O vs wlb_attn_fwd", B.tensor_to_f64(go.t), B.tensor_to_f64(o_auto), rows=real)
    if real.any():
        assert np.abs(B.tensor_to_f64(gl.t)[:, real] - B.tensor_to_f64(lse_auto)[:, real]).max() <= LSE_ABS
    # a second layer with the same mask: the schedule in the library's array is reused
    go2 = Guarded(torch, (n_q, hq, d), torch.bfloat16, dev, "O")
    gl2 = Guarded(torch, (hq, n_q), torch.float32, dev, "LSE")
    B.wlb_attn_fwd_static(attn.desc_reuse, q, k, v, None, None, go2.t, gl2.t)
    torch.cuda.synchronize()
    go2.check()
    gl2.check()
    assert torch.equal(go2.t, o_items) and torch.equal(gl2.t, lse_items)


def test_two_calls_in_a_row_second_one_smaller():
    _run_both(301, [2600, 1, 37, 900, 130, 64, 700], 8, 2, 128, 2, 1)     # several tiles, pads, GQA
    _run_both(302, [300, 45, 1, 77], 4, 4, 64, 1, 0)                      # smaller: fewer rows, keys, tables
    _run_both(303, [5], 2, 1, 128, 1, 0)                                  # smaller again: less than one tile


def test_limits_and_flags():
    import torch
    docs = [64]
    w, tens = wl.small_case(304, docs, 2, 1, 64)
    dev = "cuda:0"
    q = B.bf16_bits_to_tensor(tens["q"], dev)
    k, v = B.bf16_bits_to_tensor(tens["k"], dev), B.bf16_bits_to_tensor(tens["v"], dev)
    o = torch.empty_like(q)
    lse = torch.empty((2, 64), dtype=torch.float32, device=dev)
    qi = torch.arange(64, dtype=torch.int32, device=dev)
    cu = torch.tensor([0, 64], dtype=torch.int32, device=dev)
    with pytest.raises(B.WlbError) as e:      # a schedule larger than the library's array (nothing is launched)
        B.wlb_attn_fwd_static(B._desc(300000, 300000, 1, 2, 1, 64, 0.125), q, k, v, qi, cu, o, lse)
    assert e.value.status == 3
    with pytest.raises(B.WlbError) as e:      # the gang schedule needs partial-result scratch
        B.wlb_attn_fwd_static(B._desc(64, 64, 1, 2, 1, 64, 0.125, B.ATTN_SCHEDULE_GANGS), q, k, v, qi, cu, o, lse)
    assert e.value.status == 1
