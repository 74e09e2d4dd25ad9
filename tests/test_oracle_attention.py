"""Pins for oracle/attention.py (CPU only): the oracle is checked against things
other than itself -- a dense brute force with an explicit boolean mask, closed
forms, a library SDPA routine with autograd, finite differences, invariants."""
import math

import numpy as np
import pytest
import torch

from oracle import attention as oat
from oracle import shard as osh
from paper_2503_17924_amd import workloads as wl


def _case(seed, docs, hq, hkv, d):
    w, t = wl.small_case(seed, docs, hq, hkv, d)
    f = {n: wl.bf16_bits_to_f64(a) for n, a in t.items()}
    cu = np.concatenate([[0], np.cumsum(docs)]).astype(np.int32)
    return w, f, cu


def _brute_force(q, k, v, q_idx, cu, scale):
    """Dense softmax over the whole packed sequence with an explicit mask matrix,
    scalar loops, no max subtraction (tiny inputs only)."""
    n_q, hq, d = q.shape
    t, hkv, _ = k.shape
    doc_of = np.zeros(t, dtype=int)
    for i in range(len(cu) - 1):
        doc_of[cu[i]:cu[i + 1]] = i
    o = np.zeros((n_q, hq, d))
    lse = np.full((hq, n_q), -np.inf)
    for i in range(n_q):
        g = q_idx[i]
        if g < 0:
            continue
        allowed = [(doc_of[j] == doc_of[g]) and (j <= g) for j in range(t)]
        for h in range(hq):
            hk = h // (hq // hkv)
            w = [math.exp(scale * float(np.dot(q[i, h], k[j, hk]))) if allowed[j] else 0.0 for j in range(t)]
            z = sum(w)
            for j in range(t):
                o[i, h] += (w[j] / z) * v[j, hk]
            lse[h, i] = math.log(z)
    return o, lse


def test_matches_brute_force_with_explicit_mask():
    docs = [5, 1, 9, 3]
    w, f, cu = _case(3, docs, 4, 2, 8)
    q_idx = np.arange(sum(docs))
    o, lse = oat.attn_fwd(f["q"], f["k"], f["v"], q_idx, cu, w.scale)
    bo, blse = _brute_force(f["q"], f["k"], f["v"], q_idx, cu, w.scale)
    np.testing.assert_allclose(o, bo, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, blse, rtol=1e-12, atol=1e-13)


def test_brute_force_on_a_sharded_rank_with_pads():
    docs = [5, 7, 2]
    w, f, cu = _case(4, docs, 2, 1, 4)
    for r in range(2):
        sh = osh.shard(docs, 2, r, osh.PER_DOC_PADDED)
        qi = sh["q_idx"]
        qrows = f["q"][np.maximum(qi, 0)]
        o, lse = oat.attn_fwd(qrows, f["k"], f["v"], qi, cu, w.scale)
        bo, blse = _brute_force(qrows, f["k"], f["v"], qi, cu, w.scale)
        np.testing.assert_allclose(o, bo, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse, blse, rtol=1e-12, atol=1e-13)
        assert (o[qi < 0] == 0).all() and np.isneginf(lse[:, qi < 0]).all()


def test_packed_equals_each_document_alone():
    docs = [17, 1, 40, 6]
    w, f, cu = _case(5, docs, 4, 2, 16)
    o, lse = oat.attn_fwd(f["q"], f["k"], f["v"], np.arange(sum(docs)), cu, w.scale)
    for i, L in enumerate(docs):
        s, e = cu[i], cu[i + 1]
        o1, l1 = oat.attn_fwd(f["q"][s:e], f["k"][s:e], f["v"][s:e], np.arange(L), [0, L], w.scale)
        np.testing.assert_allclose(o[s:e], o1, rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(lse[:, s:e], l1, rtol=1e-13, atol=1e-14)


def test_single_token_document_returns_its_value():
    docs = [4, 1, 1, 3]
    w, f, cu = _case(6, docs, 4, 2, 8)
    o, lse = oat.attn_fwd(f["q"], f["k"], f["v"], np.arange(sum(docs)), cu, w.scale)
    for tok in (4, 5):
        for h in range(4):
            np.testing.assert_allclose(o[tok, h], f["v"][tok, h // 2], rtol=1e-14)
            assert lse[h, tok] == pytest.approx(w.scale * np.dot(f["q"][tok, h], f["k"][tok, h // 2]), rel=1e-13)
    # first token of every document also sees only itself
    for s in cu[:-1]:
        np.testing.assert_allclose(o[s, 0], f["v"][s, 0], rtol=1e-14)


def test_constant_value_within_document():
    docs = [12, 7]
    w, f, cu = _case(7, docs, 2, 2, 8)
    v = f["v"].copy()
    v[0:12] = v[0]
    v[12:19] = v[12]
    o, _ = oat.attn_fwd(f["q"], f["k"], v, np.arange(19), cu, w.scale)
    for h in range(2):
        np.testing.assert_allclose(o[:12, h], np.broadcast_to(v[0, h], (12, 8)), rtol=1e-13)
        np.testing.assert_allclose(o[12:, h], np.broadcast_to(v[12, h], (7, 8)), rtol=1e-13)


def test_zero_query_closed_form():
    # q = 0 makes every visible key equally likely: O is the running mean of V
    # inside the document and LSE = ln(position + 1)
    docs = [300, 45, 1, 700]
    w, f, cu = _case(8, docs, 2, 1, 8)
    t = sum(docs)
    o, lse = oat.attn_fwd(np.zeros_like(f["q"]), f["k"], f["v"], np.arange(t), cu, w.scale)
    for i, L in enumerate(docs):
        s = cu[i]
        pm = np.cumsum(f["v"][s:s + L, 0], axis=0) / np.arange(1, L + 1)[:, None]
        for h in range(2):
            np.testing.assert_allclose(o[s:s + L, h], pm, rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(lse[h, s:s + L], np.log(np.arange(1, L + 1)), rtol=1e-12, atol=1e-14)


def _torch_sdpa(q, k, v, do, mask, scale, group):
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    kk = tk.repeat_interleave(group, dim=1)
    vv = tv.repeat_interleave(group, dim=1)
    out = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], kk.permute(1, 0, 2)[None], vv.permute(1, 0, 2)[None],
        attn_mask=torch.tensor(mask)[None, None], scale=scale)[0].permute(1, 0, 2)
    out.backward(torch.tensor(do, dtype=torch.float64))
    return out.detach().numpy(), tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("docs,hq,hkv", [([64], 2, 2), ([33], 4, 1), ([20, 1, 50, 9], 4, 2)])
def test_against_library_sdpa_and_autograd(docs, hq, hkv):
    w, f, cu = _case(9, docs, hq, hkv, 16)
    t = sum(docs)
    doc_of = np.repeat(np.arange(len(docs)), docs)
    mask = (doc_of[:, None] == doc_of[None, :]) & (np.arange(t)[None, :] <= np.arange(t)[:, None])
    ro, rdq, rdk, rdv = _torch_sdpa(f["q"], f["k"], f["v"], f["do"], mask, w.scale, hq // hkv)
    o, _ = oat.attn_fwd(f["q"], f["k"], f["v"], np.arange(t), cu, w.scale)
    dq, dk, dv = oat.attn_bwd(f["q"], f["k"], f["v"], f["do"], np.arange(t), cu, w.scale)
    np.testing.assert_allclose(o, ro, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dq, rdq, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dk, rdk, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dv, rdv, rtol=1e-10, atol=1e-11)


def test_backward_by_central_finite_differences():
    docs = [6, 3]
    w, f, cu = _case(10, docs, 2, 1, 4)
    qi = np.arange(9)
    dq, dk, dv = oat.attn_bwd(f["q"], f["k"], f["v"], f["do"], qi, cu, w.scale)

    def loss(q, k, v):
        return float((oat.attn_fwd(q, k, v, qi, cu, w.scale)[0] * f["do"]).sum())

    eps = 1e-5
    rng = np.random.default_rng(0)
    for name, grad in (("q", dq), ("k", dk), ("v", dv)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in grad.shape)
            args = {n: f[n].copy() for n in ("q", "k", "v")}
            args[name][idx] += eps
            up = loss(**args)
            args[name][idx] -= 2 * eps
            dn = loss(**args)
            assert (up - dn) / (2 * eps) == pytest.approx(grad[idx], rel=1e-6, abs=1e-8)


def test_dv_column_sums_equal_do_sums():
    # rows of P sum to one, so sum_j dV_j = sum over rows and grouped heads of dO
    docs = [40, 13, 77]
    w, f, cu = _case(11, docs, 4, 2, 8)
    _, _, dv = oat.attn_bwd(f["q"], f["k"], f["v"], f["do"], np.arange(130), cu, w.scale)
    for i in range(3):
        s, e = cu[i], cu[i + 1]
        for hk in range(2):
            want = f["do"][s:e, 2 * hk:2 * hk + 2].sum(axis=(0, 1))
            np.testing.assert_allclose(dv[s:e, hk].sum(axis=0), want, rtol=1e-11, atol=1e-12)


def test_dq_dk_inner_product_identity():
    # sum_i <q_i, dQ_i> = sum_j <k_j, dK_j>: both equal scale * sum_ij dS_ij z_ij / scale
    docs = [25, 60]
    w, f, cu = _case(12, docs, 4, 2, 8)
    dq, dk, _ = oat.attn_bwd(f["q"], f["k"], f["v"], f["do"], np.arange(85), cu, w.scale)
    assert (f["q"] * dq).sum() == pytest.approx((f["k"] * dk).sum(), rel=1e-10)


@pytest.mark.parametrize("mode", [osh.PER_DOC_PADDED, osh.PER_SEQ])
def test_rank_outputs_reassemble_the_unsharded_result(mode):
    docs = [37, 5, 64, 22]          # total 128, divisible by 2*CP for the per-sequence mode
    cp = 4
    w, f, cu = _case(13, docs, 4, 2, 8)
    t = sum(docs)
    o, lse = oat.attn_fwd(f["q"], f["k"], f["v"], np.arange(t), cu, w.scale)
    dq, dk, dv = oat.attn_bwd(f["q"], f["k"], f["v"], f["do"], np.arange(t), cu, w.scale)
    o_u, dq_u = np.zeros_like(o), np.zeros_like(dq)
    dk_s, dv_s = np.zeros_like(dk), np.zeros_like(dv)
    for r in range(cp):
        qi = osh.shard(docs, cp, r, mode)["q_idx"]
        real = qi >= 0
        rows = np.maximum(qi, 0)
        o_r, _ = oat.attn_fwd(f["q"][rows], f["k"], f["v"], qi, cu, w.scale)
        dq_r, dk_r, dv_r = oat.attn_bwd(f["q"][rows], f["k"], f["v"], f["do"][rows], qi, cu, w.scale)
        o_u[qi[real]] = o_r[real]
        dq_u[qi[real]] = dq_r[real]
        assert (dq_r[~real] == 0).all()
        dk_s += dk_r
        dv_s += dv_r
    np.testing.assert_allclose(o_u, o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dq_u, dq, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dk_s, dk, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dv_s, dv, rtol=1e-11, atol=1e-12)


def test_useful_pairs():
    assert oat.useful_pairs(np.arange(7), [0, 3, 7]) == 6 + 10
    assert oat.useful_pairs(np.array([2, -1, 6]), [0, 3, 7]) == 3 + 4
