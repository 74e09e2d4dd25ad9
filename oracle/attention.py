"""Oracle: document-masked causal attention, forward and backward, in fp64.

TEST INFRASTRUCTURE ONLY.  Nothing here is used by the HIP path.

What is computed (paper Section 1 and Section 3.2: several documents are packed
into one sequence and a mask keeps a token from attending to tokens of another
document; within a document the mask is causal; Section 2.1: a context-parallel
rank holds a subset of the query rows and the gathered K/V of all tokens, and
the K/V gradients it produces are partial sums to be reduce-scattered):

for local row i with global token index g = q_idx[i], lying in document [s, e),
query head h and KV head h' = h // (Hq // Hkv):

    z_ij  = scale * <q_ih, k_jh'>            for j in [s, g]   (diagonal included)
    LSE_ih = log sum_j exp(z_ij)             (natural log)
    P_ij  = exp(z_ij - LSE_ih)
    O_ih  = sum_j P_ij v_jh'

backward (the standard softmax-attention derivative; the paper measures it but
does not restate it), with dO the gradient w.r.t. O:

    delta_ih = <dO_ih, O_ih>
    dP_ij = <dO_ih, v_jh'>
    dS_ij = P_ij (dP_ij - delta_ih)
    dQ_ih  = scale * sum_j dS_ij k_jh'
    dK_jh' = scale * sum_{h in group} sum_i dS_ij q_ih      (this rank's rows only)
    dV_jh' =         sum_{h in group} sum_i P_ij  dO_ih

Rows with q_idx = -1 are padding: O = 0, LSE = -inf, dQ = 0, no contribution.

Inputs are float arrays (the tests pass bf16-rounded values widened to fp64);
every sum is carried in fp64 and outputs stay fp64.  Rows are processed in
blocks only to bound memory: each row's result is independent of the blocking.

Pins (tests/test_oracle_attention.py): brute-force dense masked softmax on tiny
inputs, packed == per-document, single-token document returns V, constant V,
the Q = 0 closed form (prefix mean of V, LSE = ln(pos+1)), a library causal
SDPA routine with autograd for the single-document case, central finite
differences for the backward, and the dV / dO column-sum invariant.
"""
from __future__ import annotations

import numpy as np

_ROW_BLOCK_ELEMS = 1 << 24   # rows*keys per fp64 score block (128 MiB)


def _doc_of_rows(q_idx: np.ndarray, cu_seqlens_k: np.ndarray):
    """For each local row: (document id, document start); pads get (-1, 0)."""
    q_idx = np.asarray(q_idx, dtype=np.int64)
    cu = np.asarray(cu_seqlens_k, dtype=np.int64)
    doc = np.searchsorted(cu, q_idx, side="right") - 1
    doc = np.where(q_idx < 0, -1, doc)
    if (q_idx >= cu[-1]).any():
        raise ValueError("q_idx entry beyond the packed sequence")
    return doc


def attn_fwd(q, k, v, q_idx, cu_seqlens_k, scale):
    """q [n_q,Hq,D], k,v [T,Hkv,D] -> O [n_q,Hq,D] fp64, LSE [Hq,n_q] fp64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    q_idx = np.asarray(q_idx, dtype=np.int64)
    cu = np.asarray(cu_seqlens_k, dtype=np.int64)
    n_q, hq, d = q.shape
    t, hkv, _ = k.shape
    assert hq % hkv == 0 and cu[-1] == t and q_idx.shape == (n_q,)
    group = hq // hkv
    o = np.zeros((n_q, hq, d), dtype=np.float64)
    lse = np.full((hq, n_q), -np.inf, dtype=np.float64)
    doc = _doc_of_rows(q_idx, cu)
    for dd in np.unique(doc[doc >= 0]):
        s, e = int(cu[dd]), int(cu[dd + 1])
        rows_all = np.nonzero(doc == dd)[0]
        step = max(1, _ROW_BLOCK_ELEMS // max(1, e - s))
        for b in range(0, len(rows_all), step):
            rows = rows_all[b:b + step]
            pos = q_idx[rows] - s                                  # position inside the document
            visible = np.arange(e - s)[None, :] <= pos[:, None]    # j <= i, same document
            for h in range(hq):
                hk = h // group
                z = scale * (q[rows, h, :] @ k[s:e, hk, :].T)
                z = np.where(visible, z, -np.inf)
                m = z.max(axis=1, keepdims=True)
                p = np.exp(z - m)
                l = p.sum(axis=1, keepdims=True)
                o[rows, h, :] = (p / l) @ v[s:e, hk, :]
                lse[h, rows] = (m + np.log(l))[:, 0]
    return o, lse


def attn_bwd(q, k, v, do, q_idx, cu_seqlens_k, scale):
    """Returns dQ [n_q,Hq,D], dK [T,Hkv,D], dV [T,Hkv,D] (fp64); dK/dV hold the
    contribution of the given rows only (a context-parallel rank's partial)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    q_idx = np.asarray(q_idx, dtype=np.int64)
    cu = np.asarray(cu_seqlens_k, dtype=np.int64)
    n_q, hq, d = q.shape
    t, hkv, _ = k.shape
    group = hq // hkv
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    doc = _doc_of_rows(q_idx, cu)
    for dd in np.unique(doc[doc >= 0]):
        s, e = int(cu[dd]), int(cu[dd + 1])
        rows_all = np.nonzero(doc == dd)[0]
        step = max(1, _ROW_BLOCK_ELEMS // max(1, e - s))
        for b in range(0, len(rows_all), step):
            rows = rows_all[b:b + step]
            pos = q_idx[rows] - s
            visible = np.arange(e - s)[None, :] <= pos[:, None]
            for h in range(hq):
                hk = h // group
                kk, vv = k[s:e, hk, :], v[s:e, hk, :]
                z = scale * (q[rows, h, :] @ kk.T)
                z = np.where(visible, z, -np.inf)
                m = z.max(axis=1, keepdims=True)
                p = np.exp(z - m)
                p = p / p.sum(axis=1, keepdims=True)
                out = p @ vv
                delta = (do[rows, h, :] * out).sum(axis=1, keepdims=True)
                dp = do[rows, h, :] @ vv.T
                ds = p * (dp - delta)
                dq[rows, h, :] = scale * (ds @ kk)
                dk[s:e, hk, :] += scale * (ds.T @ q[rows, h, :])
                dv[s:e, hk, :] += p.T @ do[rows, h, :]
    return dq, dk, dv


def useful_pairs(q_idx, cu_seqlens_k) -> int:
    """In-document causal (query, key) pairs of the given rows, diagonal included."""
    q_idx = np.asarray(q_idx, dtype=np.int64)
    cu = np.asarray(cu_seqlens_k, dtype=np.int64)
    doc = _doc_of_rows(q_idx, cu)
    real = doc >= 0
    return int((q_idx[real] - cu[doc[real]] + 1).sum())
