"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

A full fp64 oracle pass over a 128K-token sequence costs about 1e14 flops, so these tests
compare what the oracle can compute in seconds -- sampled query rows (O, LSE, dQ), whole short
documents and the tail keys of the longest document (dK, dV: a rank's partial needs only that
rank's rows of the document) -- and check two identities that hold at any size on the full
output: sum_j dV_j = sum of dO over the rows and grouped heads that see j's document, and
sum_i <q_i, dQ_i> = sum_j <k_j, dK_j>."""
import numpy as np
import pytest

from oracle import attention as oat
from oracle import pack as opk
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl
from gpu_helpers import Case, check_close, LSE_ABS

pytestmark = pytest.mark.gpu


def _rows_sample(q_idx, cu, n, rng):
    """Real local rows: the first and last rows of every document present, the rows on both sides of the middle of
    its local rows (under per-document sharding the boundary between the early and the late chunk, which share a
    wavefront), plus random ones."""
    real = np.nonzero(q_idx >= 0)[0]
    doc = np.searchsorted(cu, q_idx[real], side="right") - 1
    picks = []
    for d in np.unique(doc):
        r = real[doc == d]
        picks += [r[0], r[-1], r[len(r) // 2], r[max(len(r) // 2 - 1, 0)]]
    picks += rng.choice(real, size=min(n, len(real)), replace=False).tolist()
    return np.unique(np.asarray(picks))


def _check_rows(c, o, lse, dq, rows, tag):
    """Oracle on a subset of rows: O, LSE and dQ are per-row quantities."""
    q = c.f64("q")[rows]
    k, v = c.f64("k"), c.f64("v")
    ro, rlse = oat.attn_fwd(q, k, v, c.q_idx[rows], c.cu_k, c.scale)
    check_close(f"O {tag}", o[rows], ro)
    assert np.abs(lse[:, rows] - rlse).max() <= LSE_ABS
    if dq is not None:
        rdq, _, _ = oat.attn_bwd(q, k, v, c.f64("do")[rows], c.q_idx[rows], c.cu_k, c.scale)
        # scale of the whole tensor: sampled rows only see part of it, use the GPU tensor's max as well
        check_close(f"dQ {tag}", dq[rows], rdq)


def _check_dkv_for_rows(c, dk, dv, rows, key_lo, key_hi, tag):
    """Rows must contain every local row that can see keys [key_lo, key_hi)."""
    _, rdk, rdv = oat.attn_bwd(c.f64("q")[rows], c.f64("k"), c.f64("v"), c.f64("do")[rows], c.q_idx[rows], c.cu_k,
                               c.scale)
    check_close(f"dK {tag}", dk[key_lo:key_hi], rdk[key_lo:key_hi])
    check_close(f"dV {tag}", dv[key_lo:key_hi], rdv[key_lo:key_hi])


def _check_identities(c, dq, dk, dv):
    real = c.q_idx >= 0
    cu = c.cu_k
    g = c.hq // c.hkv
    do = c.f64("do")
    doc = np.searchsorted(cu, c.q_idx[real], side="right") - 1
    # rows of P sum to one  =>  column sums of dV over a document equal the sums of dO
    for d in np.unique(doc):
        rows = np.nonzero(real)[0][doc == d]
        want = do[rows].reshape(len(rows), c.hkv, g, c.d).sum(axis=(0, 2))
        got = dv[cu[d]:cu[d + 1]].sum(axis=0)
        scale = max(np.abs(want).max(), 1.0)
        assert np.abs(got - want).max() / scale < 2e-2, f"dV column sums, document {d}"
    lhs = float((c.f64("q")[real] * dq[real]).sum())
    rhs = float((c.f64("k") * dk).sum())
    assert abs(lhs - rhs) <= 2e-2 * max(abs(lhs), abs(rhs), 1.0), (lhs, rhs)
    # keys that no local row can see get exactly zero
    seen = np.zeros(c.t_kv, dtype=bool)
    for d in np.unique(doc):
        rows = c.q_idx[np.nonzero(real)[0][doc == d]]
        seen[cu[d]:rows.max() + 1] = True
    assert (dk[~seen] == 0).all() and (dv[~seen] == 0).all()


def _full_size_case(cfg, rank, mode):
    w = wl.config(cfg)
    tens = w.tensors()
    sh = B.wlb_shard(w.doc_len, w.cp, rank, mode)
    return w, Case(tens, sh["q_idx"], sh["cu_seqlens_k"], w.hq, w.hkv, w.head_dim, w.scale)


@pytest.mark.parametrize("rank,mode", [(0, B.SHARD_PER_DOC_PADDED), (5, B.SHARD_PER_DOC_PADDED), (7, B.SHARD_PER_SEQ)])
def test_config2_128k_cp8_rank(rank, mode):
    w, c = _full_size_case(2, rank, mode)
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rng = np.random.default_rng(rank)
    rows = _rows_sample(c.q_idx, c.cu_k, 40, rng)
    _check_rows(c, o, lse, dq, rows, f"rank {rank}")
    if (c.q_idx < 0).any():
        pad = c.q_idx < 0
        assert (o[pad] == 0).all() and (dq[pad] == 0).all() and np.isneginf(lse[:, pad]).all()
    # dK/dV: every short document whole, and the last 512 keys of the longest one
    cu = c.cu_k
    real = np.nonzero(c.q_idx >= 0)[0]
    doc = np.searchsorted(cu, c.q_idx[real], side="right") - 1
    for d in np.unique(doc):
        L = cu[d + 1] - cu[d]
        rows_d = real[doc == d]
        if L <= 4096:
            _check_dkv_for_rows(c, dk, dv, rows_d, cu[d], cu[d + 1], f"document {d}")
        else:
            lo = cu[d + 1] - 512
            tail = rows_d[c.q_idx[rows_d] >= lo]
            if len(tail):
                _check_dkv_for_rows(c, dk, dv, tail, lo, cu[d + 1], f"tail of document {d}")
    _check_identities(c, dq, dk, dv)


@pytest.mark.parametrize("rank,mode", [(1, B.SHARD_PER_DOC_PADDED), (0, B.SHARD_PER_DOC_NOPAD)])
def test_config5_64k_mha_cp2_rank(rank, mode):
    # the 64K context window of the paper's evaluation (Section 6.1), multi-head attention (hq = hkv = 8)
    w, c = _full_size_case(5, rank, mode)
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rows = _rows_sample(c.q_idx, c.cu_k, 24, np.random.default_rng(50 + rank))
    _check_rows(c, o, lse, dq, rows, f"c5 rank {rank}")
    cu = c.cu_k
    real = np.nonzero(c.q_idx >= 0)[0]
    doc = np.searchsorted(cu, c.q_idx[real], side="right") - 1
    checked = 0
    for d in np.unique(doc):
        if cu[d + 1] - cu[d] <= 1024 and checked < 12:
            _check_dkv_for_rows(c, dk, dv, real[doc == d], cu[d], cu[d + 1], f"document {d}")
            checked += 1
    _check_identities(c, dq, dk, dv)


def test_config1_32k_gqa():
    w, c = _full_size_case(1, 0, B.SHARD_PER_DOC_PADDED)
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rows = _rows_sample(c.q_idx, c.cu_k, 24, np.random.default_rng(1))
    _check_rows(c, o, lse, dq, rows, "c1")
    cu = c.cu_k
    for d in range(len(cu) - 1):
        L = cu[d + 1] - cu[d]
        if L <= 1024:
            _check_dkv_for_rows(c, dk, dv, np.arange(cu[d], cu[d + 1]), cu[d], cu[d + 1], f"document {d}")
    _check_identities(c, dq, dk, dv)


@pytest.mark.parametrize("cp", [1, 4])
def test_config4_tiny_document_tail(cp):
    """The straggler config's 32768-token tail of 1..64-token documents as its own sequence:
    small enough for a complete oracle pass, and the regime where many documents share a tile."""
    w = wl.config(4)
    docs = w.doc_len[1:]
    assert docs.sum() == 32768
    rng = np.random.default_rng(w.tensor_seed)
    tens = {n: wl.normal_bf16(rng, (32768, h, w.head_dim)) for n, h in (("q", w.hq), ("k", w.hkv), ("v", w.hkv), ("do", w.hq))}
    for rank in sorted({0, cp - 1}):
        sh = B.wlb_shard(docs, cp, rank, B.SHARD_PER_DOC_PADDED)
        c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], w.hq, w.hkv, w.head_dim, w.scale)
        c.check_fwd(f" cp {cp} rank {rank}")
        c.check_bwd(f" cp {cp} rank {rank}")


@pytest.mark.parametrize("cp,flags", [(1, 0), (4, 0), (4, B.ATTN_SCHEDULE_GANGS)])
def test_config4_straggler_full(cp, flags):
    """flags = 0: the schedule the library picks for this shape (one workgroup per tile and head);
    the gang schedule is forced once as well, so that tiles of a 98K-token document are cut and
    merged at full size with 8 query heads per KV head."""
    w = wl.config(4)
    tens = w.tensors()
    sh = B.wlb_shard(w.doc_len, cp, cp - 1, B.SHARD_PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], w.hq, w.hkv, w.head_dim, w.scale)
    c.flags = flags
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rng = np.random.default_rng(4)
    real = np.nonzero(c.q_idx >= 0)[0]
    rows = np.unique(np.concatenate([rng.choice(real, 48, replace=False), real[:3], real[-3:]]))
    _check_rows(c, o, lse, dq, rows, f"cp {cp}")
    # tiny documents after the long one: whole; long document: its last 256 keys
    cu = c.cu_k
    tiny = real[c.q_idx[real] >= cu[1]]
    sel = tiny[c.q_idx[tiny] < cu[1] + 4096]
    _check_dkv_for_rows(c, dk, dv, sel, cu[1], int(cu[np.searchsorted(cu, cu[1] + 4096, side="right") - 1]), "tiny documents")
    lo = cu[1] - 256
    tail = real[(c.q_idx[real] >= lo) & (c.q_idx[real] < cu[1])]
    _check_dkv_for_rows(c, dk, dv, tail, lo, cu[1], "tail of the long document")
    _check_identities(c, dq, dk, dv)


def test_config3_pack_then_attention():
    """The document pool streamed through the packer (global batches of 8 windows, left-overs
    carried forward); the heaviest micro-batch of the first iteration runs forward+backward."""
    w = wl.config(3)
    a, b = 6, 640000
    seqs = opk.pack_fixed_arrival(w.doc_len, 131072)
    docs = np.asarray(sum(seqs[:8], []), dtype=np.int32)
    assign, mb_len, mb_cost = B.wlb_pack(docs, 8, 131072, a, b)
    want = opk.pack(docs, 8, 131072, a, b)
    assert assign.tolist() == list(want[0]) and mb_cost.tolist() == list(want[2])
    assert mb_len.max() <= 131072
    j = int(np.argmax(mb_cost))
    mb_docs = docs[assign == j]
    t = int(mb_docs.sum())
    rng = np.random.default_rng(w.tensor_seed)
    tens = {n: wl.normal_bf16(rng, (t, h, w.head_dim)) for n, h in (("q", w.hq), ("k", w.hkv), ("v", w.hkv), ("do", w.hq))}
    sh = B.wlb_shard(mb_docs, 1, 0, B.SHARD_PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], w.hq, w.hkv, w.head_dim, w.scale)
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rows = _rows_sample(c.q_idx, c.cu_k, 16, np.random.default_rng(3))
    _check_rows(c, o, lse, dq, rows, "micro-batch")
    # dK/dV element by element: every document of up to 4096 tokens whole (at CP = 1 a document's keys are
    # seen by its own rows only), and the last 512 keys of the longer ones
    cu = c.cu_k
    for dd in range(len(cu) - 1):
        L = cu[dd + 1] - cu[dd]
        lo = cu[dd] if L <= 4096 else cu[dd + 1] - 512
        _check_dkv_for_rows(c, dk, dv, np.arange(lo, cu[dd + 1]), lo, cu[dd + 1], f"document {dd}")
    _check_identities(c, dq, dk, dv)


def _dkv_item_table(c):
    """(items per key tile, stages per item) of the dK/dV schedule in the case's workspace."""
    lay = B.wlb_attn_plan_layout(c.attn.desc)
    ws = c.attn.workspace.cpu().numpy()
    arr = lambda off, n: ws[off:off + 4 * n].view(np.int32)
    ways = arr(lay.off_key_ways, lay.n_key_tiles)
    krange = arr(lay.off_key_range, 2 * lay.n_key_tiles).reshape(-1, 2)
    stages = (krange[:, 1] - krange[:, 0]) * ((c.hq // c.hkv) // ways)
    return ways, stages


@pytest.mark.parametrize("docs,cp,rank,min_stages", [([20480, 900, 37, 3000, 1], 2, 0, 150), ([700, 12288, 5, 2100], 1, 0, 150)])
def test_whole_long_document_every_gradient_element(docs, cp, rank, min_stages):
    """Every element of dQ, dK and dV of a long document against the oracle, at head_dim 128 with 8 query
    heads per KV head.  The document is long enough that its key tiles are divided by heads into 2, 4 and 8
    dK/dV work items (fp32 partial results summed by the fix-up pass) and that an item streams more than 150
    stages (row group x head) through the three stage buffers; both work schedules of the forward / dQ kernels run."""
    hq, hkv, d = 8, 1, 128
    w, tens = wl.small_case(131, docs, hq, hkv, d)
    sh = B.wlb_shard(np.asarray(docs, dtype=np.int32), cp, rank, B.SHARD_PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], hq, hkv, d, w.scale)
    real = c.q_idx >= 0
    rows = _rows_sample(c.q_idx, c.cu_k, 64, np.random.default_rng(131))
    ref = None
    for flags in (B.ATTN_SCHEDULE_GANGS, B.ATTN_SCHEDULE_ITEMS):
        c.flags = flags
        o, lse = c.run_fwd()
        dq, dk, dv = c.run_bwd()
        if ref is None:
            ways, stages = _dkv_item_table(c)
            assert {2, 4, 8} <= set(ways.tolist()), "the key tiles of this input must be split 2, 4 and 8 ways"
            assert stages[ways > 1].max() > min_stages, "a split item must stream more than 150 stages"
            ref = c.oracle_bwd()
        _check_rows(c, o, lse, None, rows, f"flags {flags}")
        check_close(f"dQ flags {flags}", dq, ref[0], rows=real)
        check_close(f"dK flags {flags}", dk, ref[1])
        check_close(f"dV flags {flags}", dv, ref[2])
        # per key tile as well: an error confined to one work item must not hide in the tensor-wide mean
        for name, got, want in (("dK", dk, ref[1]), ("dV", dv, ref[2])):
            scale = np.abs(want).max()
            err = np.abs(got - want).reshape(len(got), -1)
            tile_mean = np.add.reduceat(err.mean(axis=1), np.arange(0, len(got), 128)) / 128
            assert tile_mean.max() / scale <= 2e-3, f"{name}: key tile {int(tile_mean.argmax())} mean err {tile_mean.max() / scale:.3e}"
        assert (dq[~real] == 0).all()


def test_tensors_close_to_the_4gib_limit():
    """Q, dO, O and dQ of 3.75 GiB each (122880 rows x 128 heads x 128): the kernels address tensors
    with 32-bit offsets, so rows on both sides of the 2 GiB mark and at the very end are compared
    with the oracle.  480 documents of 256 tokens keep the arithmetic small; each sampled document is
    a self-contained problem (CP = 1), so the oracle runs on it alone."""
    import torch
    n_docs, doc, hq, hkv, d = 480, 256, 128, 16, 128
    t = n_docs * doc
    scale = 1.0 / float(np.sqrt(d))
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(4096)
    mk = lambda n, h: torch.randn((n, h, d), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    k, v = mk(t, hkv), mk(t, hkv)
    q = torch.empty((t, hq, d), dtype=torch.bfloat16, device=dev)
    do = torch.empty_like(q)
    for r0 in range(0, t, 8192):                     # in pieces: no 7.5 GiB fp32 temporary
        q[r0:r0 + 8192] = mk(min(8192, t - r0), hq)
        do[r0:r0 + 8192] = mk(min(8192, t - r0), hq)
    assert q.numel() * 2 > 3.7 * 2**30
    cu = (np.arange(n_docs + 1) * doc).astype(np.int32)
    attn = B.Attention(np.arange(t, dtype=np.int32), cu, t, hq, hkv, d, scale)
    o, lse = attn.forward(q, k, v)
    dq, dk, dv = attn.backward(q, k, v, o, lse, do)
    torch.cuda.synchronize()
    f64 = lambda x: x.double().cpu().numpy()
    # 2 GiB / 32 KiB per row = row 65536 = first row of document 256
    for i in (0, 255, 256, 300, n_docs - 1):
        a, b = i * doc, (i + 1) * doc
        qi, cui = np.arange(doc, dtype=np.int32), np.array([0, doc], dtype=np.int32)
        args = (f64(q[a:b]), f64(k[a:b]), f64(v[a:b]))
        ro, rlse = oat.attn_fwd(*args, qi, cui, scale)
        check_close(f"O document {i}", f64(o[a:b]), ro)
        assert np.abs(f64(lse[:, a:b]) - rlse).max() <= LSE_ABS
        rdq, rdk, rdv = oat.attn_bwd(*args, f64(do[a:b]), qi, cui, scale)
        check_close(f"dQ document {i}", f64(dq[a:b]), rdq)
        check_close(f"dK document {i}", f64(dk[a:b]), rdk)
        check_close(f"dV document {i}", f64(dv[a:b]), rdv)
    # nothing anywhere is left unwritten or non-finite
    for name, x in (("O", o), ("dQ", dq), ("dK", dk), ("dV", dv)):
        assert bool(torch.isfinite(x.view(-1)[::257].float()).all()), name


@pytest.mark.parametrize("flags", [0, B.ATTN_SCHEDULE_GANGS])
def test_half_million_token_document(flags):
    """A 500000-token document (4x the benchmark's window), CP=4, rank 0 (first and last chunk of
    every document): thousands of key tiles per query tile, work lines of millions of units."""
    docs = [500000, 24288]
    w, tens = wl.small_case(91, docs, 2, 1, 64)
    sh = B.wlb_shard(np.asarray(docs, dtype=np.int32), 4, 0, B.SHARD_PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], 2, 1, 64, w.scale)
    c.flags = flags
    o, lse = c.run_fwd()
    dq, dk, dv = c.run_bwd()
    rows = _rows_sample(c.q_idx, c.cu_k, 24, np.random.default_rng(9))
    _check_rows(c, o, lse, dq, rows, "500K")
    cu = c.cu_k
    for d in range(2):
        lo = cu[d + 1] - 512
        tail = np.nonzero((c.q_idx >= lo) & (c.q_idx < cu[d + 1]))[0]
        assert len(tail)
        _check_dkv_for_rows(c, dk, dv, tail, lo, cu[d + 1], f"tail of document {d}")
    _check_identities(c, dq, dk, dv)
