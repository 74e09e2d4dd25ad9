"""GPU parity tests (run with -m gpu): the HIP path through the C ABI against the fp64
oracle, element by element, on seeded inputs that span several tiles and ragged tails."""
import numpy as np
import pytest

from oracle import shard as osh
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl
from gpu_helpers import Case, check_close

pytestmark = pytest.mark.gpu


def _cu(docs):
    return np.concatenate([[0], np.cumsum(docs)]).astype(np.int32)


def _small(seed, docs, hq, hkv, d, cp=1, rank=0, mode=0):
    w, tens = wl.small_case(seed, docs, hq, hkv, d)
    sh = osh.shard(docs, cp, rank, mode)
    return Case(tens, sh["q_idx"], sh["cu_seqlens_k"], hq, hkv, d, w.scale)


FWD_CASES = [
    # docs, hq, hkv, d, cp
    ([300, 45, 1, 700, 130], 4, 2, 128, 1),        # several tiles, ragged tail, 1-token document
    ([64, 64, 128], 2, 2, 64, 1),                  # tile-aligned documents, head_dim 64
    ([1] * 70, 2, 1, 128, 1),                      # only single-token documents
    ([1000], 8, 1, 128, 1),                        # one document, GQA 8:1
    ([3], 1, 1, 64, 1),                            # fewer rows than a tile
    ([5, 900, 2, 3, 333, 64, 1, 77], 4, 4, 64, 2), # per-document sharding with padding
    ([517, 3, 40, 1200], 8, 2, 128, 4),            # documents shorter than 2*CP chunks -> empty chunks
]


@pytest.mark.parametrize("docs,hq,hkv,d,cp", FWD_CASES)
def test_forward_matches_oracle(docs, hq, hkv, d, cp):
    for r in range(cp):
        c = _small(20 + r, docs, hq, hkv, d, cp, r, osh.PER_DOC_PADDED)
        c.check_fwd(f" rank {r}")


def test_forward_per_sequence_sharding():
    docs = [700, 41, 3, 1000, 304]        # T = 2048, divisible by 2*CP
    for r in range(4):
        c = _small(31, docs, 4, 1, 128, 4, r, osh.PER_SEQ)
        c.check_fwd(f" rank {r}")


def test_forward_all_padding_rows():
    w, tens = wl.small_case(5, [40], 2, 1, 64)
    c = Case(tens, np.full(70, -1, dtype=np.int32), _cu([40]), 2, 1, 64, w.scale)
    o, lse = c.run_fwd()
    assert (o == 0).all() and np.isneginf(lse).all()


def test_out_of_range_row_indices_are_padding():
    """q_idx entries outside [0, t_kv) other than -1 are treated like -1 (stated in the header)."""
    import torch
    docs = [200, 57, 1]
    t = sum(docs)
    w, tens = wl.small_case(33, docs, 2, 1, 64)
    clean = np.arange(t, dtype=np.int32)
    bad = np.array([3, 64, 199, 200, 256, 257], dtype=np.int64)
    clean[bad] = -1
    c = Case(tens, clean, _cu(docs), 2, 1, 64, w.scale)
    dirty = clean.copy()
    dirty[bad] = np.array([-5, t, t + 1000, 2**31 - 1, -2**31, -2], dtype=np.int64).astype(np.int32)
    c.attn.q_idx.copy_(torch.from_numpy(dirty))
    c.check_fwd()
    c.check_bwd()


def test_one_token():
    for d in (64, 128):
        c = _small(34, [1], 1, 1, d)
        o, lse = c.run_fwd()
        assert np.array_equal(o[0, 0], c.f64("v")[0, 0])          # a one-token document returns its own V
        c.check_fwd()
        c.check_bwd()


def test_forward_rows_in_arbitrary_order():
    # the mask is per row; nothing requires q_idx to be sorted
    docs = [200, 333, 90]
    w, tens = wl.small_case(6, docs, 2, 2, 128)
    rng = np.random.default_rng(0)
    q_idx = rng.permutation(sum(docs)).astype(np.int32)[:400]
    q_idx[::17] = -1
    Case(tens, q_idx, _cu(docs), 2, 2, 128, w.scale).check_fwd()


@pytest.mark.parametrize("flag", [B.ATTN_SCHEDULE_GANGS, B.ATTN_SCHEDULE_ITEMS])
def test_wavefront_with_rows_of_two_chunks_and_three_documents(flag):
    """32 consecutive rows (one wavefront of the forward and dQ kernels) that hold rows of an early and of a late
    chunk of one long document, rows of a second document and a row of a third, padding in between: the kernels
    cross the keys between the chunks, and the other documents' keys, with whole lanes switched off, in several
    ranges.  Every output element against the oracle, forward and backward."""
    docs = [2000, 700, 300, 77]
    cu = _cu(docs)
    rows = ([int(cu[0]) + i for i in range(0, 9)] + [-1, -1] + [int(cu[0]) + 1900 + i for i in range(7)]
            + [int(cu[1]) + 130 + 3 * i for i in range(8)] + [-1] + [int(cu[2]) + 299] + [int(cu[1]) + 699, int(cu[1]), -1, int(cu[0]) + 1999])
    assert len(rows) == 32
    # a second wavefront of ordinary rows and a third that starts in the last document
    rows += [int(cu[0]) + 640 + i for i in range(32)] + [int(cu[3]) + i for i in range(20)]
    w, tens = wl.small_case(97, docs, 8, 2, 128)
    c = Case(tens, np.asarray(rows, dtype=np.int32), cu, 8, 2, 128, w.scale)
    c.flags = flag
    c.check_fwd(" mixed wavefront")
    c.check_bwd(" mixed wavefront")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_match_oracle(seed):
    """A seeded sweep over valid small inputs: document mixes (tiny, mixed, one long plus tiny, medium), head counts
    with groups of 1 to 8 query heads per KV head, both head dimensions, CP 1 to 4 with padded and padding-free maps,
    every schedule flag, and for some cases shuffled rows with extra padding.  Forward and backward, every element."""
    rng = np.random.default_rng(seed)
    for it in range(25):
        n_docs = int(rng.integers(1, 12))
        kind = int(rng.integers(0, 4))
        if kind == 0:
            docs = rng.integers(1, 70, size=n_docs * 6).tolist()
        elif kind == 1:
            docs = rng.integers(1, 1500, size=n_docs).tolist()
        elif kind == 2:
            docs = [int(rng.integers(1500, 4000))] + rng.integers(1, 100, size=n_docs).tolist()
        else:
            docs = rng.integers(100, 700, size=n_docs).tolist()
        if sum(docs) > 6000:
            docs = docs[:max(1, len(docs) // 2)]
        hkv = int(rng.choice([1, 2, 3, 4]))
        hq = hkv * int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
        if hq > 16:
            hq, hkv = 8, 2
        d = int(rng.choice([64, 128]))
        cp = int(rng.choice([1, 1, 2, 3, 4]))
        rank = int(rng.integers(0, cp))
        mode = int(rng.choice([osh.PER_DOC_PADDED, osh.PER_DOC_NOPAD])) if cp > 1 else osh.PER_DOC_PADDED
        flag = int(rng.choice([0, B.ATTN_SCHEDULE_GANGS, B.ATTN_SCHEDULE_ITEMS, B.ATTN_SCHEDULE_ITEMS | B.ATTN_NO_SHORT_PATH]))
        tag = f" seed {seed} case {it}: docs {docs} hq {hq} hkv {hkv} d {d} cp {cp} rank {rank} mode {mode} flag {flag}"
        w, tens = wl.small_case(1000 * seed + it, docs, hq, hkv, d)
        sh = osh.shard(docs, cp, rank, mode)
        q_idx = sh["q_idx"].copy()
        if rng.random() < 0.3 and len(q_idx) > 4:
            q_idx = rng.permutation(q_idx)
            q_idx[rng.integers(0, len(q_idx), size=max(1, len(q_idx) // 10))] = -1
        c = Case(tens, q_idx, sh["cu_seqlens_k"], hq, hkv, d, w.scale)
        c.flags = flag
        c.check_fwd(tag)
        c.check_bwd(tag)


def test_forward_config0_both_ranks():
    w = wl.config(0)
    tens = w.tensors(names=("q", "k", "v"))
    for r in range(2):
        sh = B.wlb_shard(w.doc_len, 2, r, B.SHARD_PER_DOC_PADDED)
        Case(tens, sh["q_idx"], sh["cu_seqlens_k"], w.hq, w.hkv, w.head_dim, w.scale).check_fwd(f" rank {r}")


def test_forward_is_deterministic_and_plan_reuse_changes_nothing():
    c = _small(40, [900, 50, 400], 4, 2, 128)
    o1, l1 = c.run_fwd()
    o2, l2 = c.run_fwd()              # second call reuses the schedule in the workspace
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (6, 2, 64), (12, 1, 128), (3, 3, 64), (16, 1, 128), (32, 2, 64)])
@pytest.mark.parametrize("flag", [B.ATTN_SCHEDULE_GANGS, B.ATTN_SCHEDULE_ITEMS])
def test_both_row_schedules_match_oracle(flag, hq, hkv, d):
    """Forward and dQ have two work schedules (fixed gangs with tiles cut at share ends and merged
    from partial results / one workgroup per tile and head); both forced here on an input with
    documents from 1 token to several tiles, pads, and tiles that straddle documents, for head
    groups of 1, 2, 3, 12 and 16 query heads per KV head and both head dimensions."""
    docs = [900, 1, 37, 2600, 130, 64, 700]
    w, tens = wl.small_case(77, docs, hq, hkv, d)
    for cp, r in ((1, 0), (2, 1)):
        sh = osh.shard(docs, cp, r, osh.PER_DOC_PADDED)
        c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], hq, hkv, d, w.scale)
        c.flags = flag
        c.check_fwd(f" cp {cp} rank {r}")
        c.check_bwd(f" cp {cp} rank {r}")


def test_gang_share_weights_change_the_cuts_not_the_result():
    """wlb_attn_set_gang_weights: very uneven weights (by half of the launch and by XCD) move the points where
    query tiles are cut between gangs; the results still match the oracle, and the defaults come back."""
    docs = [2600, 1, 37, 900, 130, 64, 700]
    w, tens = wl.small_case(79, docs, 8, 1, 128)
    sh = osh.shard(docs, 2, 1, osh.PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], 8, 1, 128, w.scale)
    c.flags = B.ATTN_SCHEDULE_GANGS
    o0, _ = c.run_fwd()
    try:
        B.wlb_attn_set_gang_weights(0, [100, 5, 60, 1000, 7, 300, 90, 33, 11, 250, 40, 40, 900, 2, 75, 120])
        B.wlb_attn_set_gang_weights(1, [3, 500, 60, 10, 700, 30, 90, 330, 110, 25, 400, 4, 90, 200, 75, 12])
        c.check_fwd(" uneven weights")
        c.check_bwd(" uneven weights")
        with pytest.raises(B.WlbError):
            B.wlb_attn_set_gang_weights(0, [0] * 16)
        with pytest.raises(B.WlbError):
            B.wlb_attn_set_gang_weights(2, [1] * 16)
    finally:
        B.wlb_attn_set_gang_weights(0, None)
        B.wlb_attn_set_gang_weights(1, None)
    o1, _ = c.run_fwd()
    assert np.array_equal(o0, o1), "default weights restored: same cuts, same bits"


def test_gang_weights_calibrated_from_the_clocks_keep_the_result():
    """binding.calibrate_gang_weights: XCD factors measured from the gangs' recorded clocks on the caller's own
    launches; positive weights in the documented range result, the halves keep their default ratio, and forward
    and backward still match the oracle."""
    docs = [3000, 5, 1200, 64, 333]
    w, tens = wl.small_case(83, docs, 8, 2, 128)
    sh = osh.shard(docs, 1, 0, osh.PER_DOC_PADDED)
    c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], 8, 2, 128, w.scale)
    c.flags = B.ATTN_SCHEDULE_GANGS
    default = [B.wlb_attn_get_gang_weights(k).copy() for k in (0, 1)]
    try:
        def launch():
            c.run_fwd()
            c.run_bwd()
        factors = B.calibrate_gang_weights([c.attn], launch, rounds=2, extra_flags=B.ATTN_SCHEDULE_GANGS)
        assert factors is not None and len(factors["fwd"]) == 8 and len(factors["dq"]) == 8
        for k, name in enumerate(("fwd", "dq")):
            got = B.wlb_attn_get_gang_weights(k).astype(np.float64).reshape(2, 8)
            assert (got >= 1).all() and (got <= 1e6).all()
            f = np.asarray(factors[name])
            assert (f >= 0.8).all() and (f <= 1.25).all()
            want = default[k].astype(np.float64).reshape(2, 8) * f[None, :] * 10.0
            assert np.abs(got - want).max() <= 1.0      # rounding to integers plus the factors' four decimals
        c.check_fwd(" calibrated weights")
        c.check_bwd(" calibrated weights")
        assert B.calibrate_gang_weights([c.attn], launch) is None, "without the flag this problem does not use gangs"
    finally:
        B.wlb_attn_set_gang_weights(0, None)
        B.wlb_attn_set_gang_weights(1, None)
    assert all(np.array_equal(B.wlb_attn_get_gang_weights(k), default[k]) for k in (0, 1))


def test_plan_tables_and_report_describe_the_schedule():
    """binding.plan_tables / plan_report: the host view of the schedule holds the row intervals of the mask's
    definition (document start up to the row itself), orders and running sums that fit together, and the
    text report names the shape and the counts."""
    docs = [700, 3, 1500, 64, 64, 9]
    c = _small(91, docs, 4, 2, 128)
    c.attn.plan()
    t = B.plan_tables(c.attn)
    cu = _cu(docs)
    pos = np.arange(sum(docs))
    start = cu[np.searchsorted(cu, pos, side="right") - 1]
    assert np.array_equal(t["row_lo"], start) and np.array_equal(t["row_hi"], pos + 1)
    lay = t["layout"]
    assert sorted(t["fwd_order"].tolist()) == list(range(lay.n_fwd_tiles))
    assert t["fwd_prefix"][0] == 0 and (np.diff(t["fwd_prefix"]) > 0).all()
    assert int(t["key_item_base"][-1]) == int((t["key_ways"] * 2).sum())
    text = B.plan_report(c.attn, "case")
    assert f"n_q {sum(docs)}" in text and f"{lay.n_fwd_tiles} query tiles" in text and "dK/dV items" in text


def test_gang_schedule_on_one_row():
    """Degenerate work lines: a single query row, and fewer units of work than gangs."""
    for docs in ([1], [5, 1, 2]):
        w, tens = wl.small_case(78, docs, 8, 1, 128)
        sh = osh.shard(docs, 1, 0, osh.PER_DOC_PADDED)
        c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], 8, 1, 128, w.scale)
        c.flags = B.ATTN_SCHEDULE_GANGS
        c.check_fwd(f" docs {docs}")
        c.check_bwd(f" docs {docs}")


SHORT_CASES = [
    # docs, hq, hkv, d, cp: documents of a few dozen tokens, where whole query tiles take the short-hull path
    (list(range(1, 65)) * 2, 16, 2, 128, 1),       # every length 1..64 twice, 8 heads per KV head (two per wavefront)
    ([64] * 9 + [5], 4, 4, 128, 1),                # one head per KV head, last tile ragged
    ([33, 1, 64, 17, 2, 48, 9, 60, 31] * 5, 6, 2, 64, 1),   # three heads per KV head, head_dim 64
    ([40, 7, 64, 23, 12] * 9, 8, 1, 128, 2),       # sharded: pads, and key windows too wide for some tiles
    ([64, 64, 300, 20, 20, 20, 64, 1000, 8, 8], 2, 1, 128, 1),   # short and long tiles in one launch
]


@pytest.mark.parametrize("docs,hq,hkv,d,cp", SHORT_CASES)
def test_short_hull_path_matches_oracle(docs, hq, hkv, d, cp):
    """Tiles whose 32-row blocks each see at most 96 keys run as short-hull units inside the
    one-workgroup-per-item launches (forward, dQ with its own delta).  The schedule must mark them,
    the results must match the oracle, and switching the path off must change nothing beyond rounding."""
    import torch
    w, tens = wl.small_case(90, docs, hq, hkv, d)
    for r in sorted({0, cp - 1}):
        sh = osh.shard(docs, cp, r, osh.PER_DOC_PADDED)
        c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], hq, hkv, d, w.scale)
        c.flags = B.ATTN_SCHEDULE_ITEMS
        c.check_fwd(f" short rank {r}")
        c.check_bwd(f" short rank {r}")
        lay = B.wlb_attn_plan_layout(c.attn.desc)
        ws = c.attn.workspace.cpu().numpy()
        hull = ws[lay.off_block_hull:lay.off_block_hull + 8 * lay.n_blocks32].view(np.int32).reshape(-1, 2)
        short = ws[lay.off_tile_short:lay.off_tile_short + 4 * lay.n_fwd_tiles].view(np.int32)
        lo, hi = (ws[o:o + 4 * len(c.q_idx)].view(np.int32) for o in (lay.off_row_lo, lay.off_row_hi))
        want_short = []
        for t in range(lay.n_fwd_tiles):
            ok = True
            for b in range(4 * t, min(4 * t + 4, lay.n_blocks32)):
                rows = slice(32 * b, min(32 * b + 32, len(c.q_idx)))
                real = hi[rows] > 0
                if real.any():
                    assert hull[b, 0] == lo[rows][real].min() and hull[b, 1] == hi[rows][real].max()
                    ok &= hull[b, 1] - (hull[b, 0] // 32) * 32 <= 96
                else:
                    assert hull[b, 1] <= hull[b, 0]
            want_short.append(int(ok))
        assert short.tolist() == want_short
        if cp == 1:
            assert sum(want_short) > 0, "this input is meant to exercise the short-hull path"
        o1, l1 = c.run_fwd()
        g1 = c.run_bwd()
        c.flags = B.ATTN_SCHEDULE_ITEMS | B.ATTN_NO_SHORT_PATH
        o2, l2 = c.run_fwd()
        g2 = c.run_bwd()
        real = c.q_idx >= 0
        check_close("O short vs general", o1, o2, rows=real)
        for name, a, b in zip(("dQ", "dK", "dV"), g1, g2):
            check_close(f"{name} short vs general", a, b)


ROW_ITEM_OVERHEAD = 6     # units of fixed cost per query tile in the forward / dQ work line
DKV_SPLIT = 6             # a dK/dV item is at most 1/DKV_SPLIT of a compute unit's mean load
DKV_MIN_ITEM_STAGES = 32  # items this short are not split further


def test_schedule_tables():
    """The schedule in the workspace: row intervals equal the definition, group hulls cover
    their rows, fully visible ranges are visible to every real row, orders are permutations
    sorted heaviest first, and a key tile's group range covers every group that can see it."""
    import torch
    docs = [517, 3, 40, 1200, 64, 9]
    w, tens = wl.small_case(41, docs, 2, 1, 64)
    for cp, r in ((1, 0), (4, 1)):
        sh = osh.shard(docs, cp, r, osh.PER_DOC_PADDED)
        c = Case(tens, sh["q_idx"], sh["cu_seqlens_k"], 2, 1, 64, w.scale)
        c.attn.plan()
        torch.cuda.synchronize()
        lay = B.wlb_attn_plan_layout(c.attn.desc)
        ws = c.attn.workspace.cpu().numpy()

        def arr(off, n):
            return ws[off:off + 4 * n].view(np.int32)

        n_q = len(c.q_idx)
        lo, hi = arr(lay.off_row_lo, n_q), arr(lay.off_row_hi, n_q)
        cu = c.cu_k
        for i, g in enumerate(c.q_idx):
            if g < 0:
                assert lo[i] > hi[i]
            else:
                d = np.searchsorted(cu, g, side="right") - 1
                assert lo[i] == cu[d] and hi[i] == g + 1
        grp = arr(lay.off_group, 4 * lay.n_groups).reshape(-1, 4)
        for g in range(lay.n_groups):
            rows = slice(g * lay.group_rows, min((g + 1) * lay.group_rows, n_q))
            real = c.q_idx[rows] >= 0
            if not real.any():
                assert grp[g, 1] <= grp[g, 0]
                continue
            assert grp[g, 0] == lo[rows][real].min() and grp[g, 1] == hi[rows][real].max()
            assert grp[g, 2] == lo[rows][real].max() and grp[g, 3] == hi[rows][real].min()
        order = arr(lay.off_fwd_order, lay.n_fwd_tiles)
        cost = arr(lay.off_fwd_cost, lay.n_fwd_tiles)
        assert sorted(order.tolist()) == list(range(lay.n_fwd_tiles))
        assert (np.diff(cost[order]) <= 0).all()
        # forward / dQ work line: running sum, in order, of key tiles + the fixed per-tile cost
        prefix = ws[lay.off_fwd_prefix:lay.off_fwd_prefix + 8 * (lay.n_fwd_tiles + 1)].view(np.int64)
        assert prefix[0] == 0 and (np.diff(prefix) == cost[order] + ROW_ITEM_OVERHEAD).all()
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        assert lay.row_gangs == 8 * max(1, (2 * n_cu // 8) // (c.hq // c.hkv))
        korder = arr(lay.off_key_order, lay.n_key_tiles)
        krange = arr(lay.off_key_range, 2 * lay.n_key_tiles).reshape(-1, 2)
        assert sorted(korder.tolist()) == list(range(lay.n_key_tiles))
        for kt in range(lay.n_key_tiles):
            k0, k1 = kt * lay.bwd_key_tile, min((kt + 1) * lay.bwd_key_tile, c.t_kv)
            sees = [g for g in range(lay.n_groups) if grp[g, 1] > grp[g, 0] and grp[g, 0] < k1 and grp[g, 1] > k0]
            if sees:
                assert krange[kt, 0] == sees[0] and krange[kt, 1] == sees[-1] + 1
            else:
                assert krange[kt, 0] == krange[kt, 1]
        # dK/dV items: a tile is cut by heads into a power-of-two number of items, tiles are ordered by
        # item cost (groups in range x heads per item), heaviest first, and the item / partial-slot
        # bases are the running sums in that order
        ways = arr(lay.off_key_ways, lay.n_key_tiles)
        item_base = arr(lay.off_key_item_base, lay.n_key_tiles + 1)
        slot_base = arr(lay.off_key_slot_base, lay.n_key_tiles + 1)
        g_heads = c.hq // c.hkv
        assert all(w in (1, 2, 4, 8) and g_heads % w == 0 for w in ways.tolist())
        span = krange[:, 1] - krange[:, 0]
        icost = span * (g_heads // ways)
        assert (np.diff(icost[korder]) <= 0).all()
        assert item_base[0] == 0 and slot_base[0] == 0
        assert (np.diff(item_base) == ways[korder] * c.hkv).all()
        assert (np.diff(slot_base) == np.where(ways[korder] > 1, ways[korder] * c.hkv, 0)).all()
        assert item_base[-1] <= lay.dkv_max_items and slot_base[-1] <= lay.dkv_max_partials
        # no item is heavier than the threshold unless it is already a single head
        total = int(span.sum()) * c.hq
        assert (icost[ways < g_heads] <= max(DKV_MIN_ITEM_STAGES, -(-total // (DKV_SPLIT * n_cu)))).all()


def test_schedule_orders_with_thousands_of_tiles():
    """600K tokens: more tiles than one pass of the counting rank holds.  Both orders must be the
    stable sort by cost, heaviest first (ties by index), and the running sums must follow them."""
    import torch
    rng = np.random.default_rng(5)
    docs = [200000, 70001] + rng.integers(1, 3000, size=220).tolist()
    cu = np.concatenate([[0], np.cumsum(docs)]).astype(np.int32)
    t = int(cu[-1])
    attn = B.Attention(np.arange(t, dtype=np.int32), cu, t, 2, 1, 64, 0.125)
    attn.plan()
    torch.cuda.synchronize()
    lay = B.wlb_attn_plan_layout(attn.desc)
    assert lay.n_fwd_tiles > 4096 and lay.n_key_tiles > 4096
    ws = attn.workspace.cpu().numpy()
    arr = lambda off, n: ws[off:off + 4 * n].view(np.int32)
    cost = arr(lay.off_fwd_cost, lay.n_fwd_tiles)
    # a query tile's cost: 64-key tiles from its first row's document start to its last row
    tile_rows = t // lay.n_fwd_tiles + (t % lay.n_fwd_tiles > 0)
    assert tile_rows == 128
    first = np.arange(lay.n_fwd_tiles) * 128
    last = np.minimum(first + 128, t) - 1
    lo = cu[np.searchsorted(cu, first, side="right") - 1]
    assert (cost == (last + 1 + 63) // 64 - lo // 64).all()
    order = arr(lay.off_fwd_order, lay.n_fwd_tiles)
    assert (order == np.lexsort((np.arange(lay.n_fwd_tiles), -cost))).all()
    prefix = ws[lay.off_fwd_prefix:lay.off_fwd_prefix + 8 * (lay.n_fwd_tiles + 1)].view(np.int64)
    assert prefix[0] == 0 and (np.diff(prefix) == cost[order].astype(np.int64) + ROW_ITEM_OVERHEAD).all()
    krange = arr(lay.off_key_range, 2 * lay.n_key_tiles).reshape(-1, 2)
    ways = arr(lay.off_key_ways, lay.n_key_tiles)
    icost = (krange[:, 1] - krange[:, 0]) * (2 // ways)
    korder = arr(lay.off_key_order, lay.n_key_tiles)
    assert (korder == np.lexsort((np.arange(lay.n_key_tiles), -icost))).all()
    item_base = arr(lay.off_key_item_base, lay.n_key_tiles + 1)
    assert item_base[0] == 0 and (np.diff(item_base) == ways[korder]).all()


BWD_CASES = [
    ([300, 45, 1, 700, 130], 4, 2, 128, 1),
    ([64, 64, 128], 2, 2, 64, 1),
    ([1] * 70, 2, 1, 128, 1),
    ([1000], 8, 1, 128, 1),
    ([3], 1, 1, 64, 1),
    ([5, 900, 2, 3, 333, 64, 1, 77], 4, 4, 64, 2),
    ([517, 3, 40, 1200], 8, 2, 128, 4),
]


@pytest.mark.parametrize("docs,hq,hkv,d,cp", BWD_CASES)
def test_backward_matches_oracle(docs, hq, hkv, d, cp):
    for r in range(cp):
        c = _small(50 + r, docs, hq, hkv, d, cp, r, osh.PER_DOC_PADDED)
        c.check_fwd(f" rank {r}")
        c.check_bwd(f" rank {r}")


def test_backward_per_sequence_sharding_and_rank_sum():
    """Per-rank dK/dV partials add up to the unsharded gradient (what the reduce-scatter of
    all-gather context parallelism would deliver)."""
    docs = [700, 41, 3, 1000, 304]
    cp = 4
    full = _small(60, docs, 4, 1, 128)
    full.run_fwd()
    _, rdk, rdv = full.oracle_bwd()
    dk_sum, dv_sum = np.zeros_like(rdk), np.zeros_like(rdv)
    for r in range(cp):
        c = _small(60, docs, 4, 1, 128, cp, r, osh.PER_SEQ)
        c.check_fwd(f" rank {r}")
        c.check_bwd(f" rank {r}")
        _, dk, dv = c.run_bwd()
        dk_sum += dk
        dv_sum += dv
    check_close("sum of dK partials", dk_sum, rdk)
    check_close("sum of dV partials", dv_sum, rdv)


def test_backward_rows_in_arbitrary_order_with_garbage_in_padding():
    docs = [200, 333, 90]
    w, tens = wl.small_case(61, docs, 4, 2, 128)
    rng = np.random.default_rng(1)
    q_idx = rng.permutation(sum(docs)).astype(np.int32)[:400]
    q_idx[::13] = -1
    c = Case(tens, q_idx, _cu(docs), 4, 2, 128, w.scale)
    # padding rows may hold anything, including NaN and Inf bit patterns
    pad = np.nonzero(q_idx < 0)[0]
    for name in ("q", "do"):
        t = c.dev[name].view(dtype=__import__("torch").int16)
        t[pad[0::2]] = 0x7FC0          # NaN
        t[pad[1::2]] = 0x7F80          # +Inf
    c.check_fwd()
    c.check_bwd()


def test_backward_is_deterministic():
    c = _small(62, [900, 50, 400], 4, 2, 128)
    c.run_fwd()
    a = c.run_bwd()
    b = c.run_bwd()
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_padding_free_sharding_forward_backward():
    """Padding-free per-document maps go through the same kernels: the mask is per row."""
    docs = [517, 3, 41, 1203, 66, 9, 217]          # T = 2056 = 8 * 257: every rank gets 514 slots, none padding
    cp = 4
    sizes = set()
    for r in range(cp):
        c = _small(70, docs, 8, 2, 128, cp, r, osh.PER_DOC_NOPAD)
        assert (c.q_idx >= 0).all()
        sizes.add(len(c.q_idx))
        c.check_fwd(f" rank {r}")
        c.check_bwd(f" rank {r}")
    assert sizes == {sum(docs) // cp}


@pytest.mark.parametrize("flag", [0, B.ATTN_SCHEDULE_GANGS])
def test_graph_replay_matches_eager_calls(flag):
    """The library only launches kernels on the caller's stream, so schedule + forward + backward
    can be captured into a HIP graph.  Every replay must reproduce the eager results bit for bit,
    with eager calls and other inputs in between (the workspace is shared and rewritten)."""
    import torch
    c = _small(81, [700, 3, 260, 1, 90], 4, 2, 128)
    other = _small(82, [700, 3, 260, 1, 90], 4, 2, 128)
    a = c.attn
    n_q = len(c.q_idx)
    q, k, v, do = (c.dev[n].clone() for n in ("q", "k", "v", "do"))
    o = torch.empty_like(q)
    lse = torch.empty((c.hq, n_q), dtype=torch.float32, device=q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def step():
        a.plan()
        a.forward(q, k, v, o, lse, extra_flags=flag)
        a.backward(q, k, v, o, lse, do, dq, dk, dv, extra_flags=flag)

    def results():
        torch.cuda.synchronize()
        return [t.clone() for t in (o, lse, dq, dk, dv)]

    step()
    eager = results()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(4):
        for t in (o, lse, dq, dk, dv):
            t.fill_(float("nan"))
        if replay == 2:
            # other inputs through the same graph, then back
            for dst, name in ((q, "q"), (k, "k"), (v, "v"), (do, "do")):
                dst.copy_(other.dev[name])
            graph.replay()
            step()
            for dst, name in ((q, "q"), (k, "k"), (v, "v"), (do, "do")):
                dst.copy_(c.dev[name])
        graph.replay()
        got = results()
        for name, x, y in zip(("O", "LSE", "dQ", "dK", "dV"), got, eager):
            assert torch.equal(x, y), f"{name} differs on replay {replay}"
        step()                                        # eager work between the replays
        for name, x, y in zip(("O", "LSE", "dQ", "dK", "dV"), results(), eager):
            assert torch.equal(x, y), f"{name} differs in the eager call after replay {replay}"
