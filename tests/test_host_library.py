"""CPU tests of the C-ABI library: it loads, exports every declared symbol, and its host
entry points (wlb_pack, wlb_shard) are bit-exact against the oracle, including error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import pack as opk
from oracle import shard as osh
from paper_2503_17924_amd import binding as B
from paper_2503_17924_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wlb.h")).read()
    declared = set(re.findall(r"\b(wlb_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("cp,mode", [(1, 0), (2, 0), (2, 1), (4, 0), (4, 1), (8, 0), (8, 1), (3, 0), (1, 2), (2, 2), (3, 2), (4, 2), (8, 2)])
def test_shard_matches_oracle_random(cp, mode):
    rng = np.random.default_rng(100 * cp + mode)
    for trial in range(6):
        docs = rng.integers(1, 200, size=int(rng.integers(1, 40))).astype(np.int32)
        if mode == 1:
            rem = int(docs.sum()) % (2 * cp)
            if rem:
                docs[-1] += 2 * cp - rem
        for r in range(cp):
            want = osh.shard(docs, cp, r, mode)
            got = B.wlb_shard(docs, cp, r, mode)
            for key in ("q_idx", "cu_seqlens_q", "seg_k_begin", "seg_k_end", "cu_seqlens_k"):
                assert got[key].dtype == np.int32
                assert got[key].tolist() == want[key].tolist(), key
            assert got["useful_pairs"] == want["useful_pairs"]


@pytest.mark.parametrize("cfg,cp,modes", [(0, 2, (0, 1, 2)), (2, 8, (0, 1, 2)), (4, 4, (0, 1, 2)), (1, 1, (0,))])
def test_shard_matches_oracle_on_benchmark_configs(cfg, cp, modes):
    w = wl.config(cfg)
    for mode in modes:
        for r in sorted({0, cp - 1, cp // 2}):
            want = osh.shard(w.doc_len, cp, r, mode)
            got = B.wlb_shard(w.doc_len, cp, r, mode)
            for key in ("q_idx", "cu_seqlens_q", "seg_k_begin", "seg_k_end", "cu_seqlens_k"):
                assert np.array_equal(got[key], want[key]), key
            assert got["useful_pairs"] == want["useful_pairs"]


def test_shard_errors():
    for args in (([4, 0], 2, 0, 0), ([4], 2, 2, 0), ([5], 2, 0, 1), ([4], 0, 0, 0), ([4], 2, 0, 7), ([4], 2, -1, 0)):
        with pytest.raises(B.WlbError) as e:
            B.wlb_shard(np.asarray(args[0], dtype=np.int32), *args[1:])
        assert e.value.status == 1
    with pytest.raises(B.WlbError) as e:
        B.wlb_shard(np.full(3, 2**30, dtype=np.int32), 2, 0, 0)
    assert e.value.status == 3


def test_pack_matches_oracle_random():
    rng = np.random.default_rng(42)
    for trial in range(40):
        n = int(rng.integers(0, 120))
        docs = rng.integers(1, 5000, size=n).astype(np.int32)
        nmb = int(rng.integers(1, 9))
        l_max = int(rng.integers(4000, 40000))
        a, b = int(rng.integers(0, 50)), int(rng.integers(0, 10**6))
        want = opk.pack(docs, nmb, l_max, a, b)
        got = B.wlb_pack(docs, nmb, l_max, a, b)
        assert got[0].tolist() == list(want[0])
        assert got[1].tolist() == list(want[1])
        assert got[2].tolist() == list(want[2])


def test_pack_matches_oracle_on_the_document_pool():
    w = wl.config(3)
    a, b = 6, 640000
    want = opk.pack(w.doc_len, 8, 131072, a, b)
    got = B.wlb_pack(w.doc_len, 8, 131072, a, b)
    assert got[0].tolist() == list(want[0])
    assert got[1].tolist() == list(want[1]) and got[2].tolist() == list(want[2])
    # streamed as Algorithm 1's outer loop: global batches of 8 windows, left-overs carried over
    seqs = opk.pack_fixed_arrival(w.doc_len, 131072)
    batches = [sum(seqs[i:i + 8], []) for i in range(0, len(seqs), 8)]
    remained = []
    for cur in batches[:6]:
        docs = np.asarray(remained + cur, dtype=np.int32)
        want = opk.pack(docs, 8, 131072, a, b)
        got = B.wlb_pack(docs, 8, 131072, a, b)
        assert got[0].tolist() == list(want[0])
        assert got[2].tolist() == list(want[2])
        remained = [int(d) for d, j in zip(docs, want[0]) if j < 0]


def test_pack_errors_and_limits():
    d = np.asarray([3, 4], dtype=np.int32)
    for args in ((d, 0, 10, 1, 1), (d, 2, 0, 1, 1), (np.asarray([3, 0], dtype=np.int32), 2, 10, 1, 1)):
        with pytest.raises(B.WlbError) as e:
            B.wlb_pack(*args)
        assert e.value.status == 1
    with pytest.raises(B.WlbError):
        B.wlb_pack(d, 2, 2**40, 2**20, 0)           # a * l_max^2 overflows 64 bits
    # largest admissible costs stay exact
    got = B.wlb_pack(np.asarray([2**18], dtype=np.int32), 1, 2**18, 2**24, 2**40)
    assert int(got[2][0]) == 2**24 * 2**36 + 2**40 * 2**18
    # a document longer than l_max is left over
    assert B.wlb_pack(np.asarray([11, 5], dtype=np.int32), 2, 10, 1, 0)[0].tolist() == [-1, 0]


def test_schedule_choice_uses_the_pair_count_when_given():
    """One rank of a 128K micro-batch made of one long document among 500 tiny ones: 128 query tiles x 8 heads are
    few items per workgroup slot, and nearly all work sits in the long document's tiles.  From the mean document
    length alone the host takes the work for small and picks one workgroup per item; with the rank's pair count
    (wlb_shard's useful_pairs) in the descriptor it picks the gang schedule, as it does for a few long documents.
    With many items per slot it is one workgroup per item either way; a negative count is an error."""
    docs = np.asarray([100000] + [62] * 500 + [72], dtype=np.int32)
    assert docs.sum() == 131072
    sh = B.wlb_shard(docs, 8, 3, B.SHARD_PER_DOC_PADDED)
    n_q, pairs = len(sh["q_idx"]), sh["useful_pairs"]
    assert pairs > 5e8
    blind = B.wlb_attn_plan_layout(B._desc(n_q, 131072, len(docs), 8, 1, 128, 0.1))
    told = B.wlb_attn_plan_layout(B._desc(n_q, 131072, len(docs), 8, 1, 128, 0.1, visible_pairs=pairs))
    assert (blind.uses_gangs, told.uses_gangs) == (0, 1)
    assert B.wlb_attn_plan_layout(B._desc(n_q, 131072, 16, 8, 1, 128, 0.1)).uses_gangs == 1
    assert B.wlb_attn_plan_layout(B._desc(131072, 131072, len(docs), 16, 2, 128, 0.1, visible_pairs=8 * pairs)).uses_gangs == 0
    assert B.wlb_attn_plan_layout(B._desc(n_q, 131072, len(docs), 8, 1, 128, 0.1, flags=B.ATTN_SCHEDULE_ITEMS,
                                          visible_pairs=pairs)).uses_gangs == 0
    with pytest.raises(B.WlbError):
        B.wlb_attn_plan_layout(B._desc(n_q, 131072, len(docs), 8, 1, 128, 0.1, visible_pairs=-1))


def test_attention_argument_checks_need_no_gpu():
    d = B._desc(128, 128, 1, 4, 3, 128, 0.1)
    with pytest.raises(B.WlbError) as e:
        B.wlb_attn_workspace_size(d)
    assert e.value.status == 1
    d = B._desc(128, 128, 1, 4, 2, 96, 0.1)
    with pytest.raises(B.WlbError) as e:
        B.wlb_attn_workspace_size(d)
    assert e.value.status == 3
    # tensors are addressed with 32-bit offsets: Q [n_q][hq][D] bf16 must stay under 4 GiB, tile tail included
    for n_q, ok in ((131072 - 129, True), (131072 - 128, False), (131072, False)):
        d = B._desc(n_q, 4096, 1, 128, 128, 128, 0.1)          # 32 KiB per row
        if ok:
            B.wlb_attn_workspace_size(d)
        else:
            with pytest.raises(B.WlbError) as e:
                B.wlb_attn_workspace_size(d)
            assert e.value.status == 3
    d = B._desc(1000, 4096, 5, 8, 2, 128, 0.1)
    f, b = B.wlb_attn_workspace_size(d)
    lay = B.wlb_attn_plan_layout(d)
    # forward: schedule + partial results of the query tiles cut at a gang boundary (2 per gang and member)
    part = 2 * lay.row_gangs * (8 // 2) * (128 * 128 + 256) * 4
    assert f == lay.plan_bytes + part and b >= f + 4 * 8 * 1000
    assert lay.n_groups == 16 and lay.n_fwd_tiles == 8 and lay.n_key_tiles == 32
    # null pointers are rejected before anything is launched
    st = B.lib().wlb_attn_fwd(ctypes.byref(d), None, None, None, None, None, None, None, None, ctypes.c_size_t(0), None)
    assert st == 1 and b"null" in B.lib().wlb_last_error()


@pytest.mark.parametrize("thresholds,l_max", [((), 131072), ((65536,), 196608), ((65536, 98304), 196608),
                                              ((32768, 65536, 98304), 131072)])
def test_stream_packer_matches_oracle_on_the_document_pool(thresholds, l_max):
    w = wl.config(3)
    seqs = opk.pack_fixed_arrival(w.doc_len, 131072)
    batches = [sum(seqs[i:i + 8], []) for i in range(0, len(seqs) - 7, 8)]
    ref = opk.StreamPacker(8, l_max, 6, 640000, thresholds=thresholds)
    got = B.Packer(8, l_max, 6, 640000, thresholds)
    nid = 0
    for cur in batches:
        ids = list(range(nid, nid + len(cur)))
        nid += len(cur)
        placed, mb_len, mb_cost = ref.step(zip(ids, cur))
        oid, olen, omb, glen, gcost = got.step(ids, cur)
        assert list(zip(oid.tolist(), olen.tolist(), omb.tolist())) == placed
        assert glen.tolist() == mb_len and gcost.tolist() == mb_cost
        assert got.pending() == ref.pending_counts()
    got.close()


def test_stream_packer_random_and_errors():
    rng = np.random.default_rng(77)
    ref = opk.StreamPacker(3, 500, 1, 7, thresholds=[200, 350])
    got = B.Packer(3, 500, 1, 7, [200, 350])
    nid = 0
    for it in range(60):
        cur = rng.integers(1, 500, size=int(rng.integers(0, 12))).tolist()
        ids = list(range(nid, nid + len(cur)))
        nid += len(cur)
        placed, mb_len, mb_cost = ref.step(zip(ids, cur))
        oid, olen, omb, glen, gcost = got.step(ids, cur)
        assert list(zip(oid.tolist(), olen.tolist(), omb.tolist())) == placed
        assert glen.tolist() == mb_len and gcost.tolist() == mb_cost
    before = got.pending()
    with pytest.raises(B.WlbError):
        got.step([nid], [501])                      # longer than l_max: rejected, state unchanged
    assert got.pending() == before
    with pytest.raises(B.WlbError):
        B.Packer(3, 500, 1, 7, [300, 300])
    with pytest.raises(B.WlbError):
        B.Packer(0, 500, 1, 7)


def test_select_sharding_matches_oracle_bit_for_bit():
    from oracle import select as osel
    rng = np.random.default_rng(123)
    q_grid, kv_grid = [16, 128, 1024, 16384], [128, 4096, 131072]
    for trial in range(25):
        tab = rng.uniform(5.0, 900.0, size=(4, 3))
        prof = B.KernelProfile(q_grid, kv_grid, tab)
        cp = int(rng.choice([1, 2, 4, 8]))
        n = int(rng.integers(1, 40))
        doc = rng.integers(1, 5000, size=n)
        doc[-1] += (-int(doc.sum())) % (2 * cp)           # per-sequence mode needs 2*cp | T
        hq, d = int(rng.choice([1, 8, 32])), int(rng.choice([64, 128]))
        for mode in (0, 1, 2):
            want = [osel.rank_latency(doc.tolist(), cp, r, mode, hq, d, 128, 64, q_grid, kv_grid, tab.tolist())
                    for r in range(cp)]
            got = B.wlb_predict_latency(doc, cp, mode, hq, d, prof)
            assert got.tolist() == want
        m, a, b = B.wlb_select_sharding(doc, cp, hq, d, prof)
        assert (m, a, b) == osel.select(doc.tolist(), cp, hq, d, 128, 64, q_grid, kv_grid, tab.tolist())


def test_select_sharding_hand_example_and_errors():
    prof = B.KernelProfile([2, 8], [8, 32], [[1000e-12, 2000e-12], [2000e-12, 4000e-12]], tile_q=4, tile_k=4)
    m, a, b = B.wlb_select_sharding([8, 24], 2, 1, 1, prof)
    assert m == B.SHARD_PER_SEQ and abs(a - 1.0752) < 1e-6 and abs(b - 2.217035) < 1e-5
    with pytest.raises(B.WlbError):
        B.wlb_select_sharding([8, 23], 2, 1, 1, prof)                     # per-sequence needs 4 | T
    with pytest.raises(B.WlbError):
        B.wlb_select_sharding([8, 24], 2, 1, 1, B.KernelProfile([8, 2], [8, 32], [[1, 1], [1, 1]]))
    with pytest.raises(B.WlbError):
        B.wlb_select_sharding([8, 24], 2, 1, 1, B.KernelProfile([2, 8], [8, 32], [[1, 0], [1, 1]]))


def test_pack_optimal_matches_exhaustive_search_and_bounds_the_greedy():
    rng = np.random.default_rng(2024)
    gaps = []
    for trial in range(60):
        n, nb = int(rng.integers(1, 9)), int(rng.integers(1, 4))
        doc = rng.integers(1, 200, size=n)
        l_max = int(max(doc.max(), rng.integers(int(doc.sum()) // nb + 1, int(doc.sum()) + 2)))
        a, b = int(rng.integers(0, 4)), int(rng.integers(0, 500))
        want = opk.pack_optimal_bruteforce(doc.tolist(), nb, l_max, a, b)
        if want is None:
            with pytest.raises(B.WlbError):
                B.wlb_pack_optimal(doc, nb, l_max, a, b)
            continue
        assign, mb_len, mb_cost, opt, proven = B.wlb_pack_optimal(doc, nb, l_max, a, b)
        assert proven and opt == want
        # the returned assignment is feasible and attains the optimum
        for j in range(nb):
            sel = doc[assign == j]
            assert int(sel.sum()) == mb_len[j] <= l_max
            assert sum(opk.cost(int(d), a, b) for d in sel) == mb_cost[j]
        assert set(assign.tolist()) <= set(range(nb)) and int(mb_cost.max()) == opt
        g_assign, _, g_cost = B.wlb_pack(doc, nb, l_max, a, b)
        if (g_assign >= 0).all():
            assert int(g_cost.max()) >= opt
            gaps.append(int(g_cost.max()) / max(opt, 1))
    assert gaps and max(gaps) < 1.5


def test_pack_optimal_node_limit_and_errors():
    doc = np.arange(40, 0, -1, dtype=np.int32) * 37
    assign, mb_len, mb_cost, opt, proven = B.wlb_pack_optimal(doc, 8, 131072, 6, 640000, node_limit=20000)
    assert not proven and (assign >= 0).all() and int(mb_cost.max()) == opt
    with pytest.raises(B.WlbError):
        B.wlb_pack_optimal(np.ones(65, dtype=np.int32), 2, 100, 1, 1)
    with pytest.raises(B.WlbError):
        B.wlb_pack_optimal([60, 60, 60], 2, 100, 1, 1)          # three documents of 60 cannot share two bins of 100


def test_missing_library_is_an_error_not_a_fallback(tmp_path):
    """With no built library every product call raises; nothing falls back to another implementation."""
    import subprocess
    import sys
    code = (
        "import numpy as np\n"
        "from paper_2503_17924_amd import binding as B\n"
        "for call in (lambda: B.wlb_pack(np.array([3, 2], dtype=np.int32), 2, 10, 1, 1),\n"
        "             lambda: B.wlb_shard(np.array([8], dtype=np.int32), 2, 0, 0),\n"
        "             lambda: B.wlb_attn_workspace_size(B._desc(8, 8, 1, 1, 1, 64, 1.0))):\n"
        "    try:\n"
        "        call()\n"
        "    except RuntimeError as e:\n"
        "        assert 'missing' in str(e)\n"
        "    else:\n"
        "        raise SystemExit('a call succeeded without the library')\n"
        "print('ok')\n")
    env = dict(os.environ, WLB_LIBRARY=str(tmp_path / "no_such_libwlb.so"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env,
                       cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr
