"""Pins for oracle/pack.py (CPU only)."""
import heapq
import itertools
import os

import numpy as np
import pytest

from oracle import pack as opk

GOLD = os.path.join(os.path.dirname(__file__), "golden", "pack_examples.txt")


def _golden_cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [[int(x) for x in p.split()] for p in line.split("|")]
        out.append(tuple(parts))
    return out


@pytest.mark.parametrize("head,docs,assign,mb_len,mb_cost", _golden_cases())
def test_hand_worked_examples(head, docs, assign, mb_len, mb_cost):
    n, l_max, a, b = head
    got = opk.pack(docs, n, l_max, a, b)
    assert list(got[0]) == assign
    assert list(got[1]) == mb_len
    assert list(got[2]) == mb_cost


def test_linear_cost_no_limit_is_lpt():
    # with cost = length and no length limit the rule is Graham's longest-processing-time
    # list scheduling; an independent heap formulation must give the same loads
    rng = np.random.default_rng(7)
    for trial in range(20):
        docs = rng.integers(1, 500, size=40).tolist()
        n = int(rng.integers(2, 7))
        _, mb_len, mb_cost = opk.pack(docs, n, 10**9, 0, 1)
        heap = [(0, j) for j in range(n)]
        for d in sorted(docs, reverse=True):
            load, j = heapq.heappop(heap)
            heapq.heappush(heap, (load + d, j))
        assert sorted(load for load, _ in heap) == sorted(mb_len)
        assert mb_len == mb_cost
        # LPT guarantee: makespan <= (4/3 - 1/(3N)) * optimum, optimum >= max(mean, longest)
        lower = max(sum(docs) / n, max(docs))
        assert max(mb_len) <= (4 / 3 - 1 / (3 * n)) * lower + max(docs)


def _check_valid(docs, assign, mb_len, mb_cost, n, l_max, a, b):
    assert len(assign) == len(docs)
    for j in range(n):
        members = [d for d, x in zip(docs, assign) if x == j]
        assert sum(members) == mb_len[j] <= l_max
        assert sum(a * d * d + b * d for d in members) == mb_cost[j]
    assert all(-1 <= x < n for x in assign)


def test_validity_and_leftover_rule():
    rng = np.random.default_rng(11)
    for trial in range(30):
        docs = rng.integers(1, 300, size=60).tolist()
        n, l_max, a, b = 4, 700, 3, 50
        assign, mb_len, mb_cost = opk.pack(docs, n, l_max, a, b)
        _check_valid(docs, assign, mb_len, mb_cost, n, l_max, a, b)
        # replay: a document is left over only if even the fewest-token micro-batch is too full
        order = sorted(range(len(docs)), key=lambda i: -docs[i])
        lens = [0] * n
        for i in order:
            if assign[i] < 0:
                assert min(lens) + docs[i] > l_max
            else:
                lens[assign[i]] += docs[i]


def test_greedy_never_beats_bruteforce_optimum():
    # Equation 2 (minimise the max micro-batch workload subject to the length cap)
    rng = np.random.default_rng(5)
    for trial in range(15):
        docs = rng.integers(1, 30, size=7).tolist()
        n, l_max, a, b = 3, 60, 2, 7
        assign, mb_len, mb_cost = opk.pack(docs, n, l_max, a, b)
        if min(assign) < 0:
            continue
        best = None
        for x in itertools.product(range(n), repeat=len(docs)):
            lens = [0] * n
            cost = [0] * n
            for d, j in zip(docs, x):
                lens[j] += d
                cost[j] += a * d * d + b * d
            if max(lens) <= l_max:
                best = max(cost) if best is None else min(best, max(cost))
        assert best is not None and max(mb_cost) >= best
        assert max(mb_cost) <= 2 * best      # list scheduling never exceeds twice the optimum


def test_equal_lengths_keep_arrival_order():
    docs = [5, 5, 5, 5]
    assign, _, _ = opk.pack(docs, 2, 100, 1, 0)
    assert assign == [0, 1, 0, 1]


def test_stream_carries_leftovers_forward():
    batches = [[10, 10, 9], [3, 2], [1]]
    out, tail = opk.pack_stream(batches, 2, 10, 1, 0)
    assert out[0][0] == [10, 10, 9] and out[0][1] == [0, 1, -1]
    assert out[1][0][:1] == [9]                       # the left-over heads the next set
    assert sorted(x for x in out[1][1]) == [0, 1, -1] or min(out[1][1]) >= 0
    total_in = sum(sum(b) for b in batches)
    total_packed = sum(sum(o[2]) for o in out)
    assert total_in == total_packed + sum(tail)


def test_fixed_arrival_packing():
    seqs = opk.pack_fixed_arrival([5, 4, 7, 3], 8)
    assert seqs == [[5, 3], [1, 7], [3]]
    assert opk.imbalance([3, 1, 2]) == pytest.approx(1.5)


def test_errors():
    with pytest.raises(ValueError):
        opk.pack([3, 0], 2, 10, 1, 1)
    with pytest.raises(ValueError):
        opk.pack([3], 0, 10, 1, 1)


def _stream_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "stream_packer_example.txt")
    steps, cur = [], {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(" ", 1)
        if key == "batch":
            cur = {"batch": [tuple(int(x) for x in t.split(":")) for t in rest.split()]}
            steps.append(cur)
        elif key == "placed":
            cur["placed"] = [tuple(int(x) for x in t.split(":")) for t in rest.split()]
        else:
            cur[key] = [int(x) for x in rest.split()]
    return steps


def test_stream_packer_hand_worked_example():
    sp = opk.StreamPacker(2, 20, 1, 0, thresholds=[10])
    for st in _stream_example():
        placed, mb_len, mb_cost = sp.step(st["batch"])
        assert placed == st["placed"]
        assert mb_len == st["mb_len"] and mb_cost == st["mb_cost"]
        assert list(sp.pending_counts()) == st["state"]


def test_stream_packer_without_queues_is_the_plain_stream():
    rng = np.random.default_rng(9)
    batches = [rng.integers(1, 400, size=30).tolist() for _ in range(6)]
    want, tail = opk.pack_stream(batches, 3, 900, 2, 11)
    sp = opk.StreamPacker(3, 900, 2, 11)
    nid = 0
    for cur, (docs, assign, mb_len, mb_cost) in zip(batches, want):
        placed, got_len, got_cost = sp.step([(nid + i, d) for i, d in enumerate(cur)])
        nid += len(cur)
        assert got_len == mb_len and got_cost == mb_cost
        assert sorted(d for _, d, _ in placed) == sorted(d for d, j in zip(docs, assign) if j >= 0)
    assert sp.pending_counts() == (len(tail), 0)


def test_stream_packer_invariants():
    rng = np.random.default_rng(10)
    n, l_max = 4, 3000
    sp = opk.StreamPacker(n, l_max, 3, 100, thresholds=[800, 1600])
    arrived, placed_ids = {}, []
    nid = 0
    for it in range(40):
        batch = []
        for _ in range(int(rng.integers(5, 25))):
            d = int(rng.integers(1, 2500))
            batch.append((nid, d))
            arrived[nid] = d
            nid += 1
        placed, mb_len, mb_cost = sp.step(batch)
        for i, d, j in placed:
            assert arrived[i] == d and 0 <= j < n
            placed_ids.append(i)
        assert max(mb_len) <= l_max
        lens = [d for _, d, _ in placed]
        assert lens == sorted(lens, reverse=True)
    assert len(placed_ids) == len(set(placed_ids))
    rem, queued = sp.pending_counts()
    assert len(placed_ids) + rem + queued == nid


def test_outlier_delay_improves_balance_on_the_long_tailed_pool():
    """Analogue of the paper's packing comparison (Section 6.4, Table 2) on the synthetic pool:
    with L_max = 1.5 windows, queues for the very long documents lower the imbalance degree."""
    from paper_2503_17924_amd import workloads as wl
    w = wl.config(3)
    window = 131072
    seqs = opk.pack_fixed_arrival(w.doc_len, window)
    batches = [sum(seqs[i:i + 8], []) for i in range(0, len(seqs) - 7, 8)]
    a, b = 6, 640000

    def run(thresholds):
        sp = opk.StreamPacker(8, window * 3 // 2, a, b, thresholds=thresholds)
        degs, nid = [], 0
        for cur in batches:
            placed, mb_len, mb_cost = sp.step([(nid + i, d) for i, d in enumerate(cur)])
            nid += len(cur)
            if min(mb_cost) > 0:
                degs.append(opk.imbalance(mb_cost))
        return float(np.mean(degs))

    fixed = float(np.mean([opk.imbalance([sum(opk.cost(d, a, b) for d in s) for s in seqs[i:i + 8]])
                           for i in range(0, len(seqs) - 7, 8)]))
    plain = run([])
    two_q = run([window // 2, window * 3 // 4])
    assert plain < fixed
    assert two_q < plain


def test_exhaustive_optimum_on_textbook_partition_instances():
    # linear cost (a=0, b=1) without a binding length limit is multiway number partitioning
    assert opk.pack_optimal_bruteforce([3, 3, 2, 2, 2], 2, 100, 0, 1) == 6          # {3,3} | {2,2,2}; LPT gives 7
    assert opk.pack_optimal_bruteforce([8, 7, 6, 5, 4], 2, 100, 0, 1) == 15         # {8,7} | {6,5,4}
    assert opk.pack_optimal_bruteforce([5, 5, 5, 5], 2, 10, 0, 1) == 10
    assert opk.pack_optimal_bruteforce([5, 5, 5, 5], 2, 9, 0, 1) is None            # the length limit makes it infeasible
    assert opk.pack_optimal_bruteforce([3, 2, 2], 2, 100, 1, 0) == 9                # quadratic cost: {3} | {2,2} = max(9, 8)
    # the length limit can force a worse optimum: {4,1} | {3,2} is forbidden when l_max = 4... so is everything
    assert opk.pack_optimal_bruteforce([4, 3, 2, 1], 2, 5, 0, 1) == 5
    # greedy LPT on the first instance is strictly worse than the optimum
    assert max(opk.pack([3, 3, 2, 2, 2], 2, 100, 0, 1)[2]) == 7
