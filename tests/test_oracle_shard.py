"""Pins for oracle/shard.py (CPU only)."""
import os

import numpy as np
import pytest

from oracle import shard as osh

GOLD = os.path.join(os.path.dirname(__file__), "golden", "shard_examples.txt")


def _golden_cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        fields = [x.strip() for x in line.split("|")]
        head, docs, exp = fields[:3]
        mode, cp, rank = head.split()
        segs = [[int(x) for x in f.split()] for f in fields[3:]]
        assert len(segs) in (0, 3), line
        out.append(({"per_doc": osh.PER_DOC_PADDED, "per_seq": osh.PER_SEQ, "per_doc_nopad": osh.PER_DOC_NOPAD}[mode], int(cp), int(rank),
                    [int(x) for x in docs.split()], [int(x) for x in exp.split()], segs))
    return out


@pytest.mark.parametrize("mode,cp,rank,docs,exp,segs", _golden_cases())
def test_hand_worked_examples(mode, cp, rank, docs, exp, segs):
    r = osh.shard(docs, cp, rank, mode)
    assert r["q_idx"].tolist() == exp
    if segs:
        assert r["cu_seqlens_q"].tolist() == segs[0]
        assert r["seg_k_begin"].tolist() == segs[1]
        assert r["seg_k_end"].tolist() == segs[2]


def test_golden_file_pins_the_segments_of_every_mode():
    modes = {m for m, _, _, _, _, segs in _golden_cases() if segs}
    assert modes == {osh.PER_DOC_PADDED, osh.PER_SEQ, osh.PER_DOC_NOPAD}
    # and a rank that holds two non-adjacent remaining tokens of one document (padding-free mode)
    assert any(m == osh.PER_DOC_NOPAD and segs and len(segs[1]) != len(set(segs[1])) and
               any(b - a == 1 for a, b in zip(segs[0], segs[0][1:])) for m, _, _, _, _, segs in _golden_cases())


def _rand_docs(rng, n, hi):
    return rng.integers(1, hi, size=n, endpoint=True).tolist()


@pytest.mark.parametrize("cp", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("mode", [osh.PER_DOC_PADDED, osh.PER_SEQ])
def test_ranks_partition_the_sequence(cp, mode):
    rng = np.random.default_rng(cp * 10 + mode)
    docs = _rand_docs(rng, 13, 97)
    total = sum(docs)
    if mode == osh.PER_SEQ and total % (2 * cp):
        docs[-1] += 2 * cp - total % (2 * cp)
        total = sum(docs)
    seen, sizes = [], set()
    for r in range(cp):
        out = osh.shard(docs, cp, r, mode)
        q = out["q_idx"]
        seen.extend(q[q >= 0].tolist())
        sizes.add(len(q))
        real = q[q >= 0]
        assert (np.diff(real) > 0).all()           # strictly increasing real entries
        assert out["cu_seqlens_q"][-1] == len(q)
        assert out["cu_seqlens_k"].tolist() == np.concatenate([[0], np.cumsum(docs)]).tolist()
    assert sorted(seen) == list(range(total))       # every token on exactly one rank
    assert len(sizes) == 1                          # same number of slots on every rank
    if mode == osh.PER_SEQ:
        assert sizes.pop() == total // cp


@pytest.mark.parametrize("cp", [2, 4, 8])
def test_pair_count_closed_form_when_divisible(cp):
    # chunk m of a document with chunk length c contributes m*c*c + c(c+1)/2 causal
    # pairs, so the symmetric pair (r, 2CP-1-r) always gives (2CP-1)c^2 + c(c+1).
    n = 2 * cp
    docs = [n * c for c in (1, 3, 7, 20)]
    want = sum((n - 1) * c * c + c * (c + 1) for c in (1, 3, 7, 20))
    for r in range(cp):
        assert osh.shard(docs, cp, r, osh.PER_DOC_PADDED)["useful_pairs"] == want
    total_pairs = sum(L * (L + 1) // 2 for L in docs)
    assert want * cp == total_pairs


def test_useful_pairs_sum_to_total_with_padding():
    docs = [5, 1, 17, 33, 2]
    for cp in (2, 3, 4):
        tot = sum(osh.shard(docs, cp, r, osh.PER_DOC_PADDED)["useful_pairs"] for r in range(cp))
        assert tot == sum(L * (L + 1) // 2 for L in docs)


def test_cp1_is_identity_without_padding():
    docs = [3, 1, 7]
    for mode in (osh.PER_DOC_PADDED, osh.PER_SEQ):
        out = osh.shard(docs, 1, 0, mode)
        assert out["q_idx"].tolist() == list(range(11))
        assert out["cu_seqlens_q"].tolist() == [0, 3, 4, 11]
        assert out["seg_k_begin"].tolist() == [0, 3, 4]
        assert out["seg_k_end"].tolist() == [3, 4, 11]


def test_single_divisible_document_same_in_both_modes():
    for cp in (2, 4):
        for r in range(cp):
            a = osh.shard([8 * cp], cp, r, osh.PER_DOC_PADDED)
            b = osh.shard([8 * cp], cp, r, osh.PER_SEQ)
            for key in ("q_idx", "cu_seqlens_q", "seg_k_begin", "seg_k_end"):
                assert a[key].tolist() == b[key].tolist()


def _chunk_of(mode, cp, docs, tok):
    """The definition, written out for one token: (document, chunk) it belongs to; chunk -1 = one of a
    document's remaining tokens in the padding-free mode."""
    cu = np.concatenate([[0], np.cumsum(docs)])
    d = int(np.searchsorted(cu, tok, side="right") - 1)
    n = 2 * cp
    if cp == 1:
        return d, 0
    if mode == osh.PER_SEQ:
        return d, tok // (cu[-1] // n)
    L, p = docs[d], tok - cu[d]
    if mode == osh.PER_DOC_PADDED:
        return d, p // -(-L // n)
    c = L // n
    return d, (p // c if p < c * n else -1)


@pytest.mark.parametrize("mode", [osh.PER_DOC_PADDED, osh.PER_SEQ, osh.PER_DOC_NOPAD])
@pytest.mark.parametrize("cp,docs", [(2, [5, 12, 1, 30]), (3, [7, 29, 2, 64, 11, 1, 6]), (4, [3, 50, 21, 9, 13])])
def test_segments_describe_the_rows(mode, cp, docs):
    """cu_seqlens_q / seg_k_begin / seg_k_end against their definition: the segments tile the slots in
    order; the real rows of a segment are consecutive tokens of one chunk of one document; two segments in
    a row differ in document or chunk or are separated by a gap (maximal runs); seg_k_begin is the
    document's start and seg_k_end one past the segment's last real token."""
    docs = list(docs)
    total = sum(docs)
    if mode == osh.PER_SEQ and total % (2 * cp):
        docs[-1] += 2 * cp - total % (2 * cp)
    for r in range(cp):
        out = osh.shard(docs, cp, r, mode)
        cu_k, cu_q = out["cu_seqlens_k"], out["cu_seqlens_q"]
        assert cu_q[0] == 0 and cu_q[-1] == len(out["q_idx"]) and (np.diff(cu_q) > 0).all()
        assert len(out["seg_k_begin"]) == len(out["seg_k_end"]) == len(cu_q) - 1
        prev = None
        for s in range(len(out["seg_k_begin"])):
            rows = out["q_idx"][cu_q[s]:cu_q[s + 1]]
            real = rows[rows >= 0]
            kb, ke = out["seg_k_begin"][s], out["seg_k_end"][s]
            assert kb in cu_k.tolist()
            if mode == osh.PER_DOC_NOPAD:
                assert len(real) == len(rows)
            if not len(real):
                assert ke == kb
                prev = None
                continue
            assert (np.diff(real) == 1).all()                     # consecutive tokens
            assert (rows[:len(real)] >= 0).all()                  # padding only at a segment's end
            keys = {_chunk_of(mode, cp, docs, int(t)) for t in real}
            assert len(keys) == 1                                 # one chunk of one document
            d, chunk = next(iter(keys))
            assert cu_k[d] == kb and ke == real.max() + 1
            if chunk >= 0:
                assert chunk in (r, 2 * cp - 1 - r) or cp == 1
            # maximal: the segment before it is another (document, chunk) or does not end right before it
            if prev is not None and prev[0] == (d, chunk):
                assert prev[1] + 1 < real[0]
            prev = ((d, chunk), int(real[-1]))


def test_padding_free_pair_count_is_the_sum_over_the_rows():
    docs = [7, 29, 2, 64, 11, 1, 6]
    for cp in (2, 3):
        cu = np.concatenate([[0], np.cumsum(docs)])
        for r in range(cp):
            out = osh.shard(docs, cp, r, osh.PER_DOC_NOPAD)
            q = out["q_idx"]
            want = int((q - cu[np.searchsorted(cu, q, side="right") - 1] + 1).sum())
            assert out["useful_pairs"] == want


def test_per_sequence_is_imbalanced_per_document_is_not():
    # a long document followed by short ones: the paper's motivating case (Section 3.1)
    docs = [96] + [4] * 8
    cp = 4
    seq = [osh.shard(docs, cp, r, osh.PER_SEQ)["useful_pairs"] for r in range(cp)]
    doc = [osh.shard(docs, cp, r, osh.PER_DOC_PADDED)["useful_pairs"] for r in range(cp)]
    assert max(seq) / (sum(seq) / cp) > 1.2
    assert max(doc) / (sum(doc) / cp) < 1.05


def test_errors():
    with pytest.raises(ValueError):
        osh.shard([4, 0], 2, 0, osh.PER_DOC_PADDED)
    with pytest.raises(ValueError):
        osh.shard([4], 2, 2, osh.PER_DOC_PADDED)
    with pytest.raises(ValueError):
        osh.shard([5], 2, 0, osh.PER_SEQ)


@pytest.mark.parametrize("cp", [2, 3, 4, 8])
def test_padding_free_partition_and_equal_counts(cp):
    rng = np.random.default_rng(cp)
    docs = _rand_docs(rng, 17, 131)
    total = sum(docs)
    docs[-1] += (2 * cp - total % (2 * cp)) % (2 * cp)          # 2*CP | T, as the paper assumes
    seen, sizes = [], []
    for r in range(cp):
        out = osh.shard(docs, cp, r, osh.PER_DOC_NOPAD)
        q = out["q_idx"]
        assert (q >= 0).all()                                   # no padding slots at all
        assert (np.diff(q) > 0).all()
        seen.extend(q.tolist())
        sizes.append(len(q))
    assert sorted(seen) == list(range(sum(docs)))
    assert len(set(sizes)) == 1 and sizes[0] == sum(docs) // cp  # every worker the same number of tokens


def test_padding_free_equals_padded_when_everything_divides():
    docs = [16, 32, 8]
    for r in range(4):
        a = osh.shard(docs, 4, r, osh.PER_DOC_NOPAD)
        b = osh.shard(docs, 4, r, osh.PER_DOC_PADDED)
        for key in ("q_idx", "cu_seqlens_q", "seg_k_begin", "seg_k_end"):
            assert a[key].tolist() == b[key].tolist()


def test_padding_free_counts_differ_by_at_most_one_otherwise():
    docs = [5, 9, 2, 31]                                         # T = 47, not divisible
    sizes = [len(osh.shard(docs, 4, r, osh.PER_DOC_NOPAD)["q_idx"]) for r in range(4)]
    assert max(sizes) - min(sizes) <= 1 and sum(sizes) == 47


def test_padding_free_balances_attention_work():
    rng = np.random.default_rng(3)
    docs = rng.integers(200, 3000, size=12).tolist()
    cp = 4
    pairs = [osh.shard(docs, cp, r, osh.PER_DOC_NOPAD)["useful_pairs"] for r in range(cp)]
    assert sum(pairs) == sum(L * (L + 1) // 2 for L in docs)
    assert max(pairs) / (sum(pairs) / cp) < 1.02
