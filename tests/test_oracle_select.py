"""Pins of the adaptive-sharding oracle (paper Section 5.3)."""
import os

import numpy as np
import pytest

from oracle import attention as oat
from oracle import select as osel
from oracle import shard as osh

GOLD = os.path.join(os.path.dirname(__file__), "golden", "select_example.txt")
EX_TABLE = dict(q_grid=[2, 8], kv_grid=[8, 32], tflops=[[1000e-12, 2000e-12], [2000e-12, 4000e-12]])


def test_hand_worked_example():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    for mode, rank, want in rows:
        got = osel.rank_latency([8, 24], 2, int(rank), int(mode), 1, 1, 4, 4, **EX_TABLE)
        assert got == pytest.approx(float(want), rel=2e-6), (mode, rank)
    mode, lat_seq, lat_doc = osel.select([8, 24], 2, 1, 1, 4, 4, **EX_TABLE)
    assert mode == osel.PER_SEQ and lat_seq == pytest.approx(1.0752, rel=2e-6) and lat_doc == pytest.approx(2.217035, rel=2e-6)


@pytest.mark.parametrize("n,tq,tk", [(1, 128, 64), (7, 128, 64), (5, 4, 4), (3, 8, 2)])
def test_padded_pairs_closed_form_for_a_whole_causal_document(n, tq, tk):
    # Q_len = KV_len = n*tq with tk | tq: tile t sees (t+1)*tq keys, so the count is tq^2 * n(n+1)/2
    L = n * tq
    assert osel.padded_pairs(L, L, tq, tk) == tq * tq * n * (n + 1) // 2


def test_padded_pairs_bound_useful_pairs_and_tile_rounding():
    rng = np.random.default_rng(5)
    for _ in range(200):
        kv = int(rng.integers(1, 700))
        q = int(rng.integers(1, kv + 1))
        tq, tk = int(rng.choice([4, 16, 128])), int(rng.choice([4, 16, 64]))
        useful = sum(kv - q + i + 1 for i in range(q))
        got = osel.padded_pairs(q, kv, tq, tk)
        assert got >= useful
        assert got % (tq * tk) == 0
        # never more than one extra key tile per row tile plus the row padding of the last tile
        nt = -(-q // tq)
        assert got <= sum(tq * (kv - q + min((t + 1) * tq, q) + tk - 1) for t in range(nt))
    assert osel.padded_pairs(5, 0, 4, 4) == 0 and osel.padded_pairs(0, 9, 4, 4) == 0


def test_useful_pairs_of_a_segment_match_the_attention_oracle():
    # the (Q_len, KV_len) shape of a segment describes the same causal trapezoid the attention oracle counts
    doc = [37, 90]
    for mode in (0, 1):
        if mode == 1 and sum(doc) % 8:
            continue
        for r in range(4):
            sh = osh.shard(doc, 4, r, mode)
            cu_q, kb, ke = sh["cu_seqlens_q"], sh["seg_k_begin"], sh["seg_k_end"]
            tot = 0
            for s in range(len(kb)):
                real = [g for g in sh["q_idx"][cu_q[s]:cu_q[s + 1]] if g >= 0]
                tot += sum(g - kb[s] + 1 for g in real)
            assert tot == oat.useful_pairs(sh["q_idx"], sh["cu_seqlens_k"])


def test_flat_table_makes_latency_proportional_to_padded_operations():
    doc = [300, 45, 1000, 7]
    flat = dict(q_grid=[1, 4096], kv_grid=[1, 4096], tflops=[[2.0, 2.0], [2.0, 2.0]])
    for mode in (0, 2):
        for r in range(2):
            sh = osh.shard(doc, 2, r, mode)
            pairs = sum(osel.padded_pairs(int(sh["cu_seqlens_q"][s + 1] - sh["cu_seqlens_q"][s]),
                                          int(sh["seg_k_end"][s] - sh["seg_k_begin"][s]), 128, 64)
                        for s in range(len(sh["seg_k_begin"])))
            got = osel.rank_latency(doc, 2, r, mode, 8, 128, 128, 64, **flat)
            assert got == pytest.approx(pairs * 14.0 * 128 * 8 / 2e12, rel=1e-12)


def test_single_divisible_document_predicts_the_same_for_both_shardings():
    tab = dict(q_grid=[64, 512, 4096], kv_grid=[64, 4096, 32768],
               tflops=[[10.0, 50.0, 60.0], [40.0, 300.0, 500.0], [50.0, 600.0, 900.0]])
    mode, a, b = osel.select([8192], 4, 8, 128, 128, 64, **tab)
    assert a == b and mode == osel.PER_SEQ          # ties go to per-sequence


def test_lookup_interpolates_and_clamps():
    tab = EX_TABLE
    assert osel.lookup(tab["q_grid"], tab["kv_grid"], tab["tflops"], 1, 1) == 1000e-12
    assert osel.lookup(tab["q_grid"], tab["kv_grid"], tab["tflops"], 100, 100) == 4000e-12
    assert osel.lookup(tab["q_grid"], tab["kv_grid"], tab["tflops"], 5, 20) == pytest.approx(2250e-12, rel=1e-12)


def test_short_documents_favour_per_sequence_and_a_skewed_mix_favours_per_document():
    # a table with the shape the paper describes: poor rates for short query chunks
    tab = dict(q_grid=[16, 128, 1024, 16384], kv_grid=[128, 4096, 131072],
               tflops=[[5.0, 20.0, 25.0], [40.0, 200.0, 250.0], [100.0, 500.0, 700.0], [120.0, 600.0, 900.0]])
    many_short = [256] * 512                       # balanced already: per-document only shreds the chunks
    assert osel.select(many_short, 8, 8, 128, 128, 64, **tab)[0] == osel.PER_SEQ
    skewed = [114688] + [2048] * 8                 # one long document: per-sequence is badly imbalanced
    assert osel.select(skewed, 8, 8, 128, 128, 64, **tab)[0] == osel.PER_DOC
