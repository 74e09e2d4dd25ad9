"""Oracle: context-parallel sharding maps (exact integers).

TEST INFRASTRUCTURE ONLY.  Nothing here is used by the HIP path.

Per-sequence sharding (paper Section 3.1, "CP Level Imbalance", and Section 5.1):
the packed sequence of T tokens is cut into 2*CP equal chunks and worker r takes
chunks r and 2*CP-1-r.

Per-document sharding (paper Section 5.1): every document is cut into 2*CP
chunks and worker r takes the symmetric pair r, 2*CP-1-r of every document; a
document whose length is not divisible by 2*CP is extended with padding tokens.

Padding-free per-document sharding (paper Section 5.1, "Avoid Padding"): a document of
length L is split into a part divisible by 2*CP and the R = L mod 2*CP remaining tokens; the
divisible part is sharded like a document of that length, the remaining tokens are dealt to
the CP workers round-robin.  As printed, the formula defines D_i as floor(L_i / (2*CP)), a
chunk length, while the text uses D_i as the divisible part; the reading here is
D_i = 2*CP * floor(L_i / (2*CP)).  Also open in the paper and fixed here: the remaining tokens
are the LAST R_i tokens of the document, and the round-robin is one counter that runs on
across documents (token number t of all remaining tokens, in sequence order, goes to worker
t mod CP), which is what gives every worker the same number of tokens when 2*CP divides the
sequence length.  A rank's slots stay document-major: front chunk, back chunk, then its
remaining tokens of that document.

Readings where the paper is silent (all shared with the C library by design):
  * padding goes at the document's tail: chunk length c = ceil(L / (2*CP)),
    chunk m covers document positions [m*c, (m+1)*c), positions >= L are pads;
  * pads are materialised as slots with q_idx = -1, so every rank has the same
    number of slots, sum over documents of 2*c;
  * a rank's slots are document-major; within a document the front chunk (r)
    comes before the back chunk (2*CP-1-r);
  * CP = 1 is the identity map with no padding, one segment per document;
  * per-sequence mode requires 2*CP | T;
  * a segment is a maximal run of slots that belong to one chunk and one
    document; seg_k_begin is the document start and seg_k_end is one past the
    last key the segment's last real row may see (= begin if it has no real row).

Pins (tests/test_oracle_shard.py): all ranks' real entries partition [0, T);
equal slot counts; the closed-form pair count (2CP-1)c^2 + c(c+1) per rank when
2*CP | L; CP = 1 identity; single document with 2*CP | L gives the same map in
both modes; hand-worked small examples under tests/golden/ (q_idx of every mode,
and cu_seqlens_q / seg_k_begin / seg_k_end of every mode, the round-robin remainder
runs of the padding-free mode included); the segment arrays of all three modes
against their definition (maximal runs of consecutive tokens of one chunk of one
document, seg_k_end one past the last real token).
"""
from __future__ import annotations

import numpy as np

PER_DOC_PADDED = 0
PER_SEQ = 1
PER_DOC_NOPAD = 2


def _segments_to_arrays(segs, doc_len):
    """segs: list of (slot list, doc_start). Builds the output arrays."""
    q_idx, cu_q, kb, ke = [], [0], [], []
    for slots, doc_start in segs:
        q_idx.extend(slots)
        cu_q.append(len(q_idx))
        real = [g for g in slots if g >= 0]
        kb.append(doc_start)
        ke.append(real[-1] + 1 if real else doc_start)
    cu_k = np.concatenate([[0], np.cumsum(np.asarray(doc_len, dtype=np.int64))])
    return (np.asarray(q_idx, dtype=np.int32), np.asarray(cu_q, dtype=np.int32),
            np.asarray(kb, dtype=np.int32), np.asarray(ke, dtype=np.int32), cu_k.astype(np.int32))


def shard(doc_len, cp: int, rank: int, mode: int):
    """Returns dict(q_idx, cu_seqlens_q, seg_k_begin, seg_k_end, cu_seqlens_k, useful_pairs)."""
    doc_len = [int(x) for x in doc_len]
    if cp < 1 or not (0 <= rank < cp) or any(L <= 0 for L in doc_len) or mode not in (PER_DOC_PADDED, PER_SEQ, PER_DOC_NOPAD):
        raise ValueError("invalid sharding arguments")
    starts = [0]
    for L in doc_len:
        starts.append(starts[-1] + L)
    total = starts[-1]
    n = 2 * cp
    segs = []
    if cp == 1:
        for d, L in enumerate(doc_len):
            segs.append((list(range(starts[d], starts[d] + L)), starts[d]))
    elif mode == PER_DOC_PADDED:
        for d, L in enumerate(doc_len):
            c = -(-L // n)
            for m in (rank, n - 1 - rank):
                slots = [starts[d] + p if p < L else -1 for p in range(m * c, (m + 1) * c)]
                segs.append((slots, starts[d]))
    elif mode == PER_DOC_NOPAD:
        t = 0                                     # running count of remaining tokens over the whole sequence
        for d, L in enumerate(doc_len):
            c = L // n
            if c > 0:
                for m in (rank, n - 1 - rank):
                    segs.append((list(range(starts[d] + m * c, starts[d] + (m + 1) * c)), starts[d]))
            run = []
            for p in range(c * n, L):
                if t % cp == rank:
                    if run and run[-1] != starts[d] + p - 1:
                        segs.append((run, starts[d]))
                        run = []
                    run.append(starts[d] + p)
                t += 1
            if run:
                segs.append((run, starts[d]))
    else:
        if total % n != 0:
            raise ValueError("per-sequence sharding needs 2*CP | T")
        c = total // n
        for m in (rank, n - 1 - rank):
            lo, hi = m * c, (m + 1) * c
            for d, L in enumerate(doc_len):
                a, b = max(lo, starts[d]), min(hi, starts[d] + L)
                if a < b:
                    segs.append((list(range(a, b)), starts[d]))
    q_idx, cu_q, kb, ke, cu_k = _segments_to_arrays(segs, doc_len)
    pairs = 0
    for (slots, doc_start) in segs:
        for g in slots:
            if g >= 0:
                pairs += g - doc_start + 1
    return dict(q_idx=q_idx, cu_seqlens_q=cu_q, seg_k_begin=kb, seg_k_end=ke,
                cu_seqlens_k=cu_k, useful_pairs=pairs)
