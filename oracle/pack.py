"""Oracle: workload-aware variable-length packing (exact integers).

TEST INFRASTRUCTURE ONLY.  Nothing here is used by the HIP path.

`pack` is the greedy core of the paper's Algorithm 1 (Section 4.3): the pending
documents are sorted by length, longest first; each goes to the micro-batch
with the least workload if it fits under L_max, else to the micro-batch with
the fewest tokens if it fits there, else it is left over for the next
iteration.  A micro-batch's workload is the sum over its documents of
W_a(d) + W_l(d) (Equation 2, Section 4.1) with W_a quadratic in the document
length (Section 3.2: causal attention work is proportional to sum d_i^2) and
W_l linear (Section 4.1, operation latency vs. document length):
cost(d) = a*d*d + b*d in unsigned integers.

Readings where the paper is silent or at odds with itself:
  * fit test is `<= L_max` (Equation 2's constraint; the algorithm listing
    prints a strict `<`, under which a window-length document could never be
    placed);
  * the sort is stable: equal lengths keep arrival order;
  * ties in "least workload" / "fewest tokens" go to the lowest index.

`pack_stream` is the outer loop of Algorithm 1 without outlier queues: the
left-over documents of one iteration head the next iteration's document set.
`pack_fixed_arrival` is the baseline the paper calls original packing
(Section 2.2, Section 6.1): documents in arrival order fill fixed-length
sequences; a document that crosses the end of a sequence is cut there and the
rest starts the next sequence as a new document.
`imbalance` is the max-over-mean degree of Section 3.3.

Pins (tests/test_oracle_pack.py): with a=0, b=1 and no length limit the greedy
is the textbook longest-processing-time rule (checked on a hand-worked instance
and against a heap formulation); assignment validity; a document is left over
only when even the shortest micro-batch cannot take it; brute-force optimum of
Equation 2 on tiny inputs bounds the greedy from below and the LPT 4/3 bound
holds for linear cost.
"""
from __future__ import annotations


def cost(d: int, a: int, b: int) -> int:
    return a * d * d + b * d


def pack(doc_len, n_microbatch: int, l_max: int, a: int, b: int):
    """Returns (assign[n_docs] with -1 = left over, mb_len[N], mb_cost[N])."""
    doc_len = [int(x) for x in doc_len]
    if n_microbatch < 1 or l_max < 1 or a < 0 or b < 0 or any(d <= 0 for d in doc_len):
        raise ValueError("invalid packing arguments")
    order = sorted(range(len(doc_len)), key=lambda i: -doc_len[i])   # stable: ties keep arrival order
    work = [0] * n_microbatch
    length = [0] * n_microbatch
    assign = [-1] * len(doc_len)
    for i in order:
        d = doc_len[i]
        w_idx = min(range(n_microbatch), key=lambda j: (work[j], j))
        l_idx = min(range(n_microbatch), key=lambda j: (length[j], j))
        if length[w_idx] + d <= l_max:
            j = w_idx
        elif length[l_idx] + d <= l_max:
            j = l_idx
        else:
            continue
        assign[i] = j
        work[j] += cost(d, a, b)
        length[j] += d
    return assign, length, work


def pack_optimal_bruteforce(doc_len, n_microbatch: int, l_max: int, a: int, b: int):
    """Equation 2 by exhaustive search (Section 4.1): every document in exactly one micro-batch,
    every micro-batch at most l_max tokens, minimise the largest micro-batch cost.  Returns the
    optimal value, or None when no assignment satisfies the length limit.  Exponential: tiny
    inputs only (it tries all n_microbatch^n assignments, nothing pruned, so that it stays an
    independent check of the library's branch-and-bound solver)."""
    import itertools
    doc_len = [int(x) for x in doc_len]
    best = None
    for assign in itertools.product(range(n_microbatch), repeat=len(doc_len)):
        length = [0] * n_microbatch
        work = [0] * n_microbatch
        for d, j in zip(doc_len, assign):
            length[j] += d
            work[j] += cost(d, a, b)
        if max(length) <= l_max:
            w = max(work)
            if best is None or w < best:
                best = w
    return best


def pack_stream(batches, n_microbatch: int, l_max: int, a: int, b: int):
    """batches: iterable of lists of document lengths (one list per global batch).
    Returns a list with one entry per iteration: (doc_lengths_considered, assign,
    mb_len, mb_cost); left-over documents are carried to the front of the next
    iteration's set, and whatever is left at the end is returned as the tail."""
    remained = []
    out = []
    for cur in batches:
        docs = list(remained) + [int(x) for x in cur]
        assign, mb_len, mb_cost = pack(docs, n_microbatch, l_max, a, b)
        remained = [d for d, j in zip(docs, assign) if j < 0]
        out.append((docs, assign, mb_len, mb_cost))
    return out, remained


def pack_fixed_arrival(doc_len, window: int):
    """Arrival-order packing into sequences of exactly `window` tokens (the last
    may be shorter).  Returns a list of sequences, each a list of document
    lengths; a document crossing a boundary is split there."""
    seqs, cur, used = [], [], 0
    for d in doc_len:
        d = int(d)
        while d > 0:
            take = min(d, window - used)
            cur.append(take)
            used += take
            d -= take
            if used == window:
                seqs.append(cur)
                cur, used = [], 0
    if cur:
        seqs.append(cur)
    return seqs


def imbalance(values) -> float:
    """Max over mean of a list of per-micro-batch (or per-rank) workloads."""
    values = [float(x) for x in values]
    return max(values) / (sum(values) / len(values))


class StreamPacker:
    """The whole of Algorithm 1 (Section 4.3) with the outlier delay of Section 4.2, as a
    stateful object: one `step` per global batch.

    `thresholds` are the queue bounds L_1 < ... < L_n.  A document of length >= L_1 is an
    outlier and waits in queue i with L_i <= length < L_{i+1} (the last queue has no upper
    bound).  After the current batch has been read, every queue that holds at least N
    documents releases its N oldest ones (first in, first out) into the pending set, queues in
    index order.  The pending set -- left-overs of the previous iteration first, then this
    batch's ordinary documents in arrival order, then the released outliers -- is sorted by
    length (stable) and packed greedily exactly as `pack` does; what fits nowhere is carried
    over in that sorted order.

    Readings: "greater than L_1" and "L_i <= Doc_len" disagree about length == L_1; the second
    (inclusive) is used.  A queue holding 2N or more documents still releases N per iteration.
    Documents longer than l_max can never be placed and are rejected.
    """

    def __init__(self, n_microbatch: int, l_max: int, a: int, b: int, thresholds=()):
        thresholds = [int(x) for x in thresholds]
        if n_microbatch < 1 or l_max < 1 or a < 0 or b < 0:
            raise ValueError("invalid packer arguments")
        if any(t <= 0 for t in thresholds) or any(x >= y for x, y in zip(thresholds, thresholds[1:])):
            raise ValueError("thresholds must be positive and strictly increasing")
        self.n, self.l_max, self.a, self.b = n_microbatch, l_max, a, b
        self.thresholds = thresholds
        self.queues = [[] for _ in thresholds]       # FIFO lists of (doc_id, length)
        self.remained = []                           # (doc_id, length) in carried order
        self.iteration = 0

    def _queue_of(self, length):
        q = -1
        for i, t in enumerate(self.thresholds):
            if length >= t:
                q = i
        return q

    def step(self, docs):
        """docs: iterable of (doc_id, length) in arrival order.  Returns
        (placed, mb_len, mb_cost) where placed is a list of (doc_id, length, micro_batch) in
        placement (sorted) order."""
        docs = [(int(i), int(d)) for i, d in docs]
        if any(d <= 0 or d > self.l_max for _, d in docs):
            raise ValueError("document length out of range")
        pending = list(self.remained)
        for i, d in docs:
            q = self._queue_of(d)
            if q >= 0:
                self.queues[q].append((i, d))
            else:
                pending.append((i, d))
        for q in self.queues:
            if len(q) >= self.n:
                pending.extend(q[:self.n])
                del q[:self.n]
        order = sorted(range(len(pending)), key=lambda k: -pending[k][1])
        work = [0] * self.n
        length = [0] * self.n
        placed, remained = [], []
        for k in order:
            i, d = pending[k]
            w_idx = min(range(self.n), key=lambda j: (work[j], j))
            l_idx = min(range(self.n), key=lambda j: (length[j], j))
            if length[w_idx] + d <= self.l_max:
                j = w_idx
            elif length[l_idx] + d <= self.l_max:
                j = l_idx
            else:
                remained.append((i, d))
                continue
            placed.append((i, d, j))
            work[j] += cost(d, self.a, self.b)
            length[j] += d
        self.remained = remained
        self.iteration += 1
        return placed, length, work

    def pending_counts(self):
        return len(self.remained), sum(len(q) for q in self.queues)
