// Host side of libwlb: error text, the greedy variable-length packer and the
// context-parallel sharding maps.  Integer-only, synchronous, no device work.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#include "wlb_internal.h"

namespace wlb {

static thread_local char g_err[512] = "";

wlb_status fail(wlb_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

}  // namespace wlb

using wlb::fail;

extern "C" const char* wlb_last_error(void) { return wlb::g_err; }

// ---------------------------------------------------------------------------------------
// Packing: greedy core of Algorithm 1 (Section 4.3) under the cost model of Equation 2.
// ---------------------------------------------------------------------------------------
extern "C" wlb_status wlb_pack(const int32_t* doc_len, int64_t n_docs, int32_t n_microbatch,
                               int64_t l_max, uint64_t cost_a, uint64_t cost_b, int32_t* assign,
                               int64_t* mb_len, uint64_t* mb_cost) {
    if (n_docs < 0 || n_microbatch < 1 || l_max < 1)
        return fail(WLB_ERR_INVALID_ARG, "wlb_pack: n_docs=%lld n_microbatch=%d l_max=%lld",
                    (long long)n_docs, n_microbatch, (long long)l_max);
    if (!mb_len || !mb_cost || (n_docs > 0 && (!doc_len || !assign)))
        return fail(WLB_ERR_INVALID_ARG, "wlb_pack: null pointer");
    // a full micro-batch must be representable: a*l_max^2 + b*l_max < 2^64
    {
        unsigned __int128 lm = (unsigned __int128)(uint64_t)l_max;
        unsigned __int128 worst = (unsigned __int128)cost_a * lm * lm + (unsigned __int128)cost_b * lm;
        bool a_over = cost_a != 0 && (lm * lm) > (~(unsigned __int128)0) / cost_a;
        if (a_over || worst > (unsigned __int128)std::numeric_limits<uint64_t>::max())
            return fail(WLB_ERR_INVALID_ARG, "wlb_pack: cost_a*l_max^2 + cost_b*l_max overflows 64 bits");
    }
    for (int64_t i = 0; i < n_docs; ++i)
        if (doc_len[i] <= 0)
            return fail(WLB_ERR_INVALID_ARG, "wlb_pack: doc_len[%lld]=%d is not positive", (long long)i, doc_len[i]);

    std::vector<int64_t> order((size_t)n_docs);
    std::iota(order.begin(), order.end(), (int64_t)0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t x, int64_t y) { return doc_len[x] > doc_len[y]; });

    const int n = n_microbatch;
    for (int j = 0; j < n; ++j) { mb_len[j] = 0; mb_cost[j] = 0; }
    for (int64_t i : order) {
        const uint64_t d = (uint64_t)doc_len[i];
        if ((int64_t)d > l_max) { assign[i] = -1; continue; }   // can never fit; also keeps costs in range
        int w = 0, l = 0;
        for (int j = 1; j < n; ++j) {
            if (mb_cost[j] < mb_cost[w]) w = j;
            if (mb_len[j] < mb_len[l]) l = j;
        }
        int dst;
        if (mb_len[w] + (int64_t)d <= l_max) dst = w;
        else if (mb_len[l] + (int64_t)d <= l_max) dst = l;
        else { assign[i] = -1; continue; }
        assign[i] = dst;
        mb_len[dst] += (int64_t)d;
        mb_cost[dst] += cost_a * d * d + cost_b * d;
    }
    return WLB_OK;
}

// ---------------------------------------------------------------------------------------
// Sharding maps (Section 3.1 per-sequence; Section 5.1 per-document with tail padding).
// ---------------------------------------------------------------------------------------
namespace {

struct ShardArgs {
    const int32_t* doc_len; int64_t n_docs; int32_t cp, rank, mode;
};

wlb_status check_shard(const ShardArgs& a, int64_t* total_out) {
    if (!a.doc_len || a.n_docs < 1) return fail(WLB_ERR_INVALID_ARG, "wlb_shard: no documents");
    if (a.cp < 1 || a.rank < 0 || a.rank >= a.cp)
        return fail(WLB_ERR_INVALID_ARG, "wlb_shard: cp=%d rank=%d", a.cp, a.rank);
    if (a.mode != WLB_SHARD_PER_DOC_PADDED && a.mode != WLB_SHARD_PER_SEQ && a.mode != WLB_SHARD_PER_DOC_NOPAD)
        return fail(WLB_ERR_INVALID_ARG, "wlb_shard: unknown mode %d", a.mode);
    int64_t total = 0, padded = 0;
    const int64_t n = 2 * (int64_t)a.cp;
    for (int64_t i = 0; i < a.n_docs; ++i) {
        if (a.doc_len[i] <= 0)
            return fail(WLB_ERR_INVALID_ARG, "wlb_shard: doc_len[%lld]=%d is not positive", (long long)i, a.doc_len[i]);
        total += a.doc_len[i];
        padded += (a.doc_len[i] + n - 1) / n * n;
    }
    if (total > std::numeric_limits<int32_t>::max() || padded > std::numeric_limits<int32_t>::max())
        return fail(WLB_ERR_UNSUPPORTED, "wlb_shard: %lld tokens do not fit int32 indices", (long long)total);
    if (a.cp > 1 && a.mode == WLB_SHARD_PER_SEQ && total % n != 0)
        return fail(WLB_ERR_INVALID_ARG, "wlb_shard: per-sequence sharding needs 2*cp | T (T=%lld, cp=%d)",
                    (long long)total, a.cp);
    *total_out = total;
    return WLB_OK;
}

// Walks the rank's segments in slot order and calls emit(doc_start, first_pos, n_slots, n_real):
// the segment's slots are document positions first_pos .. first_pos+n_slots-1 of the document
// starting at doc_start, of which the first n_real exist (the rest are padding).
template <class Emit>
void walk_segments(const ShardArgs& a, int64_t total, Emit emit) {
    const int64_t n = 2 * (int64_t)a.cp;
    if (a.cp == 1) {
        int64_t s = 0;
        for (int64_t d = 0; d < a.n_docs; ++d) { emit(s, (int64_t)0, (int64_t)a.doc_len[d], (int64_t)a.doc_len[d]); s += a.doc_len[d]; }
    } else if (a.mode == WLB_SHARD_PER_DOC_PADDED) {
        int64_t s = 0;
        for (int64_t d = 0; d < a.n_docs; ++d) {
            const int64_t L = a.doc_len[d], c = (L + n - 1) / n;
            const int64_t chunks[2] = {a.rank, n - 1 - a.rank};
            for (int64_t m : chunks) {
                const int64_t first = m * c;
                const int64_t real = std::max<int64_t>(0, std::min(L, first + c) - first);
                emit(s, first, c, real);
            }
            s += L;
        }
    } else if (a.mode == WLB_SHARD_PER_DOC_NOPAD) {
        // Section 5.1, "Avoid Padding": the part of a document divisible by 2*cp is sharded like a
        // document of that length; its last L mod 2*cp tokens are dealt round-robin, one counter
        // running on across documents.
        int64_t s = 0, t = 0;
        for (int64_t d = 0; d < a.n_docs; ++d) {
            const int64_t L = a.doc_len[d], c = L / n;
            if (c > 0) {
                emit(s, a.rank * c, c, c);
                emit(s, (n - 1 - a.rank) * c, c, c);
            }
            int64_t run_first = -1, run_len = 0;
            for (int64_t p = c * n; p < L; ++p, ++t) {
                if (t % a.cp != a.rank) continue;
                if (run_len > 0 && run_first + run_len != p) { emit(s, run_first, run_len, run_len); run_len = 0; }
                if (run_len == 0) run_first = p;
                ++run_len;
            }
            if (run_len > 0) emit(s, run_first, run_len, run_len);
            s += L;
        }
    } else {
        const int64_t c = total / n;
        const int64_t chunks[2] = {a.rank, n - 1 - a.rank};
        for (int64_t m : chunks) {
            const int64_t lo = m * c, hi = lo + c;
            int64_t s = 0;
            for (int64_t d = 0; d < a.n_docs && s < hi; ++d) {
                const int64_t e = s + a.doc_len[d];
                const int64_t x = std::max(lo, s), y = std::min(hi, e);
                if (x < y) emit(s, x - s, y - x, y - x);
                s = e;
            }
        }
    }
}

}  // namespace

extern "C" wlb_status wlb_shard_size(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t rank,
                                     int32_t mode, int64_t* n_q, int64_t* n_seg) {
    ShardArgs a{doc_len, n_docs, cp, rank, mode};
    int64_t total = 0;
    if (wlb_status st = check_shard(a, &total)) return st;
    if (!n_q || !n_seg) return fail(WLB_ERR_INVALID_ARG, "wlb_shard_size: null output");
    int64_t q = 0, s = 0;
    walk_segments(a, total, [&](int64_t, int64_t, int64_t slots, int64_t) { q += slots; ++s; });
    *n_q = q;
    *n_seg = s;
    return WLB_OK;
}

extern "C" wlb_status wlb_shard(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t rank, int32_t mode,
                                int32_t* q_idx, int32_t* cu_seqlens_q, int32_t* seg_k_begin,
                                int32_t* seg_k_end, int32_t* cu_seqlens_k, int64_t* useful_pairs) {
    ShardArgs a{doc_len, n_docs, cp, rank, mode};
    int64_t total = 0;
    if (wlb_status st = check_shard(a, &total)) return st;
    if (!q_idx) return fail(WLB_ERR_INVALID_ARG, "wlb_shard: null q_idx");
    int64_t slot = 0, seg = 0, pairs = 0;
    walk_segments(a, total, [&](int64_t doc_start, int64_t first, int64_t slots, int64_t real) {
        for (int64_t p = 0; p < slots; ++p)
            q_idx[slot + p] = p < real ? (int32_t)(doc_start + first + p) : -1;
        if (cu_seqlens_q) cu_seqlens_q[seg] = (int32_t)slot;
        if (seg_k_begin) seg_k_begin[seg] = (int32_t)doc_start;
        if (seg_k_end) seg_k_end[seg] = (int32_t)(real > 0 ? doc_start + first + real : doc_start);
        // rows at document positions first .. first+real-1 see position+1 keys each
        pairs += real * first + real * (real + 1) / 2;
        slot += slots;
        ++seg;
    });
    if (cu_seqlens_q) cu_seqlens_q[seg] = (int32_t)slot;
    if (cu_seqlens_k) {
        int64_t s = 0;
        for (int64_t d = 0; d < n_docs; ++d) { cu_seqlens_k[d] = (int32_t)s; s += doc_len[d]; }
        cu_seqlens_k[n_docs] = (int32_t)s;
    }
    if (useful_pairs) *useful_pairs = pairs;
    return WLB_OK;
}
