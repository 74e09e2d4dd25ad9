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
// Streaming packer: Algorithm 1 with the outlier waiting queues of Section 4.2.
// ---------------------------------------------------------------------------------------
struct wlb_packer {
    struct Doc { int64_t id; int32_t len; };
    int32_t n;
    int64_t l_max;
    uint64_t a, b;
    std::vector<int64_t> thresholds;
    std::vector<std::vector<Doc>> queues;   // FIFO: front = oldest
    std::vector<Doc> left_over;
};

static bool cost_fits(uint64_t cost_a, uint64_t cost_b, int64_t l_max) {
    unsigned __int128 lm = (unsigned __int128)(uint64_t)l_max;
    if (cost_a != 0 && (lm * lm) > (~(unsigned __int128)0) / cost_a) return false;
    unsigned __int128 worst = (unsigned __int128)cost_a * lm * lm + (unsigned __int128)cost_b * lm;
    return worst <= (unsigned __int128)std::numeric_limits<uint64_t>::max();
}

extern "C" wlb_status wlb_packer_create(int32_t n_microbatch, int64_t l_max, uint64_t cost_a, uint64_t cost_b,
                                        const int64_t* thresholds, int32_t n_queues, wlb_packer** out) {
    if (!out) return fail(WLB_ERR_INVALID_ARG, "wlb_packer_create: null output");
    *out = nullptr;
    if (n_microbatch < 1 || l_max < 1 || n_queues < 0 || (n_queues > 0 && !thresholds))
        return fail(WLB_ERR_INVALID_ARG, "wlb_packer_create: n_microbatch=%d l_max=%lld n_queues=%d", n_microbatch,
                    (long long)l_max, n_queues);
    if (!cost_fits(cost_a, cost_b, l_max))
        return fail(WLB_ERR_INVALID_ARG, "wlb_packer_create: cost_a*l_max^2 + cost_b*l_max overflows 64 bits");
    for (int i = 0; i < n_queues; ++i)
        if (thresholds[i] <= 0 || (i > 0 && thresholds[i] <= thresholds[i - 1]))
            return fail(WLB_ERR_INVALID_ARG, "wlb_packer_create: thresholds must be positive and strictly increasing");
    wlb_packer* p = new wlb_packer;
    p->n = n_microbatch; p->l_max = l_max; p->a = cost_a; p->b = cost_b;
    p->thresholds.assign(thresholds, thresholds + n_queues);
    p->queues.resize((size_t)n_queues);
    *out = p;
    return WLB_OK;
}

extern "C" void wlb_packer_destroy(wlb_packer* packer) { delete packer; }

extern "C" wlb_status wlb_packer_pending(const wlb_packer* packer, int64_t* n_left_over, int64_t* n_queued) {
    if (!packer || !n_left_over || !n_queued) return fail(WLB_ERR_INVALID_ARG, "wlb_packer_pending: null pointer");
    *n_left_over = (int64_t)packer->left_over.size();
    int64_t q = 0;
    for (const auto& v : packer->queues) q += (int64_t)v.size();
    *n_queued = q;
    return WLB_OK;
}

extern "C" wlb_status wlb_packer_step(wlb_packer* packer, const int32_t* doc_len, const int64_t* doc_id, int64_t n_docs,
                                      int64_t* out_doc_id, int32_t* out_doc_len, int32_t* out_mb, int64_t capacity,
                                      int64_t* n_out, int64_t* mb_len, uint64_t* mb_cost) {
    if (!packer || !n_out || !mb_len || !mb_cost || n_docs < 0 || (n_docs > 0 && (!doc_len || !doc_id)))
        return fail(WLB_ERR_INVALID_ARG, "wlb_packer_step: null pointer or negative count");
    for (int64_t i = 0; i < n_docs; ++i)
        if (doc_len[i] <= 0 || doc_len[i] > packer->l_max)
            return fail(WLB_ERR_INVALID_ARG, "wlb_packer_step: doc_len[%lld]=%d outside (0, l_max]", (long long)i, doc_len[i]);
    int64_t queued = 0;
    for (const auto& v : packer->queues) queued += (int64_t)v.size();
    const int64_t could_place = (int64_t)packer->left_over.size() + queued + n_docs;
    if (capacity < could_place || (could_place > 0 && (!out_doc_id || !out_doc_len || !out_mb)))
        return fail(WLB_ERR_BUFFER_TOO_SMALL, "wlb_packer_step: capacity %lld < %lld", (long long)capacity, (long long)could_place);

    using Doc = wlb_packer::Doc;
    std::vector<Doc> pending(packer->left_over);
    for (int64_t i = 0; i < n_docs; ++i) {
        int q = -1;
        for (size_t t = 0; t < packer->thresholds.size(); ++t)
            if (doc_len[i] >= packer->thresholds[t]) q = (int)t;
        if (q >= 0) packer->queues[(size_t)q].push_back(Doc{doc_id[i], doc_len[i]});
        else pending.push_back(Doc{doc_id[i], doc_len[i]});
    }
    for (auto& q : packer->queues)
        if ((int64_t)q.size() >= packer->n) {
            pending.insert(pending.end(), q.begin(), q.begin() + packer->n);
            q.erase(q.begin(), q.begin() + packer->n);
        }
    std::stable_sort(pending.begin(), pending.end(), [](const Doc& x, const Doc& y) { return x.len > y.len; });

    const int n = packer->n;
    for (int j = 0; j < n; ++j) { mb_len[j] = 0; mb_cost[j] = 0; }
    packer->left_over.clear();
    int64_t placed = 0;
    for (const Doc& doc : pending) {
        const uint64_t d = (uint64_t)doc.len;
        int w = 0, l = 0;
        for (int j = 1; j < n; ++j) {
            if (mb_cost[j] < mb_cost[w]) w = j;
            if (mb_len[j] < mb_len[l]) l = j;
        }
        int dst;
        if (mb_len[w] + (int64_t)d <= packer->l_max) dst = w;
        else if (mb_len[l] + (int64_t)d <= packer->l_max) dst = l;
        else { packer->left_over.push_back(doc); continue; }
        out_doc_id[placed] = doc.id;
        out_doc_len[placed] = doc.len;
        out_mb[placed] = dst;
        ++placed;
        mb_len[dst] += (int64_t)d;
        mb_cost[dst] += packer->a * d * d + packer->b * d;
    }
    *n_out = placed;
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

// ---------------------------------------------------------------------------------------
// Adaptive sharding selection (Section 5.3): padded operations / profiled rate per segment,
// summed per rank, maximum over the ranks of the CP group.  Plain IEEE double arithmetic in a
// fixed order (this file is compiled without floating-point contraction).
// ---------------------------------------------------------------------------------------
namespace {

wlb_status check_profile(const wlb_kernel_profile* t) {
    if (!t || !t->q_len || !t->kv_len || !t->tflops || t->n_q < 1 || t->n_kv < 1 || t->tile_q < 1 || t->tile_k < 1)
        return fail(WLB_ERR_INVALID_ARG, "kernel profile: null pointer, empty grid or tile < 1");
    for (int i = 0; i < t->n_q; ++i)
        if (t->q_len[i] < 1 || (i > 0 && t->q_len[i] <= t->q_len[i - 1]))
            return fail(WLB_ERR_INVALID_ARG, "kernel profile: q_len grid must be positive and strictly increasing");
    for (int i = 0; i < t->n_kv; ++i)
        if (t->kv_len[i] < 1 || (i > 0 && t->kv_len[i] <= t->kv_len[i - 1]))
            return fail(WLB_ERR_INVALID_ARG, "kernel profile: kv_len grid must be positive and strictly increasing");
    for (int64_t i = 0; i < (int64_t)t->n_q * t->n_kv; ++i)
        if (!(t->tflops[i] > 0.0)) return fail(WLB_ERR_INVALID_ARG, "kernel profile: rates must be positive");
    return WLB_OK;
}

int64_t padded_pairs(int64_t q_len, int64_t kv_len, int64_t tile_q, int64_t tile_k) {
    if (q_len <= 0 || kv_len <= 0) return 0;
    int64_t total = 0;
    const int64_t n_tiles = (q_len + tile_q - 1) / tile_q;
    for (int64_t t = 0; t < n_tiles; ++t) {
        const int64_t e = std::min((t + 1) * tile_q, q_len);
        const int64_t vis = kv_len - q_len + e;
        if (vis <= 0) continue;
        total += tile_q * ((vis + tile_k - 1) / tile_k * tile_k);
    }
    return total;
}

void bracket(const int32_t* grid, int n, int64_t x, int* i0, int* i1, double* w) {
    if (x <= grid[0]) { *i0 = *i1 = 0; *w = 0.0; return; }
    if (x >= grid[n - 1]) { *i0 = *i1 = n - 1; *w = 0.0; return; }
    int i = 0;
    while (grid[i + 1] < x) ++i;
    *i0 = i; *i1 = i + 1;
    *w = (double)(x - grid[i]) / (double)(grid[i + 1] - grid[i]);
}

double profile_lookup(const wlb_kernel_profile* t, int64_t q_len, int64_t kv_len) {
    int i0, i1, j0, j1;
    double wq, wk;
    bracket(t->q_len, t->n_q, q_len, &i0, &i1, &wq);
    bracket(t->kv_len, t->n_kv, kv_len, &j0, &j1, &wk);
    const double* T = t->tflops;
    const int nk = t->n_kv;
    const double top = T[i0 * nk + j0] * (1.0 - wk) + T[i0 * nk + j1] * wk;
    const double bot = T[i1 * nk + j0] * (1.0 - wk) + T[i1 * nk + j1] * wk;
    return top * (1.0 - wq) + bot * wq;
}

wlb_status predict(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t mode, int32_t hq, int32_t head_dim,
                   const wlb_kernel_profile* prof, double* rank_latency) {
    if (hq < 1 || head_dim < 1) return fail(WLB_ERR_INVALID_ARG, "wlb_predict_latency: hq=%d head_dim=%d", hq, head_dim);
    if (wlb_status st = check_profile(prof)) return st;
    const double flops_per_pair = 14.0 * (double)head_dim * (double)hq;
    for (int32_t r = 0; r < cp; ++r) {
        ShardArgs a{doc_len, n_docs, cp, r, mode};
        int64_t total = 0;
        if (wlb_status st = check_shard(a, &total)) return st;
        double lat = 0.0;
        walk_segments(a, total, [&](int64_t, int64_t first, int64_t slots, int64_t real) {
            const int64_t kv_len = real > 0 ? first + real : 0;
            const int64_t pairs = padded_pairs(slots, kv_len, prof->tile_q, prof->tile_k);
            if (pairs == 0) return;
            const double rate = profile_lookup(prof, slots, kv_len) * 1e12;
            lat = lat + ((double)pairs * flops_per_pair) / rate;
        });
        rank_latency[r] = lat;
    }
    return WLB_OK;
}

}  // namespace

extern "C" wlb_status wlb_predict_latency(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t mode, int32_t hq,
                                          int32_t head_dim, const wlb_kernel_profile* profile, double* rank_latency) {
    if (!rank_latency || cp < 1) return fail(WLB_ERR_INVALID_ARG, "wlb_predict_latency: null output or cp=%d", cp);
    return predict(doc_len, n_docs, cp, mode, hq, head_dim, profile, rank_latency);
}

extern "C" wlb_status wlb_select_sharding(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t hq, int32_t head_dim,
                                          const wlb_kernel_profile* profile, int32_t* mode, double* latency_per_seq,
                                          double* latency_per_doc) {
    if (!mode || !latency_per_seq || !latency_per_doc || cp < 1)
        return fail(WLB_ERR_INVALID_ARG, "wlb_select_sharding: null output or cp=%d", cp);
    std::vector<double> lat((size_t)cp);
    double worst[2];
    const int32_t modes[2] = {WLB_SHARD_PER_SEQ, WLB_SHARD_PER_DOC_PADDED};
    for (int m = 0; m < 2; ++m) {
        if (wlb_status st = predict(doc_len, n_docs, cp, modes[m], hq, head_dim, profile, lat.data())) return st;
        worst[m] = 0.0;
        for (double x : lat) if (x > worst[m]) worst[m] = x;
    }
    *latency_per_seq = worst[0];
    *latency_per_doc = worst[1];
    *mode = worst[1] < worst[0] ? WLB_SHARD_PER_DOC_PADDED : WLB_SHARD_PER_SEQ;
    return WLB_OK;
}

// ---------------------------------------------------------------------------------------
// Exact solution of Equation 2 (Section 4.1) for small inputs: depth-first branch and bound over
// the documents in descending length.  A branch is cut when its largest micro-batch cost cannot
// beat the best complete assignment; micro-batches that are still empty are interchangeable, so
// only the first of them is tried.
// ---------------------------------------------------------------------------------------
namespace {

struct OptSearch {
    int n, nb;
    int64_t l_max;
    std::vector<int64_t> len;       // documents, descending
    std::vector<uint64_t> cst;
    std::vector<int64_t> bin_len;
    std::vector<uint64_t> bin_cost;
    std::vector<int> cur, best_assign;
    uint64_t best = std::numeric_limits<uint64_t>::max();
    bool found = false;
    int64_t nodes = 0, node_limit;

    void go(int i, uint64_t cur_max) {
        if (node_limit > 0 && nodes >= node_limit) return;
        ++nodes;
        if (i == n) {
            if (!found || cur_max < best) { best = cur_max; best_assign = cur; found = true; }
            return;
        }
        bool tried_empty = false;
        for (int j = 0; j < nb; ++j) {
            if (bin_len[j] == 0) { if (tried_empty) continue; tried_empty = true; }
            if (bin_len[j] + len[i] > l_max) continue;
            const uint64_t c = bin_cost[j] + cst[i];
            const uint64_t m = std::max(cur_max, c);
            if (found && m >= best) continue;
            bin_len[j] += len[i]; bin_cost[j] = c; cur[i] = j;
            go(i + 1, m);
            bin_len[j] -= len[i]; bin_cost[j] = c - cst[i];
        }
    }
};

}  // namespace

extern "C" wlb_status wlb_pack_optimal(const int32_t* doc_len, int64_t n_docs, int32_t n_microbatch, int64_t l_max,
                                       uint64_t cost_a, uint64_t cost_b, int64_t node_limit, int32_t* assign,
                                       int64_t* mb_len, uint64_t* mb_cost, uint64_t* optimal_cost, int32_t* proven) {
    if (!doc_len || !assign || !mb_len || !mb_cost || !optimal_cost || !proven)
        return fail(WLB_ERR_INVALID_ARG, "wlb_pack_optimal: null pointer");
    if (n_docs < 1 || n_docs > 64 || n_microbatch < 1 || n_microbatch > 64 || l_max < 1)
        return fail(WLB_ERR_INVALID_ARG, "wlb_pack_optimal: n_docs=%lld (1..64) n_microbatch=%d (1..64) l_max=%lld",
                    (long long)n_docs, n_microbatch, (long long)l_max);
    if (!cost_fits(cost_a, cost_b, l_max))
        return fail(WLB_ERR_INVALID_ARG, "wlb_pack_optimal: cost_a*l_max^2 + cost_b*l_max overflows 64 bits");
    for (int64_t i = 0; i < n_docs; ++i)
        if (doc_len[i] <= 0 || doc_len[i] > l_max)
            return fail(WLB_ERR_INVALID_ARG, "wlb_pack_optimal: doc_len[%lld]=%d outside (0, l_max]", (long long)i, doc_len[i]);
    std::vector<int> order((size_t)n_docs);
    for (int i = 0; i < (int)n_docs; ++i) order[(size_t)i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return doc_len[x] > doc_len[y]; });
    OptSearch s;
    s.n = (int)n_docs; s.nb = n_microbatch; s.l_max = l_max; s.node_limit = node_limit;
    for (int i : order) {
        const uint64_t d = (uint64_t)doc_len[i];
        s.len.push_back(doc_len[i]);
        s.cst.push_back(cost_a * d * d + cost_b * d);
    }
    s.bin_len.assign((size_t)n_microbatch, 0);
    s.bin_cost.assign((size_t)n_microbatch, 0);
    s.cur.assign((size_t)n_docs, -1);
    s.go(0, 0);
    if (!s.found)
        return fail(WLB_ERR_INVALID_ARG, s.node_limit > 0 && s.nodes >= s.node_limit
                        ? "wlb_pack_optimal: node limit reached before any complete assignment"
                        : "wlb_pack_optimal: no assignment keeps every micro-batch within l_max");
    for (int j = 0; j < n_microbatch; ++j) { mb_len[j] = 0; mb_cost[j] = 0; }
    for (int k = 0; k < (int)n_docs; ++k) {
        const int i = order[(size_t)k], j = s.best_assign[(size_t)k];
        assign[i] = j;
        mb_len[j] += s.len[(size_t)k];
        mb_cost[j] += s.cst[(size_t)k];
    }
    *optimal_cost = s.best;
    *proven = !(s.node_limit > 0 && s.nodes >= s.node_limit);
    return WLB_OK;
}
