// Attention entry points of libwlb and the device-side tile scheduler.
//
// The scheduler turns (q_idx, cu_seqlens_k) into the integer tables the attention kernels
// read: for every local row the interval [lo, hi) of keys it may see (its document's start up
// to and including itself: causal inside the document, nothing outside -- paper Sections 1 and
// 3.2); for every group of 64 consecutive rows the hull of those intervals and the range every
// real row of the group sees in full; and two work lists ordered heaviest first -- query tiles
// (forward and dQ) and key tiles (dK/dV).  Kernels visit only key tiles inside a hull and
// apply the per-element mask only outside the fully visible range, which is how tiles that lie
// wholly in other documents cost nothing (the tile-level waste described in Section 5.2).
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "wlb_device.h"
#include "wlb_internal.h"

namespace wlb {

wlb_status check_desc(const wlb_attn_desc* d) {
    if (!d) return fail(WLB_ERR_INVALID_ARG, "attention: null desc");
    if (d->n_q < 1 || d->t_kv < 1 || d->n_docs < 1 || d->hq < 1 || d->hkv < 1)
        return fail(WLB_ERR_INVALID_ARG, "attention: n_q=%d t_kv=%d n_docs=%d hq=%d hkv=%d", d->n_q, d->t_kv,
                    d->n_docs, d->hq, d->hkv);
    if (d->hq % d->hkv != 0) return fail(WLB_ERR_INVALID_ARG, "attention: hq=%d not a multiple of hkv=%d", d->hq, d->hkv);
    if (d->visible_pairs < 0) return fail(WLB_ERR_INVALID_ARG, "attention: visible_pairs=%lld", (long long)d->visible_pairs);
    if ((d->flags & WLB_ATTN_SCHEDULE_GANGS) && (d->flags & WLB_ATTN_SCHEDULE_ITEMS))
        return fail(WLB_ERR_INVALID_ARG, "attention: both schedule flags set");
    if (!(d->scale > 0.0f) || !std::isfinite(d->scale)) return fail(WLB_ERR_INVALID_ARG, "attention: scale must be finite and > 0");
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(WLB_ERR_UNSUPPORTED, "attention: head_dim=%d (64 and 128 are built)", d->head_dim);
    const int64_t qe = (int64_t)d->n_q * d->hq * d->head_dim, ke = (int64_t)d->t_kv * d->hkv * d->head_dim;
    // tensors are addressed through 32-bit buffer descriptors: each must stay under 4 GiB, with
    // room for the offsets of the rows a last, partly filled tile would have past the end
    const int64_t q_margin = 2LL * kBwdKeyTile * d->hq * d->head_dim, k_margin = 2LL * kBwdKeyTile * d->hkv * d->head_dim;
    if (qe * 2 + q_margin >= (1LL << 32) || ke * 2 + k_margin >= (1LL << 32))
        return fail(WLB_ERR_UNSUPPORTED, "attention: a tensor of 4 GiB or more is not supported");
    if (d->flags & ~(WLB_ATTN_REUSE_PLAN | WLB_ATTN_BWD_SKIP_DELTA | WLB_ATTN_BWD_SKIP_DQ | WLB_ATTN_BWD_SKIP_DKV | WLB_ATTN_SCHEDULE_GANGS | WLB_ATTN_SCHEDULE_ITEMS | WLB_ATTN_NO_SHORT_PATH)) return fail(WLB_ERR_INVALID_ARG, "attention: unknown flag bits 0x%x", d->flags);
    return WLB_OK;
}

int compute_units() {
    static int cached = 0;          // the library runs on one kind of GPU per process
    if (cached == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        cached = cus;
    }
    return cached;
}

size_t dkv_partial_bytes(const wlb_attn_desc& d, const wlb_plan_layout& L) {
    // one fp32 dK^T and dV^T tile per partial result
    return (size_t)L.dkv_max_partials * (2 * (size_t)kBwdKeyTile * d.head_dim * sizeof(float));
}

bool use_row_gangs(const wlb_attn_desc& d, const wlb_plan_layout& L) {
    if (d.flags & WLB_ATTN_SCHEDULE_GANGS) return true;
    if (d.flags & WLB_ATTN_SCHEDULE_ITEMS) return false;
    const long long items = (long long)L.n_fwd_tiles * d.hq, slots = 2LL * compute_units();
    if (items >= (long long)kRowGangMaxItemsPerSlot * slots) return false;
    // and only when a slot's share is worth cutting tiles for.  The work line's length in key tiles per item:
    // from the caller's pair count when it gave one (a tile of 128 rows x 64 keys holds 8192 pairs), else
    // estimated from the mean document length (a tile sees about half its document: length / 128 key tiles),
    // since the host does not see the mask
    const long long per_item = (d.visible_pairs > 0 ? d.visible_pairs / ((long long)L.n_fwd_tiles * kFwdTileRows * 64)
                                                    : (long long)(d.t_kv / d.n_docs / (2 * 64))) + kRowItemOverhead;
    return items * per_item >= (long long)kRowGangMinUnitsPerSlot * slots;
}

// gang share weights: process-wide, set by wlb_attn_set_gang_weights (0 = not set: the defaults)
static int g_gang_weight[2][2][8];
static std::mutex g_gang_weight_mutex;

void gang_weights(int kernel, int out[2][8]) {
    std::lock_guard<std::mutex> lock(g_gang_weight_mutex);
    const int first = kernel == 0 ? kRowShareFirstFwd : kRowShareFirstDq;
    for (int h = 0; h < 2; ++h)
        for (int x = 0; x < 8; ++x)
            out[h][x] = g_gang_weight[kernel][0][0] > 0 ? g_gang_weight[kernel][h][x] : (h == 0 ? first : 100 - first);
}

bool use_short_path(const wlb_attn_desc& d, const wlb_plan_layout& L) {
    return !(d.flags & WLB_ATTN_NO_SHORT_PATH) && !use_row_gangs(d, L);
}

size_t row_partial_bytes(const wlb_attn_desc& d, const wlb_plan_layout& L) {
    return (size_t)2 * L.row_gangs * (d.hq / d.hkv) * row_partial_floats(d.head_dim) * sizeof(float);
}

void plan_layout(const wlb_attn_desc& d, wlb_plan_layout* L) {
    L->group_rows = kGroupRows;
    L->n_groups = (d.n_q + kGroupRows - 1) / kGroupRows;
    L->fwd_tile_rows = kFwdTileRows;
    L->n_fwd_tiles = (d.n_q + kFwdTileRows - 1) / kFwdTileRows;
    L->bwd_key_tile = kBwdKeyTile;
    L->n_key_tiles = (d.t_kv + kBwdKeyTile - 1) / kBwdKeyTile;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L->off_row_lo = take(sizeof(int32_t) * d.n_q);
    L->off_row_hi = take(sizeof(int32_t) * d.n_q);
    L->off_group = take(sizeof(int32_t) * 4 * L->n_groups);
    L->off_group_real = take(sizeof(int32_t) * L->n_groups);
    L->off_fwd_order = take(sizeof(int32_t) * L->n_fwd_tiles);
    L->off_fwd_cost = take(sizeof(int32_t) * L->n_fwd_tiles);
    L->off_key_order = take(sizeof(int32_t) * L->n_key_tiles);
    L->off_key_range = take(sizeof(int32_t) * 2 * L->n_key_tiles);
    size_t key_cost = take(sizeof(int32_t) * L->n_key_tiles);   // scratch for the ordering
    (void)key_cost;
    // Items per tile are the smallest power of two that brings an item under 1/kDkvSplit of a compute
    // unit's mean load, so split tiles contribute fewer than 2 * kDkvSplit * CUs items in total.
    L->dkv_max_partials = 2 * kDkvSplit * compute_units();
    L->dkv_max_items = L->n_key_tiles * d.hkv + L->dkv_max_partials;
    L->off_key_ways = take(sizeof(int32_t) * L->n_key_tiles);
    L->off_key_item_base = take(sizeof(int32_t) * (L->n_key_tiles + 1));
    L->off_key_slot_base = take(sizeof(int32_t) * (L->n_key_tiles + 1));
    L->off_dkv_counters = take(sizeof(int32_t) * kLists);
    L->row_gangs = row_gangs(d.hq, d.hkv, compute_units());
    L->uses_gangs = use_row_gangs(d, *L) ? 1 : 0;
    L->off_fwd_prefix = take(sizeof(int64_t) * (L->n_fwd_tiles + 1));
    L->n_blocks32 = L->n_groups * (kGroupRows / kShortBlockRows);
    L->off_block_hull = take(sizeof(int32_t) * 2 * L->n_blocks32);
    L->off_tile_short = take(sizeof(int32_t) * L->n_fwd_tiles);
    L->off_gang_clock = take(sizeof(uint64_t) * 2 * 2 * (size_t)L->row_gangs * (d.hq / d.hkv));
    L->plan_bytes = off;
}

static size_t off_key_cost(const wlb_plan_layout& L) {
    return align_up(L.off_key_range + sizeof(int32_t) * 2 * L.n_key_tiles, 256);
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_min(int v) {
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_max(int v) {
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_sum(int v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// One wavefront per group of 64 rows: per-row [lo, hi) and the group's {k_lo, k_hi, max_lo, min_hi}.
__global__ void __launch_bounds__(256) plan_rows_kernel(const int32_t* __restrict__ q_idx,
                                                        const int32_t* __restrict__ cu, int n_q, int t_kv,
                                                        int n_docs, int n_groups, int32_t* __restrict__ row_lo,
                                                        int32_t* __restrict__ row_hi, int32_t* __restrict__ group,
                                                        int32_t* __restrict__ group_real, int32_t* __restrict__ block_hull) {
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= n_groups) return;
    const int i = g * kGroupRows + lane;
    int lo = kPadLo, hi = 0;
    if (i < n_q) {
        const int tok = q_idx[i];
        if (tok >= 0 && tok < t_kv) {
            // last document start <= tok
            int a = 0, b = n_docs;   // invariant: cu[a] <= tok < cu[b]
            while (b - a > 1) {
                const int m = (a + b) >> 1;
                if (cu[m] <= tok) a = m; else b = m;
            }
            lo = cu[a];
            hi = tok + 1;
        }
        row_lo[i] = lo;
        row_hi[i] = hi;
    }
    const bool real = hi > 0;
    // hull of each half of the wavefront (a block of 32 rows), then of the whole group
    int b_lo = lo, b_hi = hi;                            // pads carry INT_MAX / 0
    for (int o = 16; o > 0; o >>= 1) {
        b_lo = min(b_lo, __shfl_xor(b_lo, o));
        b_hi = max(b_hi, __shfl_xor(b_hi, o));
    }
    if ((lane & 31) == 0) {
        const int b = g * (kGroupRows / kShortBlockRows) + (lane >> 5);
        block_hull[2 * b] = b_hi > 0 ? b_lo : 0;
        block_hull[2 * b + 1] = b_hi;
    }
    const int k_lo = min(b_lo, __shfl_xor(b_lo, 32));
    const int k_hi = max(b_hi, __shfl_xor(b_hi, 32));
    const int max_lo = wave_max(real ? lo : 0);
    const int min_hi = wave_min(real ? hi : kPadLo);
    if (lane == 0) {
        int4 out;
        if (k_hi == 0) out = make_int4(0, 0, 0, 0);      // no real row in this group
        else out = make_int4(k_lo, k_hi, max_lo, min_hi);
        reinterpret_cast<int4*>(group)[g] = out;
    }
    const int n_real = wave_sum(real ? 1 : 0);
    if (lane == 0) group_real[g] = n_real;
}

// cost of a forward tile = number of 64-key tiles between the hull's ends
__device__ __forceinline__ void fwd_cost_of_tile(const int32_t* __restrict__ group, int n_groups, int n_tiles,
                                                 int groups_per_tile, int32_t* __restrict__ cost,
                                                 const int32_t* __restrict__ block_hull, int32_t* __restrict__ tile_short, int t) {
    if (t >= n_tiles) return;
    {
        // short-hull tile: every block of 32 rows that has a real row sees keys inside one window of
        // kShortHullKeys keys that starts at a multiple of 32
        constexpr int per_tile = kFwdTileRows / kShortBlockRows, per_group = kGroupRows / kShortBlockRows;
        bool is_short = true;
        for (int j = 0; j < per_tile; ++j) {
            const int b = t * per_tile + j;
            if (b >= n_groups * per_group) break;
            const int lo = block_hull[2 * b], hi = block_hull[2 * b + 1];
            if (hi > lo && hi - (lo & ~31) > kShortHullKeys) is_short = false;
        }
        tile_short[t] = is_short ? 1 : 0;
    }
    int k_lo = kPadLo, k_hi = 0;
    for (int j = 0; j < groups_per_tile; ++j) {
        const int g = t * groups_per_tile + j;
        if (g >= n_groups) break;
        const int4 d = reinterpret_cast<const int4*>(group)[g];
        if (d.y > d.x) { k_lo = min(k_lo, d.x); k_hi = max(k_hi, d.y); }
    }
    cost[t] = k_hi > k_lo ? (k_hi + 63) / 64 - k_lo / 64 : 0;
}

// One wavefront per key tile: which groups have a hull that touches it.
__device__ __forceinline__ void groups_of_key_tile(const int32_t* __restrict__ group, int n_groups, int n_key_tiles,
                                                   int key_tile, int t_kv, int32_t* __restrict__ key_range,
                                                   int32_t* __restrict__ key_cost, int kt) {
    const int lane = threadIdx.x & 63;
    if (kt >= n_key_tiles) return;
    const int k0 = kt * key_tile, k1 = min(k0 + key_tile, t_kv);
    int first = kPadLo, last = 0, cnt = 0;
    for (int g = lane; g < n_groups; g += 64) {
        const int4 d = reinterpret_cast<const int4*>(group)[g];
        if (d.y > d.x && d.x < k1 && d.y > k0) { first = min(first, g); last = max(last, g + 1); ++cnt; }
    }
    first = wave_min(first);
    last = wave_max(last);
    cnt = wave_sum(cnt);
    if (lane == 0) {
        key_range[2 * kt] = cnt ? first : 0;
        key_range[2 * kt + 1] = cnt ? last : 0;
        key_cost[kt] = cnt;
    }
}

// Both read only the group table: the first fwd_blocks workgroups take the forward tiles (one per
// thread), the others the key tiles (one per wavefront).
__global__ void __launch_bounds__(256) plan_costs_kernel(const int32_t* __restrict__ group, int n_groups, int n_tiles,
                                                         int groups_per_tile, int32_t* __restrict__ fwd_cost,
                                                         int fwd_blocks, int n_key_tiles, int key_tile, int t_kv,
                                                         int32_t* __restrict__ key_range, int32_t* __restrict__ key_cost,
                                                         const int32_t* __restrict__ block_hull,
                                                         int32_t* __restrict__ tile_short) {
    if ((int)blockIdx.x < fwd_blocks)
        fwd_cost_of_tile(group, n_groups, n_tiles, groups_per_tile, fwd_cost, block_hull, tile_short,
                         blockIdx.x * 256 + threadIdx.x);
    else
        groups_of_key_tile(group, n_groups, n_key_tiles, key_tile, t_kv, key_range, key_cost,
                           ((int)blockIdx.x - fwd_blocks) * 4 + (threadIdx.x >> 6));
}

// order[rank] = index, heaviest first, ties by index (a counting rank; n is at most a few thousand).
// A workgroup ranks kOrderPerBlock elements: wavefront w compares them with every (waves)th quad of
// costs, which pass through LDS in chunks, and the partial ranks are summed in LDS.  (One element per
// thread kept the n^2 comparisons on very few compute units: 40 us for 1024 key tiles.)
constexpr int kOrderPerBlock = 64;
__device__ __forceinline__ void order_block(const int32_t* __restrict__ cost, int n, int32_t* __restrict__ order, int block) {
    constexpr int CHUNK = 2048;
    __shared__ __attribute__((aligned(16))) int s_cost[CHUNK];
    __shared__ int s_rank[kOrderPerBlock];
    const int e = threadIdx.x % kOrderPerBlock, seg = threadIdx.x / kOrderPerBlock, n_seg = blockDim.x / kOrderPerBlock;
    const int i = block * kOrderPerBlock + e;
    const int c = i < n ? cost[i] : 0;
    if (threadIdx.x < kOrderPerBlock) s_rank[threadIdx.x] = 0;
    int rank = 0;
    for (int j0 = 0; j0 < n; j0 += CHUNK) {
        const int m = min(CHUNK, n - j0);
        __syncthreads();
        // past the end: a cost below every real one (costs are >= 0), so it never counts
        for (int j = threadIdx.x; j < CHUNK; j += blockDim.x) s_cost[j] = j < m ? cost[j0 + j] : -1;
        __syncthreads();
        // entries before i win ties: an entry counts if its cost exceeds c - 1 before i, c from i on
        for (int j = 4 * seg; j < m; j += 4 * n_seg) {
            const int4 cj = *reinterpret_cast<const int4*>(&s_cost[j]);
            const int g = j0 + j;
            rank += (cj.x > c - (g + 0 < i)) + (cj.y > c - (g + 1 < i)) + (cj.z > c - (g + 2 < i)) + (cj.w > c - (g + 3 < i));
        }
    }
    atomicAdd(&s_rank[e], rank);
    __syncthreads();
    if (seg == 0 && i < n) order[s_rank[e]] = i;
}

// One workgroup.  Chooses how many items each key tile is split into and replaces the tile's
// cost by its item cost (groups in range x heads per item), the key the tiles are then ordered by.
__device__ __forceinline__ void key_split_block(const int32_t* __restrict__ key_range, int n_key_tiles, int hq, int hkv,
                                                int n_slots, int32_t* __restrict__ ways, int32_t* __restrict__ item_cost) {
    __shared__ long long part[1024];
    long long sum = 0;
    for (int kt = threadIdx.x; kt < n_key_tiles; kt += 1024) sum += key_range[2 * kt + 1] - key_range[2 * kt];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    const int G = hq / hkv;
    const long long total_stages = part[0] * hq;
    // An item of a few dozen stages is not worth splitting: its partial results and the fix-up pass
    // cost more than the shorter tail saves (small-document inputs: 0.55 -> 0.48 ms with the minimum).
    const long long thr = max((long long)kDkvMinItemStages, (total_stages + (long long)n_slots * kDkvSplit - 1) / ((long long)n_slots * kDkvSplit));
    for (int kt = threadIdx.x; kt < n_key_tiles; kt += 1024) {
        const int span = key_range[2 * kt + 1] - key_range[2 * kt];
        int w = 1;
        while (w < G && (long long)span * (G / w) > thr && G % (2 * w) == 0) w *= 2;
        ways[kt] = w;
        item_cost[kt] = span * (G / w);
    }
}

// One workgroup.  Exclusive prefix sums, by order rank, of the tiles' item counts and partial slots.
__global__ void __launch_bounds__(1024) plan_key_bases_kernel(const int32_t* __restrict__ key_order,
                                                              const int32_t* __restrict__ ways, int n_key_tiles, int hkv,
                                                              int32_t* __restrict__ item_base, int32_t* __restrict__ slot_base,
                                                              int32_t* __restrict__ dkv_counters) {
    __shared__ int s_items[1024], s_slots[1024];
    if (threadIdx.x < kLists) dkv_counters[threadIdx.x] = 0;
    const int per = (n_key_tiles + 1023) / 1024;
    const int r0 = threadIdx.x * per, r1 = min(r0 + per, n_key_tiles);
    int items = 0, slots = 0;
    for (int r = r0; r < r1; ++r) {
        const int w = ways[key_order[r]];
        items += w * hkv;
        slots += w > 1 ? w * hkv : 0;
    }
    s_items[threadIdx.x] = items;
    s_slots[threadIdx.x] = slots;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 1024 per-thread totals
    for (int o = 1; o < 1024; o <<= 1) {
        const int a = (int)threadIdx.x >= o ? s_items[threadIdx.x - o] : 0;
        const int b = (int)threadIdx.x >= o ? s_slots[threadIdx.x - o] : 0;
        __syncthreads();
        s_items[threadIdx.x] += a;
        s_slots[threadIdx.x] += b;
        __syncthreads();
    }
    int ib = s_items[threadIdx.x] - items, sb = s_slots[threadIdx.x] - slots;
    for (int r = r0; r < r1; ++r) {
        item_base[r] = ib;
        slot_base[r] = sb;
        const int w = ways[key_order[r]];
        ib += w * hkv;
        sb += w > 1 ? w * hkv : 0;
    }
    if (threadIdx.x == 1023) { item_base[n_key_tiles] = s_items[1023]; slot_base[n_key_tiles] = s_slots[1023]; }
}

// One workgroup.  prefix[r] = cost (key tiles + the fixed kRowItemOverhead each) of the query tiles of order rank < r.
__device__ __forceinline__ void fwd_prefix_block(const int32_t* __restrict__ order, const int32_t* __restrict__ cost,
                                                 int n_tiles, long long* __restrict__ prefix) {
    __shared__ long long s_sum[1024];
    const int per = (n_tiles + 1023) / 1024;
    const int r0 = min((int)threadIdx.x * per, n_tiles), r1 = min(r0 + per, n_tiles);
    long long mine = 0;
    for (int r = r0; r < r1; ++r) mine += cost[order[r]] + kRowItemOverhead;
    s_sum[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const long long add = (int)threadIdx.x >= o ? s_sum[threadIdx.x - o] : 0;
        __syncthreads();
        s_sum[threadIdx.x] += add;
        __syncthreads();
    }
    long long run = s_sum[threadIdx.x] - mine;
    for (int r = r0; r < r1; ++r) {
        prefix[r] = run;
        run += cost[order[r]] + kRowItemOverhead;
    }
    if (threadIdx.x == 1023) prefix[n_tiles] = s_sum[1023];
}

// Workgroups [0, order_blocks) rank the forward tiles; the one after them splits the key tiles
// (neither needs the other's result).
__global__ void __launch_bounds__(1024) plan_fwd_order_key_split_kernel(const int32_t* __restrict__ fwd_cost, int n_tiles,
                                                                        int32_t* __restrict__ fwd_order, int order_blocks,
                                                                        const int32_t* __restrict__ key_range,
                                                                        int n_key_tiles, int hq, int hkv, int n_slots,
                                                                        int32_t* __restrict__ ways,
                                                                        int32_t* __restrict__ item_cost) {
    if ((int)blockIdx.x < order_blocks) order_block(fwd_cost, n_tiles, fwd_order, blockIdx.x);
    else key_split_block(key_range, n_key_tiles, hq, hkv, n_slots, ways, item_cost);
}

// Workgroups [0, order_blocks) rank the key tiles by item cost; the one after them builds the
// forward work line's prefix sums.
__global__ void __launch_bounds__(1024) plan_key_order_fwd_prefix_kernel(const int32_t* __restrict__ key_cost,
                                                                         int n_key_tiles, int32_t* __restrict__ key_order,
                                                                         int order_blocks,
                                                                         const int32_t* __restrict__ fwd_order,
                                                                         const int32_t* __restrict__ fwd_cost, int n_tiles,
                                                                         long long* __restrict__ prefix) {
    if ((int)blockIdx.x < order_blocks) order_block(key_cost, n_key_tiles, key_order, blockIdx.x);
    else fwd_prefix_block(fwd_order, fwd_cost, n_tiles, prefix);
}

wlb_status launch_plan(const wlb_attn_desc& d, const wlb_plan_layout& L, const int32_t* q_idx,
                       const int32_t* cu_seqlens_k, char* ws, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    int32_t* row_lo = (int32_t*)(ws + L.off_row_lo);
    int32_t* row_hi = (int32_t*)(ws + L.off_row_hi);
    int32_t* group = (int32_t*)(ws + L.off_group);
    int32_t* group_real = (int32_t*)(ws + L.off_group_real);
    int32_t* fwd_order = (int32_t*)(ws + L.off_fwd_order);
    int32_t* fwd_cost = (int32_t*)(ws + L.off_fwd_cost);
    int32_t* key_order = (int32_t*)(ws + L.off_key_order);
    int32_t* key_range = (int32_t*)(ws + L.off_key_range);
    int32_t* key_cost = (int32_t*)(ws + off_key_cost(L));
    plan_rows_kernel<<<(L.n_groups + 3) / 4, 256, 0, stream>>>(q_idx, cu_seqlens_k, d.n_q, d.t_kv, d.n_docs,
                                                                L.n_groups, row_lo, row_hi, group, group_real,
                                                                (int32_t*)(ws + L.off_block_hull));
    int32_t* key_ways = (int32_t*)(ws + L.off_key_ways);
    const int fwd_cost_blocks = (L.n_fwd_tiles + 255) / 256, key_tile_blocks = (L.n_key_tiles + 3) / 4;
    plan_costs_kernel<<<fwd_cost_blocks + key_tile_blocks, 256, 0, stream>>>(
        group, L.n_groups, L.n_fwd_tiles, kFwdTileRows / kGroupRows, fwd_cost, fwd_cost_blocks, L.n_key_tiles,
        kBwdKeyTile, d.t_kv, key_range, key_cost, (const int32_t*)(ws + L.off_block_hull),
        (int32_t*)(ws + L.off_tile_short));
    const int fwd_order_blocks = (L.n_fwd_tiles + kOrderPerBlock - 1) / kOrderPerBlock;
    const int key_order_blocks = (L.n_key_tiles + kOrderPerBlock - 1) / kOrderPerBlock;
    plan_fwd_order_key_split_kernel<<<fwd_order_blocks + 1, 1024, 0, stream>>>(
        fwd_cost, L.n_fwd_tiles, fwd_order, fwd_order_blocks, key_range, L.n_key_tiles, d.hq, d.hkv, compute_units(),
        key_ways, key_cost);
    plan_key_order_fwd_prefix_kernel<<<key_order_blocks + 1, 1024, 0, stream>>>(
        key_cost, L.n_key_tiles, key_order, key_order_blocks, fwd_order, fwd_cost, L.n_fwd_tiles,
        (long long*)(ws + L.off_fwd_prefix));
    plan_key_bases_kernel<<<1, 1024, 0, stream>>>(key_order, key_ways, L.n_key_tiles, d.hkv,
                                                  (int32_t*)(ws + L.off_key_item_base), (int32_t*)(ws + L.off_key_slot_base),
                                                  (int32_t*)(ws + L.off_dkv_counters));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "plan launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

// ------------------------------------------------------------------------------------------
// Scratch of wlb_attn_fwd_static: the schedule tables live in this array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address
// that call returns (kept per device) is what kernels and every other use of the memory get.
static __device__ __align__(256) unsigned char scratch[WLB_ATTN_FWD_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, once resolved
static std::mutex g_scratch_mutex;

// The current device's copy of `scratch`; resolved on the first call on that device.
static wlb_status static_scratch(char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "wlb_attn_fwd_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(WLB_ERR_UNSUPPORTED, "wlb_attn_fwd_static: device %d (at most %d devices)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(WLB_ERR_HIP, "wlb_attn_fwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = (char*)g_scratch_ptr[dev];
    return WLB_OK;
}

// delta and the log2-scaled LSE copy, [hq][n_q] floats each
static size_t delta_bytes(const wlb_attn_desc& d) { return 2 * align_up(sizeof(float) * (size_t)d.hq * d.n_q, 256); }

}  // namespace wlb

using namespace wlb;

extern "C" wlb_status wlb_attn_workspace_size(const wlb_attn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!fwd_bytes || !bwd_bytes) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_workspace_size: null output");
    wlb_plan_layout L;
    plan_layout(*desc, &L);
    *fwd_bytes = L.plan_bytes + row_partial_bytes(*desc, L);
    *bwd_bytes = L.plan_bytes + delta_bytes(*desc) + dkv_partial_bytes(*desc, L) + row_partial_bytes(*desc, L);
    return WLB_OK;
}

extern "C" wlb_status wlb_attn_set_gang_weights(int32_t kernel, const int32_t* weights) {
    if (kernel != 0 && kernel != 1) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_set_gang_weights: kernel=%d (0 = forward, 1 = dQ)", kernel);
    if (weights)
        for (int i = 0; i < 16; ++i)
            if (weights[i] < 1 || weights[i] > 1000000)
                return fail(WLB_ERR_INVALID_ARG, "wlb_attn_set_gang_weights: weight %d = %d outside [1, 10^6]", i, weights[i]);
    std::lock_guard<std::mutex> lock(g_gang_weight_mutex);
    for (int i = 0; i < 16; ++i) g_gang_weight[kernel][i / 8][i % 8] = weights ? weights[i] : 0;
    return WLB_OK;
}

extern "C" wlb_status wlb_attn_get_gang_weights(int32_t kernel, int32_t* weights_out) {
    if (kernel < 0 || kernel > 1) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_get_gang_weights: kernel %d (0 = forward, 1 = dQ)", kernel);
    if (!weights_out) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_get_gang_weights: null output");
    int w[2][8];
    gang_weights(kernel, w);
    for (int i = 0; i < 16; ++i) weights_out[i] = w[i / 8][i % 8];
    return WLB_OK;
}

extern "C" wlb_status wlb_attn_plan_layout(const wlb_attn_desc* desc, wlb_plan_layout* layout) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!layout) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_plan_layout: null output");
    plan_layout(*desc, layout);
    return WLB_OK;
}

extern "C" wlb_status wlb_attn_plan(const wlb_attn_desc* desc, const int32_t* q_idx, const int32_t* cu_seqlens_k,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!q_idx || !cu_seqlens_k || !workspace) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_plan: null pointer");
    wlb_plan_layout L;
    plan_layout(*desc, &L);
    if (workspace_bytes < L.plan_bytes)
        return fail(WLB_ERR_BUFFER_TOO_SMALL, "wlb_attn_plan: workspace %zu < %zu bytes", workspace_bytes, L.plan_bytes);
    return launch_plan(*desc, L, q_idx, cu_seqlens_k, (char*)workspace, stream);
}

extern "C" wlb_status wlb_attn_fwd(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                                   const int32_t* q_idx, const int32_t* cu_seqlens_k, void* o, float* lse,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!q || !k || !v || !o || !lse || !workspace) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_fwd: null pointer");
    const bool reuse = desc->flags & WLB_ATTN_REUSE_PLAN;
    if (!reuse && (!q_idx || !cu_seqlens_k)) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_fwd: null q_idx/cu_seqlens_k");
    wlb_plan_layout L;
    plan_layout(*desc, &L);
    const size_t need = L.plan_bytes + row_partial_bytes(*desc, L);
    if (workspace_bytes < need)
        return fail(WLB_ERR_BUFFER_TOO_SMALL, "wlb_attn_fwd: workspace %zu < %zu bytes", workspace_bytes, need);
    if (!reuse)
        if (wlb_status st = launch_plan(*desc, L, q_idx, cu_seqlens_k, (char*)workspace, stream)) return st;
    return launch_fwd(*desc, L, q, k, v, o, lse, (char*)workspace, L.plan_bytes, stream);
}

extern "C" wlb_status wlb_attn_fwd_static(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                                          const int32_t* q_idx, const int32_t* cu_seqlens_k, void* o, float* lse,
                                          void* stream) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!q || !k || !v || !o || !lse) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_fwd_static: null pointer");
    if (desc->flags & ~(WLB_ATTN_REUSE_PLAN | WLB_ATTN_SCHEDULE_ITEMS))
        return fail(WLB_ERR_INVALID_ARG, "wlb_attn_fwd_static: flags 0x%x (only WLB_ATTN_REUSE_PLAN and WLB_ATTN_SCHEDULE_ITEMS apply)", desc->flags);
    const bool reuse = desc->flags & WLB_ATTN_REUSE_PLAN;
    if (!reuse && (!q_idx || !cu_seqlens_k)) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_fwd_static: null q_idx/cu_seqlens_k");
    // one workgroup per (query tile, head): the schedule that leaves no partial results, so the
    // schedule tables are all the scratch the call needs
    wlb_attn_desc d = *desc;
    d.flags |= WLB_ATTN_SCHEDULE_ITEMS;
    wlb_plan_layout L;
    plan_layout(d, &L);
    if (L.plan_bytes > (size_t)WLB_ATTN_FWD_STATIC_SCRATCH_BYTES)
        return fail(WLB_ERR_UNSUPPORTED, "wlb_attn_fwd_static: the schedule of n_q=%d, t_kv=%d needs %zu bytes, the library's array holds %zu",
                    d.n_q, d.t_kv, L.plan_bytes, (size_t)WLB_ATTN_FWD_STATIC_SCRATCH_BYTES);
    char* ws = nullptr;
    if (wlb_status st = static_scratch(&ws)) return st;
    if (!reuse)
        if (wlb_status st = launch_plan(d, L, q_idx, cu_seqlens_k, ws, stream)) return st;
    return launch_fwd(d, L, q, k, v, o, lse, ws, L.plan_bytes, stream);
}

extern "C" wlb_status wlb_attn_bwd(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                                   const void* o, const float* lse, const void* d_o, const int32_t* q_idx,
                                   const int32_t* cu_seqlens_k, void* dq, void* dk, void* dv, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    if (wlb_status st = check_desc(desc)) return st;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
        return fail(WLB_ERR_INVALID_ARG, "wlb_attn_bwd: null pointer");
    const bool reuse = desc->flags & WLB_ATTN_REUSE_PLAN;
    if (!reuse && (!q_idx || !cu_seqlens_k)) return fail(WLB_ERR_INVALID_ARG, "wlb_attn_bwd: null q_idx/cu_seqlens_k");
    wlb_plan_layout L;
    plan_layout(*desc, &L);
    const size_t need = L.plan_bytes + delta_bytes(*desc) + dkv_partial_bytes(*desc, L) + row_partial_bytes(*desc, L);
    if (workspace_bytes < need)
        return fail(WLB_ERR_BUFFER_TOO_SMALL, "wlb_attn_bwd: workspace %zu < %zu bytes", workspace_bytes, need);
    if (!reuse)
        if (wlb_status st = launch_plan(*desc, L, q_idx, cu_seqlens_k, (char*)workspace, stream)) return st;
    return launch_bwd(*desc, L, q, k, v, o, lse, d_o, dq, dk, dv, (char*)workspace, L.plan_bytes, stream);
}
