// Backward document-masked attention for gfx950.  The paper measures forward+backward
// latency of the attention kernel (Section 6.4) without restating the derivative; this is the
// standard one: with P = exp(scale*Q K^T - LSE) on the visible (same-document, causal) pairs
// and delta_i = <dO_i, O_i>,
//     dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale * dS K,  dK = scale * dS^T Q,
// dK/dV summed over the query heads that share a KV head.  As in all-gather context
// parallelism (Section 2.1) dK/dV hold only the calling rank's rows' contribution.
//
// Five kernels, no atomics, deterministic:
//   delta_kernel      delta[h][i] = -sum_d dO*O (stored negated: the dK/dV kernel starts its dP
//                     accumulators from it) and the log2-scaled LSE copy (0 / +inf for padding rows)
//   dq_kernel         query-stationary, same tiling and work schedule as the forward: S^T and dP^T
//                     per lane column, dQ^T += K^T dS^T with K^T read from LDS by transpose reads
//   dq_merge_kernel   sums the fp32 partial dQ of query tiles cut at a gang boundary
//   dkv_kernel        key-stationary: a work item owns 128 keys of one KV head and streams the row
//                     groups that can see them through LDS for some or all query heads of the KV
//                     group; dK^T, dV^T stay in registers until the single final store
//   dkv_fixup_kernel  sums the fp32 partial results of key tiles whose heads were divided among
//                     several work items (heavy tiles, so that no item is a straggler)
// S and dP are recomputed in both dq_kernel and dkv_kernel (7 GEMMs for the 5 the derivative
// needs): this keeps dQ free of atomics and of an fp32 accumulation buffer.
// Q / dO / K tiles that are read both row-wise (b128) and column-wise (transpose reads) are
// stored unpadded with an XOR swizzle of their 16-byte chunks that makes both patterns
// bank-conflict free; all tiles arrive by asynchronous global->LDS copies.
#include <hip/hip_runtime.h>

#include "wlb_device.h"
#include <algorithm>
#include <type_traits>

#include "wlb_internal.h"

namespace wlb {

struct BwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* o; const __bf16* d_o;
    const float* lse; float* delta; float* lse2;
    __bf16* dq; __bf16* dk; __bf16* dv;
    const int32_t* row_lo; const int32_t* row_hi; const int32_t* group; const int32_t* group_real;
    const int32_t* key_order; const int32_t* key_range;
    const int32_t* key_ways; const int32_t* key_item_base; const int32_t* key_slot_base;
    int32_t* dkv_counters;     // [8]: items of each XCD's list handed out so far (zero before every dK/dV launch)
    float* partial;
    RowSched sched;            // dQ: which query tiles, heads and key ranges a workgroup works on
    float* row_partial;        // dQ: partial results of the tiles cut at a gang boundary
    const int32_t* block_hull; const int32_t* tile_short;   // short-hull path (see dq_short_unit)
    unsigned long long* gang_clock;   // [workgroup][2]: real-time counter at the start / end of dq_kernel's workgroup
    int n_blocks32, use_short, delta_skips_short;
    int n_q, t_kv, hq, hkv, n_groups, n_tiles, n_key_tiles;
    float scale_log2e, scale;
};

// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) delta_kernel(const BwdParams p) {
    constexpr int LPR = D / 8;                       // lanes per (row, head)
    const size_t total = (size_t)p.n_q * p.hq;
    // gridDim.x / n_tiles workgroups share the (row, head) pairs of a query tile.  A short-hull tile, whose delta
    // and LSE copy come from the short-hull dQ units, costs its workgroups one table lookup.
    const int split = (int)gridDim.x / p.n_tiles;
    const int tile = (int)blockIdx.x / split, part = (int)blockIdx.x % split;
    if (tile >= p.n_tiles || (p.delta_skips_short && ld_const(p.tile_short + tile))) return;
    const size_t first = (size_t)tile * kFwdTileRows * p.hq * LPR, lanes = (size_t)kFwdTileRows * p.hq * LPR;
    for (size_t off = (size_t)part * 256; off < lanes; off += (size_t)split * 256) {
        const size_t idx = first + off + threadIdx.x;
        const size_t rh = idx / LPR;                 // row * hq + head
        const int c = (int)(idx % LPR);
        const bool mine = rh < total;
        float acc = 0.f;
        if (mine) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(p.d_o + rh * D + c * 8);
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(p.o + rh * D + c * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
        }
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (mine && c == 0) {
            const int row = (int)(rh / p.hq), h = (int)(rh % p.hq);
            const bool real = p.row_hi[row] > 0;
            p.delta[(size_t)h * p.n_q + row] = real ? -acc : 0.f;
            // LSE in log2 units for the dK/dV kernel; +inf makes every probability of a padding row 0
            p.lse2[(size_t)h * p.n_q + row] = real ? p.lse[(size_t)h * p.n_q + row] * 1.4426950408889634f : INFINITY;
        }
    }
}

// ------------------------------------------------------------------------------------------
// dQ, four wavefronts x 32 rows, two workgroups per CU: K and V tiles of 64 keys arrive by
// asynchronous global->LDS copies (double buffered, one barrier per tile); per block of 32
// keys a wavefront computes S^T = K Q^T and dP^T = V dO^T (lane = its query column), forms
// dS^T = P^T o (dP^T - delta) in registers and accumulates dQ^T += K^T dS^T with K^T read
// from the same swizzled K tile by transpose reads.
template <int D>
__device__ __forceinline__ void dq_piece(const BwdParams& p, char* smem, const RowPiece& pc) {
    constexpr int NW = 4, BM = 128, BN = 64;
    static_assert(BM == kFwdTileRows, "tile rows must match the schedule");
    constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, ROWB = D * 2, TILEB = BN * ROWB;

    const int G = p.hq / p.hkv;
    const int tile = pc.tile, hk = pc.hk;
    const int h = hk * G + pc.member;

    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;

    int k_lo = kPadLo, k_hi = 0;       // hull of the keys the tile's rows see
    for (int j = 0; j < BM / kGroupRows; ++j) {
        const int g = tile * (BM / kGroupRows) + j;
        if (g < p.n_groups) {
            const int4 d = reinterpret_cast<const int4*>(p.group)[g];
            if (d.y > d.x) { k_lo = min(k_lo, d.x); k_hi = max(k_hi, d.y); }
        }
    }
    int jb = 0, je = 0, fb = 0, fe = 0;
    if (k_hi > k_lo) {
        jb = k_lo / BN; je = (k_hi + BN - 1) / BN;
        // this piece's part of the tile's key tiles (the first kRowItemOverhead units of a tile's
        // stretch of the work line stand for its fixed cost)
        je = min(jb + max(pc.b - kRowItemOverhead, 0), je);
        jb = jb + max(pc.a - kRowItemOverhead, 0);
    }

    const uint32_t kv_row = (uint32_t)p.hkv * D;
    const uint32_t kv_bytes = ((uint32_t)p.t_kv * kv_row - (uint32_t)hk * D) * 2u;
    BufRsrc krs, vrs;
    krs.init(p.k + (size_t)hk * D, kv_bytes);
    vrs.init(p.v + (size_t)hk * D, kv_bytes);
    TileDma<D, BN, NW> dma;
    dma.init(wave, lane, kv_row);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    auto tile_ptr = [&](int which) { return smem_base + (uint32_t)(which * TILEB); };
    __syncthreads();            // every wavefront has left the tiles of the piece before
    if (jb < je) {
        dma.issue(krs, tile_ptr(0), jb * BN, wave);
        dma.issue(vrs, tile_ptr(2), jb * BN, wave);
    }

    const int row = tile * BM + wave * 32 + l32;
    const bool in = row < p.n_q;
    const int rc = in ? row : p.n_q - 1;
    const int lo = in ? p.row_lo[rc] : kPadLo;
    const int hi = in ? p.row_hi[rc] : 0;
    const bool real = hi > 0;
    // key tiles this wavefront needs no element-wise mask for: only outside [fb, fe) it masks.  Inside, the
    // rows of the wavefront's first document see every key and the rows of later documents none.
    bool other_doc;
    unmasked_tiles<BN>(lo, hi, real, fb, fe, other_doc);
    // padding rows: zero operands and LSE = +inf make P, dS and dQ exactly 0
    const float lsec = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;
    float lsec_unmasked = other_doc ? INFINITY : lsec;           // inside [fb, fe): +inf switches the lane off
    const float dl = real ? p.delta[(size_t)h * p.n_q + rc] : 0.f;
    bf16x8 qf[KS], dof[KS];
    {
        const __bf16* qp = p.q + ((size_t)rc * p.hq + h) * D + half * 8;
        const __bf16* gp = p.d_o + ((size_t)rc * p.hq + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
            bf16x8 g = *reinterpret_cast<const bf16x8*>(gp + ks * 16);
            if (!real) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { a[i] = (__bf16)0.f; g[i] = (__bf16)0.f; }
            }
            qf[ks] = a; dof[ks] = g;
        }
    }

    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = smem_base + l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = smem_base + key * ROWB + swz<CPR>(key, dch) * 16 + (j16 & 1) * 8;
        }

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    const float cs = p.scale_log2e;

    // one tile; the buffer index is a compile-time constant so that every LDS address is a
    // loop-invariant register plus an immediate
    auto tile_step = [&](int j, auto cur_tag) {
        constexpr int cur = decltype(cur_tag)::value;
        wait_vmem();
        __syncthreads();
        if (j + 1 < je) {
            dma.issue(krs, tile_ptr(cur ^ 1), (j + 1) * BN, wave);
            dma.issue(vrs, tile_ptr(2 + (cur ^ 1)), (j + 1) * BN, wave);
        }
        constexpr int kb_base = cur * TILEB, vb_base = (2 + cur) * TILEB;
        const bool partial = (j < fb) || (j >= fe);
        // S^T and dP^T of a 32-key block (two independent accumulation chains)
        // At head_dim 64, where the kernel is bound by the vector ALU, the dP accumulation starts from -delta
        // (the subtraction happens inside the first MFMA); at 128 that costs registers the kernel does not have.
        constexpr bool kDeltaInMfma = D == 64;
        auto scores = [&](int kb, f32x16& s, f32x16& dp) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = kDeltaInMfma ? dl : 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(kb_base + naddr[ks] + kb * 32 * ROWB));
                const bf16x8 va = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(vb_base + naddr[ks] + kb * 32 * ROWB));
                s = mfma32(ka, qf[ks], s);
                dp = mfma32(va, dof[ks], dp);
            }
        };
        // dS^T = P^T o (dP^T - delta), in place of s; ls = the row's LSE, or +inf to switch the lane off
        auto grads = [&](f32x16& s, const f32x16& dp, float ls) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = fast_exp2(fmaf(s[r], cs, -ls)) * (kDeltaInMfma ? dp[r] : dp[r] + dl);
        };
        // a block outside the fully visible range: rows that see none of its 32 keys (rows of another
        // document in the same wavefront) are switched off as whole lanes; the element-wise mask is
        // needed only where a row's interval cuts the block (diagonal, document edges)
        auto classify = [&](int kb, float& ls, bool& elementwise) __attribute__((always_inline)) {
            const int key0 = j * BN + kb * 32;
            const bool none = (key0 + 32 <= lo) || (key0 >= hi);
            const bool all = (key0 >= lo) && (key0 + 32 <= hi);
            elementwise = __any(!(none || all));
            ls = none ? INFINITY : lsec;
        };
        auto mask = [&](int kb, f32x16& ds) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = j * BN + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                ds[r] = (key >= lo && key < hi) ? ds[r] : 0.f;
            }
        };
        auto update = [&](int kb, const f32x16& ds) __attribute__((always_inline)) {
            bf16x8 dsf[2];
            dsf[0] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
            dsf[1] = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const int koff = (kb * 32 + cc * 16) * ROWB;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 a = cat4(lds_read_tr4_at(kb_base + taddr[db][0] + koff),
                                          lds_read_tr4_at(kb_base + taddr[db][1] + koff));
                    acc[db] = mfma32(a, dsf[cc], acc[db]);
                }
            }
        };
        // The vector-ALU work of a block runs beside MFMAs that do not depend on it: block 0's
        // exponentials beside block 1's score MFMAs, block 1's beside block 0's dQ update.  The mask
        // (only on a document's diagonal or edge) is a branch between those straight-line regions.
        f32x16 s0, dp0, s1, dp1;
        float ls0 = lsec_unmasked, ls1 = lsec_unmasked;
        bool em0 = false, em1 = false;
        if (partial) {
            classify(0, ls0, em0);
            classify(1, ls1, em1);
            if (!em0 && !em1) {
                // Every row sees all or none of the tile's second block.  That stays so up to the next edge of
                // a row's interval (the end of a row that sees it, the start of one still to come): the key
                // tiles from the next one up to that edge become the unmasked range, the rows that see
                // nothing switched off.  A wavefront that holds rows of two chunks of one document (or of
                // two documents) crosses the keys between them without classifying every block.
                const int key1 = j * BN + 32;
                const bool none = (key1 + 32 <= lo) || (key1 >= hi);
                int edge = none ? (lo >= key1 + 32 ? lo : kPadLo) : hi;
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) edge = min(edge, __shfl_xor(edge, o));
                const int j_edge = uniform(edge / BN);
                if (j_edge > j + 1) {
                    fb = j + 1;
                    fe = j_edge;
                    lsec_unmasked = none ? INFINITY : lsec;
                }
            }
        }
        scores(0, s0, dp0);
        scores(1, s1, dp1);
        grads(s0, dp0, ls0);
        if (em0) {
            asm volatile("");   // keep the mask a branch
            mask(0, s0);
        }
        update(0, s0);
        grads(s1, dp1, ls1);
        if (em1) {
            asm volatile("");
            mask(1, s1);
        }
        update(1, s1);
    };
    for (int j = jb; j < je; j += 2) {
        tile_step(j, std::integral_constant<int, 0>{});
        if (j + 1 < je) tile_step(j + 1, std::integral_constant<int, 1>{});
    }

    if (pc.slot >= 0) {
        // part of a tile: unscaled fp32 dQ [row][d], summed by dq_merge_kernel
        float* part = p.row_partial + (size_t)pc.slot * (BM * D + 2 * BM);
        if (in) {
            const int rl = wave * 32 + l32;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d = db * 32 + r4 * 8 + half * 4;
                    *reinterpret_cast<f32x4*>(part + (size_t)rl * D + d) =
                        f32x4{acc[db][r4 * 4 + 0], acc[db][r4 * 4 + 1], acc[db][r4 * 4 + 2], acc[db][r4 * 4 + 3]};
                }
        }
        return;
    }
    if (in) {
        __bf16* op = p.dq + ((size_t)row * p.hq + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = db * 32 + r4 * 8 + half * 4;
                bf16x4 out;
                if (real) out = pack4(acc[db][r4 * 4 + 0] * p.scale, acc[db][r4 * 4 + 1] * p.scale,
                                      acc[db][r4 * 4 + 2] * p.scale, acc[db][r4 * 4 + 3] * p.scale);
                else out = pack4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<bf16x4*>(op + d) = out;
            }
    }
}

// dQ: a fixed set of workgroups, each walking its gang's share of the work line (see RowSched).
template <int D>
__global__ void __launch_bounds__(256, 2) dq_kernel(const BwdParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[4 * 64 * D * 2];   // K0 | K1 | V0 | V1
    const unsigned long long t_start = wall_clock64();
    RowWalk walk;
    walk.start(p.sched, (int)blockIdx.x);
    RowPiece pc;
    while (walk.next(p.sched, pc)) dq_piece<D>(p, smem, pc);
    if (threadIdx.x == 0) {
        p.gang_clock[2 * blockIdx.x] = t_start;
        p.gang_clock[2 * blockIdx.x + 1] = wall_clock64();
    }
}

// dQ of short-hull tiles, the counterpart of the forward's short-hull kernel (same workgroup shape,
// same LDS layout: K window | V window | one staging tile per wavefront; see there).  A wavefront
// works on one query head at a time; that head's rows of Q and dO reach it as whole rows and pass
// through the staging tile into the MFMA operand layout.  All keys a row sees lie inside the window, so the wavefront has the row's whole
// P and dP and forms delta itself as sum_j P_ij dP_ij (equal to <dO_i, O_i> since O = P V), without
// reading O: first pass per 32-key block S^T, dP^T, P and X = P o dP (both kept as bf16), then
// dS^T = X - delta P and dQ^T += K^T dS^T.  delta (negated) and the log2-scaled LSE copy are left
// for the dK/dV kernel, which runs after this one; the separate delta pass skips these rows.
template <int D>
struct ShortDq {
    static constexpr int NW = 4, ROWB = D * 2, HULL = kShortHullKeys, STAGE = kShortBlockRows * ROWB;
    static constexpr int LDS_BYTES = 2 * HULL * ROWB + NW * STAGE;    // K window | V window | staging tiles
};

template <int D>
__device__ __forceinline__ void dq_short_unit(const BwdParams& p, char* smem, int blk, int hk) {
    constexpr int NW = 4, KS = D / 16, DB = D / 32, CPR = D / 8, ROWB = D * 2;
    constexpr int HULL = kShortHullKeys, NB = HULL / 32, STAGE = kShortBlockRows * ROWB, RPI = 64 / CPR;
    const int G = p.hq / p.hkv;
    __syncthreads();              // every wavefront has left the LDS of the unit before

    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    const int h_lo = ld_const(p.block_hull + 2 * blk), h_hi = ld_const(p.block_hull + 2 * blk + 1);
    const int row0 = blk * kShortBlockRows;
    const int row = row0 + l32;
    const bool in = row < p.n_q;
    const int rc = in ? row : p.n_q - 1;
    const uint32_t q_row = (uint32_t)p.hq * D;

    const uint32_t q_row_bytes = q_row * 2u;
    const buf_rsrc_t q_buf = make_buf(p.q, (uint32_t)p.n_q * q_row_bytes), do_buf = make_buf(p.d_o, (uint32_t)p.n_q * q_row_bytes),
                     dq_buf = make_buf(p.dq, (uint32_t)p.n_q * q_row_bytes);
    const int row_voff = RowBlock<D>::lane_off(lane, q_row_bytes);
    auto head_soff = [&](int hs) { return uniform((uint32_t)row0 * q_row_bytes + (uint32_t)(hk * G + hs) * ROWB); };

    if (h_hi <= h_lo) {
        // no real row in this block: dQ = 0; delta = 0 and LSE copy = +inf keep the rows out of dK/dV
        RowBlock<D> zero;
#pragma unroll
        for (int i = 0; i < RowBlock<D>::N; ++i) zero.v[i] = i32x4{0, 0, 0, 0};
        for (int hs = wave; hs < G; hs += NW) {
            const int h = hk * G + hs;
            zero.store(dq_buf, row_voff, head_soff(hs), q_row_bytes);
            if (in && half == 0) {
                p.delta[(size_t)h * p.n_q + row] = 0.f;
                p.lse2[(size_t)h * p.n_q + row] = INFINITY;
            }
        }
        return;
    }
    const int kstart = h_lo & ~31;
    const int nblk = (h_hi - kstart + 31) >> 5;

    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t stage = uniform(smem_base + 2 * HULL * ROWB + (uint32_t)wave * STAGE);

    const uint32_t kv_row = (uint32_t)p.hkv * D;
    const uint32_t kv_bytes = ((uint32_t)p.t_kv * kv_row - (uint32_t)hk * D) * 2u;
    BufRsrc krs, vrs;
    krs.init(p.k + (size_t)hk * D, kv_bytes);
    vrs.init(p.v + (size_t)hk * D, kv_bytes);
    TileDma<D, 32 * NW, NW> dma;                          // wavefront w copies the 32-key block w
    dma.init(wave, lane, kv_row);
    if (wave < nblk) {
        dma.issue(krs, smem_base, kstart, wave);
        dma.issue(vrs, smem_base + HULL * ROWB, kstart, wave);
    }

    const int lo = in ? p.row_lo[rc] : kPadLo;
    const int hi = in ? p.row_hi[rc] : 0;
    const bool real = hi > 0;
    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = smem_base + key * ROWB + swz<CPR>(key, dch) * 16 + (j16 & 1) * 8;
        }
    const float cs = p.scale_log2e;
    // padding rows: zero operands and LSE = +inf make P, dS and dQ exactly 0 (their Q / dO may hold anything)
    auto rows_from_stage = [&](bf16x8 (&dst)[KS]) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(stage + naddr[ks]));
            if (!real) {
#pragma unroll
                for (int i = 0; i < 8; ++i) a[i] = (__bf16)0.f;
            }
            dst[ks] = a;
        }
    };

    wait_vmem();
    __syncthreads();              // the key window is in LDS; the wavefronts do not meet again

#pragma nounroll
    for (int hs = wave; hs < G; hs += NW) {
        const int h = hk * G + hs;
        // this head's rows of Q and dO: whole rows into registers, then through the staging tile into the
        // operand layout (eight wavefronts per compute unit cover each other's load latency)
        bf16x8 qf[KS], dof[KS];
        {
            RowBlock<D> q_rows, do_rows;
            q_rows.load(q_buf, row_voff, head_soff(hs), q_row_bytes);
            do_rows.load(do_buf, row_voff, head_soff(hs), q_row_bytes);
            q_rows.to_tile(stage, lane);
            rows_from_stage(qf);
            wait_lds();
            do_rows.to_tile(stage, lane);
            rows_from_stage(dof);
        }
        const float lse_cur = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;

        // first pass: P and X = P o dP of every block (masked entries 0), delta = sum of X over the row
        bf16x8 pk[NB][2], xk[NB][2];
        float dsum = 0.f, psum = 0.f, dsum_r = 0.f, psum_r = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
                f32x16 sc, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 ka = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(smem_base + naddr[ks] + b * 32 * ROWB));
                    const bf16x8 va = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(smem_base + naddr[ks] + (HULL + b * 32) * ROWB));
                    sc = mfma32(ka, qf[ks], sc);
                    dp = mfma32(va, dof[ks], dp);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kstart + b * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    const float pr = (key >= lo && key < hi) ? fast_exp2(fmaf(sc[r], cs, -lse_cur)) : 0.f;
                    sc[r] = pr;
                    dp[r] = pr * dp[r];
                    psum += pr;
                    dsum += dp[r];
                }
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    pk[b][cc] = pack8(sc[8 * cc + 0], sc[8 * cc + 1], sc[8 * cc + 2], sc[8 * cc + 3],
                                      sc[8 * cc + 4], sc[8 * cc + 5], sc[8 * cc + 6], sc[8 * cc + 7]);
                    xk[b][cc] = pack8(dp[8 * cc + 0], dp[8 * cc + 1], dp[8 * cc + 2], dp[8 * cc + 3],
                                      dp[8 * cc + 4], dp[8 * cc + 5], dp[8 * cc + 6], dp[8 * cc + 7]);
                    // this kernel's own delta comes from the rounded X and P that dS is formed from below, so
                    // that they cancel exactly where they should (a row that sees one key: dS = 0)
#pragma unroll
                    for (int i = 0; i < 8; ++i) { dsum_r += (float)xk[b][cc][i]; psum_r += (float)pk[b][cc][i]; }
                }
            }
        }
        dsum += xhalf(dsum); psum += xhalf(psum);
        dsum_r += xhalf(dsum_r); psum_r += xhalf(psum_r);
        // delta_i = sum_j P_ij dP_ij / sum_j P_ij: the row's probabilities sum to 1 up to the rounding of
        // the stored LSE, and dividing by their actual sum keeps delta equal to dP for a row with one key
        const float delta = (real && psum_r > 0.f) ? dsum_r / psum_r : 0.f;
        if (in && half == 0) {
            p.delta[(size_t)h * p.n_q + row] = (real && psum > 0.f) ? -dsum / psum : 0.f;
            p.lse2[(size_t)h * p.n_q + row] = lse_cur;
        }
        // dS^T = X - delta P of every block, as the bf16 operand of the second pass (in place of P)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    float ds[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) ds[i] = fmaf(-delta, (float)pk[b][cc][i], (float)xk[b][cc][i]);
                    pk[b][cc] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
                }
            }
        }
        // second pass: dQ^T += K^T dS^T
        f32x16 acc[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const int koff = (b * 32 + cc * 16) * ROWB;
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const bf16x8 a = cat4(lds_read_tr4_at(taddr[db][0] + koff), lds_read_tr4_at(taddr[db][1] + koff));
                        acc[db] = mfma32(a, pk[b][cc], acc[db]);
                    }
                }
            }
        }
        // dQ rows through the staging tile (Q and dO are in registers by now), stored as whole rows
        const float f = real ? p.scale : 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *reinterpret_cast<WLB_LDS bf16x4*>((uintptr_t)(stage + l32 * ROWB + swz<CPR>(l32, db * 4 + r4) * 16 + half * 8)) =
                    pack4(acc[db][r4 * 4 + 0] * f, acc[db][r4 * 4 + 1] * f, acc[db][r4 * 4 + 2] * f, acc[db][r4 * 4 + 3] * f);
        RowBlock<D> dq_rows;
        dq_rows.from_tile(stage, lane);
        dq_rows.store(dq_buf, row_voff, head_soff(hs), q_row_bytes);
        wait_lds();                                 // the staging tile has been read back
    }
}

// The other schedule: one workgroup per (query tile in order, query head), heaviest first.
template <int D>
__global__ void __launch_bounds__(256, 2) dq_items_kernel(const BwdParams p) {
    constexpr int kLds = ShortDq<D>::LDS_BYTES > 4 * 64 * D * 2 ? ShortDq<D>::LDS_BYTES : 4 * 64 * D * 2;
    __shared__ __attribute__((aligned(1024))) char smem[kLds];
    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    int y = blockIdx.x >> 3;
    RowPiece pc;
    pc.member = y % G; y /= G;
    pc.hk = y % p.hkv;
    const int rank = (y / p.hkv) * 8 + x;
    if (rank >= p.n_tiles) return;
    pc.tile = ld_const(p.sched.order + rank);
    if (p.use_short && ld_const(p.tile_short + pc.tile)) {
        // a short-hull tile: its four blocks of 32 rows are units of their own (see dq_short_unit)
        constexpr int per_tile = kFwdTileRows / kShortBlockRows;
        for (int j = pc.member; j < per_tile; j += G) {
            const int blk = pc.tile * per_tile + j;
            if (blk < p.n_blocks32) dq_short_unit<D>(p, smem, blk, pc.hk);
        }
        return;
    }
    pc.c = (int)(ld_const64(p.sched.prefix + rank + 1) - ld_const64(p.sched.prefix + rank));
    pc.a = 0; pc.b = pc.c; pc.slot = -1;
    dq_piece<D>(p, smem, pc);
}

// Sums the partial dQ of a query tile that was cut at gang boundaries.  One workgroup per
// (gang, member): it acts if its gang's last piece is the first part of a tile, and then takes
// that part and the first piece of every later gang whose (non-empty) share begins inside the tile.
template <int D>
__global__ void __launch_bounds__(256) dq_merge_kernel(const BwdParams p) {
    constexpr int BM = kFwdTileRows, PF = BM * D + 2 * BM, V4 = D / 4;
    const RowSched& s = p.sched;
    const int job = (int)blockIdx.x / kMergeSplit, quarter = (int)blockIdx.x % kMergeSplit;
    const int gang = job / s.G, member = job % s.G;
    RowCut cut;
    if (!cut.find(s, gang)) return;
    const int tile = cut.tile;
    const int h = cut.hk * s.G + member;
    auto part = [&](int slot) { return p.row_partial + ((size_t)slot * s.G + member) * PF; };
    const float* first = part(cut.first_slot());
    constexpr int CAP = 32;
    __shared__ int s_slots[CAP], s_count;
    const int n_later = gather_later_parts<CAP>(cut, s_slots, &s_count);
    constexpr int PER = BM * V4 / kMergeSplit;
    for (int e = quarter * PER + threadIdx.x; e < (quarter + 1) * PER; e += 256) {
        const int rl = e / V4, d4 = e % V4;
        const int row = tile * BM + rl;
        if (row >= p.n_q) continue;
        const size_t at = (size_t)rl * D + d4 * 4;
        f32x4 sum = *reinterpret_cast<const f32x4*>(first + at);
        if (n_later <= CAP) {
            for (int i = 0; i < n_later; ++i) sum += *reinterpret_cast<const f32x4*>(part(s_slots[i]) + at);
        } else {
            cut.later_parts([&](int slot) { sum += *reinterpret_cast<const f32x4*>(part(slot) + at); });
        }
        const bool real = p.row_hi[row] > 0;
        *reinterpret_cast<bf16x4*>(p.dq + ((size_t)row * p.hq + h) * D + d4 * 4) =
            real ? pack4(sum[0] * p.scale, sum[1] * p.scale, sum[2] * p.scale, sum[3] * p.scale) : pack4(0.f, 0.f, 0.f, 0.f);
    }
}

// ------------------------------------------------------------------------------------------
// dK/dV with role-split wavefronts: one workgroup = 128 keys x one KV head, eight wavefronts.
// Wavefronts 0-3 ("score" role) hold the K operands of 32 keys each: they compute
// S = Q K^T, P = exp(scale*S - LSE) (masked), hand P (bf16) to their partner through LDS and
// accumulate dV^T += dO^T P.  Wavefronts 4-7 ("gradient" role) hold the V operands of the same
// keys: they compute dP = dO V^T, take P from the partner, form dS = P o (dP - delta) and
// accumulate dK^T += Q^T dS.  A wavefront that held K, V, dK^T and dV^T together would need
// more than 256 registers, i.e. one wavefront per SIMD, which measured slower here: splitting
// halves the register need, so two wavefronts share a SIMD and hide each other's LDS latencies.
// Stages (row group, query head) stream through three LDS buffers.  The gradient role works one
// stage behind the score role: between two workgroup barriers the score wavefronts run stage t
// (S, P, dV) while the gradient wavefronts run stage t-1 (dP, dS, dK) with the P that was
// written before the barrier.  One barrier per stage, and both roles carry the same load
// (32 MFMAs plus the exponentials resp. the dS products), so neither waits for the other.
// A work item is a key tile with all query heads of one KV head, or - for a tile whose work
// exceeds a threshold set by the schedule - a 1/2, 1/4 or 1/8 of those heads; such an item
// writes its dK^T / dV^T as an unscaled fp32 partial result instead of the final bf16 rows.
template <int D>
__global__ void __launch_bounds__(512) dkv_kernel(const BwdParams p) {
    constexpr int BNK = kBwdKeyTile, GR = kGroupRows, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int ROWB = D * 2, TILEB = GR * ROWB, NW = 8, NBUF = 3, PBYTES = 4 * 2 * 2 * 1024;
    static_assert(BNK == 128 && GR == 64, "tiling");

    __shared__ __attribute__((aligned(1024))) char smem[NBUF * 2 * TILEB];   // per stage buffer: Q tile | dO tile, swizzled
    // P of two stages (aligned so that one XOR switches stage): [key block][row block][half of 16 rows][lane] x 16 B
    __shared__ __attribute__((aligned(2 * PBYTES))) char pbuf[2 * PBYTES];
    __shared__ __attribute__((aligned(256))) int small_s[NBUF][4][GR];       // per stage buffer: lse2 | delta | row_lo | row_hi

    const int G = p.hq / p.hkv;
    // Work items: tiles in order (heaviest item first), a tile's items consecutive: KV head major, head
    // part minor.  The launch is one workgroup per compute unit, and each takes item after item until
    // none is left.  Item i belongs to XCD i % 8 (workgroup b runs on XCD b % 8): the same head part of
    // neighbouring tiles then shares an XCD and its L2 copy of the Q / dO tiles.  A workgroup takes its own
    // XCD's items first, through one counter per XCD, and the other XCDs' once those are gone: the XCDs
    // of one GPU differ in speed by several percent (the same ones are slower in every launch), and with
    // one workgroup per item the hardware hands every XCD the same number of them.
    __shared__ int s_item;
    const int n_items = ld_const(p.key_item_base + p.n_key_tiles);
  for (;;) {
    __syncthreads();              // every wavefront has left the LDS of the item before, and has read s_item
    if (threadIdx.x == 0) {
        int it = -1;
        for (int k = 0; k < kLists && it < 0; ++k) {
            const int c = ((int)blockIdx.x + k) % kLists;
            const int cand = atomicAdd(p.dkv_counters + c, 1) * kLists + c;
            if (cand < n_items) it = cand;
        }
        s_item = it;
    }
    __syncthreads();
    const int item = uniform(s_item);
    if (item < 0) break;
    int r = 0;
    for (int hi = p.n_key_tiles; hi - r > 1;) {
        const int mid = (r + hi) >> 1;
        if (ld_const(p.key_item_base + mid) <= item) r = mid; else hi = mid;
    }
    const int kt = ld_const(p.key_order + r);
    const int ways = ld_const(p.key_ways + kt);
    const int j = item - ld_const(p.key_item_base + r);
    const int hk = j / ways, part = j % ways;
    const int nh = G / ways;                 // query heads of this item: hk * G + part * nh + [0, nh)
    const int h_first = hk * G + part * nh;
    const bool whole = ways == 1;
    const int slot = ld_const(p.key_slot_base + r) + j;

    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    // role and key block are left as per-lane values: as scalars they raise the register pressure
    // of the two role branches past 256 (spills)
    const int role = tid >> 8, kblk = (tid >> 6) & 3;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    const float cs = p.scale_log2e;
    const int k0 = kt * BNK;
    const int kw0 = k0 + kblk * 32;
    const int mykey = kw0 + l32;

    const uint32_t q_row = (uint32_t)p.hq * D;
    const uint32_t q_total = (uint32_t)p.n_q * q_row * 2u;
    TileDma<D, GR, NW> dma;
    dma.init(wave, lane, q_row);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t small_base = (uint32_t)(uintptr_t)(WLB_LDS char*)&small_s[0][0][0];
    // The copies of a stage are issued with as little scalar work as possible (it sits between the
    // barrier and the stage's first MFMA): the Q and dO descriptors span the whole tensors and the
    // stage's row group and head go into the scalar offset (an address at or past the tensor's end
    // still reads as zeros: the hardware compares offset + scalar offset with the size); everything
    // that depends only on the wavefront is computed here.
    BufRsrc q_rs, do_rs;
    q_rs.init(p.q, q_total);
    do_rs.init(p.d_o, q_total);
    uint32_t dma_soff[TileDma<D, GR, NW>::PER], dma_lds[TileDma<D, GR, NW>::PER];
#pragma unroll
    for (int n = 0; n < TileDma<D, GR, NW>::PER; ++n) {
        const uint32_t blk = (uint32_t)(wave * TileDma<D, GR, NW>::PER + n);
        dma_soff[n] = uniform(blk * TileDma<D, GR, NW>::RPI * q_row * 2u);
        dma_lds[n] = uniform(smem_base + blk * 1024u);
    }
    const uint32_t group_bytes = (uint32_t)GR * q_row * 2u;
    auto issue_stage = [&](int g, int h, int b) {
        const uint32_t so = uniform((uint32_t)g * group_bytes + (uint32_t)h * ROWB);
        const uint32_t lo = uniform((uint32_t)b * (2 * TILEB));
#pragma unroll
        for (int n = 0; n < TileDma<D, GR, NW>::PER; ++n) {
            dma_issue_1k(q_rs.r, dma_lds[n] + lo, dma.voff[n], so + dma_soff[n]);
            dma_issue_1k(do_rs.r, dma_lds[n] + lo + TILEB, dma.voff[n], so + dma_soff[n]);
        }
    };
    // Per-row scalars of a stage (visible key interval, log2-scaled LSE, delta) are copied
    // global->LDS asynchronously as well, by wavefront 0: no register load sits between the copies
    // and the compute, so nothing makes the compiler wait on vector memory while they are in
    // flight.  Rows past n_q read as zeros (row_hi = 0: no visible key; their Q/dO rows are zero);
    // the LSE and delta descriptors are therefore per head (base + h * n_q, n_q entries).
    BufRsrc lo_rs, hi_rs, ls_rs, dl_rs;
    lo_rs.init(p.row_lo, (uint32_t)p.n_q * 4u);
    hi_rs.init(p.row_hi, (uint32_t)p.n_q * 4u);
    ls_rs.init(p.lse2, (uint32_t)p.n_q * 4u);
    dl_rs.init(p.delta, (uint32_t)p.n_q * 4u);
    const uint64_t lse_addr = (uint64_t)(uintptr_t)p.lse2, delta_addr = (uint64_t)(uintptr_t)p.delta;
    auto load_small = [&](int g, int h, int b) {
        if (wave == 0) {
            const uint64_t ho = (uint64_t)(uint32_t)h * (uint32_t)p.n_q * 4u;
            const uint64_t la = lse_addr + ho, da = delta_addr + ho;
            ls_rs.r[0] = (int)(uint32_t)la; ls_rs.r[1] = (int)(uint32_t)((la >> 32) & 0xffffu);
            dl_rs.r[0] = (int)(uint32_t)da; dl_rs.r[1] = (int)(uint32_t)((da >> 32) & 0xffffu);
            const uint32_t soff = uniform((uint32_t)(g * GR) * 4u);
            const uint32_t sl = uniform(small_base + (uint32_t)b * (4 * GR * 4));
            dma_issue_256(ls_rs.r, sl, lane * 4, soff);
            dma_issue_256(dl_rs.r, sl + GR * 4, lane * 4, soff);
            dma_issue_256(lo_rs.r, sl + 2 * GR * 4, lane * 4, soff);
            dma_issue_256(hi_rs.r, sl + 3 * GR * 4, lane * 4, soff);
        }
    };

    // LDS addresses, absolute and per role, rotated through the three stage buffers by one add per
    // stage so that every access in the regions is register + immediate:
    //   naddr: rows of the tile read row-wise      (score role: Q of its stage, gradient role: dO of its stage)
    //   taddr: rows of the tile read transposed    (score role: dO,             gradient role: Q)
    //   saddr: this lane's 4 rows of the per-row scalars;  paddr: this lane's slot of the P buffer
    // The score role starts at buffer 0 (stage 0); the gradient role works one stage behind and
    // starts at the last buffer.
    const int rot0 = role == 0 ? 0 : NBUF - 1;
    const uint32_t stage_base = smem_base + (uint32_t)rot0 * (2 * TILEB);
    uint32_t naddr[KS], taddr[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        naddr[ks] = stage_base + (role == 0 ? 0 : TILEB) + l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
    // transposed reads: rows qq and qq+8 of a 16-row step; the swizzle of row qq+8 is that of row
    // qq with bit 1 flipped, and tiles are 1 KiB aligned, so the second address is the first
    // with address bit 5 flipped plus 8 rows
    static_assert(swz<CPR>(8, 0) == (swz<CPR>(0, 0) ^ 2) && swz<CPR>(13, 5) == (swz<CPR>(5, 5) ^ 2), "row+8 flips swizzle bit 1");
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        const int qq = half * 4 + (j16 >> 2);
        const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
        taddr[db] = stage_base + (role == 0 ? TILEB : 0) + qq * ROWB + swz<CPR>(qq, dch) * 16 + (j16 & 1) * 8;
    }
    uint32_t saddr = small_base + (uint32_t)rot0 * (4 * GR * 4) + half * 16;
    // score role: P buffer of its stage, gradient role: of the stage before
    uint32_t paddr = ((uint32_t)(uintptr_t)(WLB_LDS char*)pbuf + kblk * 4096 + lane * 16) ^ (role == 0 ? 0u : (uint32_t)PBYTES);
    // b = buffer of the stage the score role just ran
    auto rotate = [&](int b) __attribute__((always_inline)) {
        const bool wrap = role == 0 ? b == NBUF - 1 : b == 0;
        const int dt = wrap ? -(NBUF - 1) * 2 * TILEB : 2 * TILEB;
        const int dsm = wrap ? -(NBUF - 1) * 4 * GR * 4 : 4 * GR * 4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) naddr[ks] += dt;
#pragma unroll
        for (int db = 0; db < DB; ++db) taddr[db] += dt;
        saddr += dsm;
        paddr ^= (uint32_t)PBYTES;
    };
    auto lds_f4 = [&](uint32_t a) __attribute__((always_inline)) { return *reinterpret_cast<const WLB_LDS f32x4*>((uintptr_t)a); };
    auto lds_i4 = [&](uint32_t a) __attribute__((always_inline)) { return *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)a); };

    // this wavefront's B operands: K rows (score role) or V rows (gradient role) of its 32 keys
    bf16x8 bop[KS];
    {
        const int kr = min(mykey, p.t_kv - 1);
        const __bf16* src = (role == 0 ? p.k : p.v) + ((size_t)kr * p.hkv + hk) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bop[ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
    }
    f32x16 acc[DB];     // dV^T (score role) or dK^T (gradient role)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // ---- pieces of a role's work on one stage
    // A stage is eight units of four (D/32) MFMAs; the operands of unit u+1 are requested from LDS
    // before the MFMAs of unit u are issued (two operand register sets), so that a wavefront by
    // itself can keep MFMAs flowing and only the first unit of a stage waits for an LDS round trip.
    struct RowOps { bf16x8 a[KS / 2]; };       // half the head dimension of 32 rows, read row-wise
    struct ColOps { bf16x4 t[DB][2]; };        // 16 rows, read transposed
    auto load_rows = [&](RowOps& o, int qb, int kh) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks)
            o.a[ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(naddr[kh * (KS / 2) + ks] + qb * 32 * ROWB));
    };
    auto load_cols = [&](ColOps& o, int st) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int t = 0; t < 2; ++t) o.t[db][t] = lds_read_tr4_at((t ? taddr[db] ^ 32u : taddr[db]) + (st * 16 + t * 8) * ROWB);
    };
    // S or dP of a 32-row block, half the head dimension: B operand = K or V
    auto mfma_rows = [&](f32x16& sc, const RowOps& o, int kh) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) sc = mfma32(o.a[ks], bop[kh * (KS / 2) + ks], sc);
    };
    // 16 rows: acc += tile^T x b  (score role: dV from dO^T, gradient role: dK from Q^T)
    auto mfma_cols = [&](const ColOps& o, const bf16x8& b) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma32(cat4(o.t[db][0], o.t[db][1]), b, acc[db]);
    };
    // Per-row scalars of 16 rows (8-row groups 2cc, 2cc+1 of row block qb; this lane's 4 rows of each):
    // requested one unit ahead like the MFMA operands
    struct RowVals { f32x4 v[2]; };
    auto load_vals = [&](RowVals& o, int which, int qb, int cc) __attribute__((always_inline)) {
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2) o.v[r2] = lds_f4(saddr + which * GR * 4 + (qb * 32 + (cc * 2 + r2) * 8) * 4);
    };
    // P of those 16 rows: exponentials, mask, bf16; returned as this wavefront's B operand and
    // handed to the partner through LDS.  The mask is needed only on a document's diagonal or edge
    // (uniform branch).
    auto probs_half = [&](const f32x16& sc, const RowVals& ls, int qb, int cc, bool masked) __attribute__((always_inline)) {
        float pr[8];
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[r2 * 4 + i] = fast_exp2(fmaf(sc[(cc * 2 + r2) * 4 + i], cs, -ls.v[r2][i]));
        if (masked) {
#pragma unroll
            for (int r2 = 0; r2 < 2; ++r2) {
                const int roff = (qb * 32 + (cc * 2 + r2) * 8) * 4;
                const i32x4 l4 = lds_i4(saddr + 2 * GR * 4 + roff);
                const i32x4 h4 = lds_i4(saddr + 3 * GR * 4 + roff);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    pr[r2 * 4 + i] = (mykey >= l4[i] && mykey < h4[i]) ? pr[r2 * 4 + i] : 0.f;
            }
        }
        const bf16x8 pk = pack8(pr[0], pr[1], pr[2], pr[3], pr[4], pr[5], pr[6], pr[7]);
        *reinterpret_cast<WLB_LDS bf16x8*>((uintptr_t)(paddr + (qb * 2 + cc) * 1024)) = pk;
        return pk;
    };
    // dS of 16 rows: P (from the partner) x (dP - delta); the dP accumulators start from -delta
    auto load_p = [&](int qb, int cc) __attribute__((always_inline)) {
        return *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(paddr + (qb * 2 + cc) * 1024));
    };
    auto ds_half = [&](const f32x16& dn, const bf16x8& pv, int cc) __attribute__((always_inline)) {
        float ds[8];
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
            for (int i = 0; i < 4; ++i) ds[r2 * 4 + i] = (float)pv[r2 * 4 + i] * dn[(cc * 2 + r2) * 4 + i];
        return pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
    };
    // -delta of the 32 rows of block qb, in accumulator order
    auto load_neg_delta = [&](f32x16& o, int qb) __attribute__((always_inline)) {
#pragma unroll
        for (int g8 = 0; g8 < 4; ++g8) {
            const f32x4 x = lds_f4(saddr + GR * 4 + (qb * 32 + g8 * 8) * 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) o[g8 * 4 + i] = x[i];
        }
    };
    // The fences pin the order "request unit u+1, run unit u"; the exponentials / dS products of
    // one row block are placed beside the MFMAs of the units that do not depend on them.
    auto fence = [] () __attribute__((always_inline)) { __builtin_amdgcn_sched_barrier(0); };
    auto score_stage = [&](bool masked) __attribute__((always_inline)) {
        f32x16 s0, s1;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
        RowOps ra, rb;
        ColOps ca, cb;
        RowVals la, lb;
        load_rows(ra, 0, 0);
        load_rows(rb, 0, 1);                          fence();  mfma_rows(s0, ra, 0);  fence();
        load_rows(ra, 1, 0);  load_vals(la, 0, 0, 0); fence();  mfma_rows(s0, rb, 1);  fence();
        load_rows(rb, 1, 1);  load_vals(lb, 0, 0, 1); fence();  mfma_rows(s1, ra, 0);
        const bf16x8 p00 = probs_half(s0, la, 0, 0, masked);
        fence();
        load_cols(ca, 0);     load_vals(la, 0, 1, 0); fence();  mfma_rows(s1, rb, 1);
        const bf16x8 p01 = probs_half(s0, lb, 0, 1, masked);
        fence();
        load_cols(cb, 1);     load_vals(lb, 0, 1, 1); fence();  mfma_cols(ca, p00);
        const bf16x8 p10 = probs_half(s1, la, 1, 0, masked);
        fence();
        load_cols(ca, 2);                             fence();  mfma_cols(cb, p01);
        const bf16x8 p11 = probs_half(s1, lb, 1, 1, masked);
        fence();
        load_cols(cb, 3);                             fence();  mfma_cols(ca, p10);  fence();
        mfma_cols(cb, p11);
    };
    auto grad_stage = [&]() __attribute__((always_inline)) {
        f32x16 d0, d1;
        RowOps ra, rb;
        ColOps ca, cb;
        bf16x8 pa, pb;
        load_rows(ra, 0, 0);  load_neg_delta(d0, 0);
        load_rows(rb, 0, 1);                           fence();  mfma_rows(d0, ra, 0);  fence();
        load_rows(ra, 1, 0);  load_neg_delta(d1, 1);  pa = load_p(0, 0);  fence();  mfma_rows(d0, rb, 1);  fence();
        load_rows(rb, 1, 1);  pb = load_p(0, 1);      fence();  mfma_rows(d1, ra, 0);
        const bf16x8 e00 = ds_half(d0, pa, 0);
        fence();
        load_cols(ca, 0);     pa = load_p(1, 0);      fence();  mfma_rows(d1, rb, 1);
        const bf16x8 e01 = ds_half(d0, pb, 1);
        fence();
        load_cols(cb, 1);     pb = load_p(1, 1);      fence();  mfma_cols(ca, e00);
        const bf16x8 e10 = ds_half(d1, pa, 0);
        fence();
        load_cols(ca, 2);                             fence();  mfma_cols(cb, e01);
        const bf16x8 e11 = ds_half(d1, pb, 1);
        fence();
        load_cols(cb, 3);                             fence();  mfma_cols(ca, e10);  fence();
        mfma_cols(cb, e11);
    };

    // stage t of the item is row group g_first + t / nh with query head h_first + t % nh; every
    // group of the tile's range is a stage (one whose hull misses the tile, rare, costs a copy and no math)
    const int g_first = ld_const(p.key_range + 2 * kt);
    const int t1 = (ld_const(p.key_range + 2 * kt + 1) - g_first) * nh;

    // The schedule data of a stage (its group's hull, fully visible range and real-row count) comes
    // by scalar loads issued right after the barrier of the stage before and is turned into flags
    // at that stage's end: a load at the top of a stage would put its latency in front of the barrier.
    struct Flags { bool full, live, pads; };
    auto flags_of = [&](const int4& gd, int real, int g) {
        Flags f;
        f.full = (gd.z <= k0) && (k0 + BNK <= gd.w);
        f.live = (gd.x < kw0 + 32) && (gd.y > kw0);
        f.pads = real < min(GR, p.n_q - g * GR);
        return f;
    };
    Flags cur_f{false, false, false};
    if (t1 > 0) {
        cur_f = flags_of(ld_const4(p.group + 4 * g_first), ld_const(p.group_real + g_first), g_first);
        issue_stage(g_first, h_first, 0);
        load_small(g_first, h_first, 0);
    }
    // no compiler-visible vector load may be pending inside the stage loop (it would wait for the copies too)
    wait_vmem();
    int g = g_first, hh = 0, b = 0;      // the score role's stage t = (g, hh) in buffer b
    bool live_prev = false;
    for (int t = 0; t <= t1 && t1 > 0; ++t) {
        const bool have = t < t1, have_next = t + 1 < t1;
        const bool full = cur_f.full, live = have && cur_f.live, has_pads = have && cur_f.pads;
        int gn = g, hn = hh + 1;
        if (hn == nh) { hn = 0; gn = g + 1; }
        const int bn = b == NBUF - 1 ? 0 : b + 1;

        wait_vmem();
        if (has_pads) {
            __syncthreads();      // stage t's tiles and row scalars are in LDS
            const int r = tid >> 3, part = tid & 7;       // 512 threads: 8 per row
            if (small_s[b][3][r] == 0) {
                const i32x4 z = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < CPR / 8; ++i) {
                    *reinterpret_cast<i32x4*>(smem + (2 * b) * TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                    *reinterpret_cast<i32x4*>(smem + (2 * b + 1) * TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                }
            }
        }
        __syncthreads();          // stage t is in LDS, P of stage t-1 is visible, everyone has left
                                  // the buffer of stage t-2 and the P buffer of stage t-2
        if (have_next) {
            issue_stage(gn, h_first + hn, bn);
            load_small(gn, h_first + hn, bn);
        }
        int4 gd_n = int4{0, 0, 0, 0};
        int real_n = 0;
        const bool new_group = have_next && gn != g;
        if (new_group) { gd_n = ld_const4(p.group + 4 * gn); real_n = ld_const(p.group_real + gn); }

        if (role == 0) {
            if (live) score_stage(!full);
        } else {
            if (live_prev) grad_stage();
        }

        if (new_group) cur_f = flags_of(gd_n, real_n, gn);
        live_prev = live;
        rotate(b);
        g = gn; hh = hn; b = bn;
    }

    if (whole) {
        if (mykey < p.t_kv) {
            __bf16* op = (role == 0 ? p.dv : p.dk) + ((size_t)mykey * p.hkv + hk) * D;
            const float f = role == 0 ? 1.0f : p.scale;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d = db * 32 + r4 * 8 + half * 4;
                    *reinterpret_cast<bf16x4*>(op + d) = pack4(acc[db][r4 * 4 + 0] * f, acc[db][r4 * 4 + 1] * f,
                                                               acc[db][r4 * 4 + 2] * f, acc[db][r4 * 4 + 3] * f);
                }
        }
    } else {
        // part of a key tile's work: unscaled fp32 partial [dK | dV][key][d], summed by dkv_fixup_kernel
        float* op = p.partial + (size_t)slot * (2 * BNK * D) + (role == 0 ? BNK * D : 0) + (size_t)(kblk * 32 + l32) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = db * 32 + r4 * 8 + half * 4;
                *reinterpret_cast<f32x4*>(op + d) = f32x4{acc[db][r4 * 4 + 0], acc[db][r4 * 4 + 1],
                                                          acc[db][r4 * 4 + 2], acc[db][r4 * 4 + 3]};
            }
    }
  }   // next item
}

// Sums the partial results of the key tiles that were split into several items.
// One workgroup per (tile in order, KV head).
template <int D>
__global__ void __launch_bounds__(256) dkv_fixup_kernel(const BwdParams p) {
    constexpr int BNK = kBwdKeyTile;
    // the item counters of the dK/dV launch that has just finished go back to zero for the next one
    if (blockIdx.x == 0 && threadIdx.x < kLists) p.dkv_counters[threadIdx.x] = 0;
    const int job = (int)blockIdx.x / kMergeSplit, quarter = (int)blockIdx.x % kMergeSplit;
    const int hk = job % p.hkv, r = job / p.hkv;
    const int kt = p.key_order[r];
    const int ways = p.key_ways[kt];
    if (ways == 1) return;                      // one item did the whole tile and wrote dK/dV itself
    const int k0 = kt * BNK, nk = min(BNK, p.t_kv - k0);
    const float* src = p.partial + (size_t)(p.key_slot_base[r] + hk * ways) * (2 * BNK * D);
    constexpr int V4 = D / 4;                   // float4 per row
    constexpr int PER = 2 * BNK * V4 / kMergeSplit;
    for (int e = quarter * PER + threadIdx.x; e < (quarter + 1) * PER; e += 256) {
        const int which = e / (BNK * V4), rem = e % (BNK * V4);
        const int key = rem / V4, d4 = rem % V4;
        if (key >= nk) continue;
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        for (int i = 0; i < ways; ++i)
                sum += *reinterpret_cast<const f32x4*>(src + (size_t)i * (2 * BNK * D) + (size_t)which * BNK * D +
                                                       (size_t)key * D + d4 * 4);
        const float f = which == 0 ? p.scale : 1.0f;
        __bf16* op = (which == 0 ? p.dk : p.dv) + ((size_t)(k0 + key) * p.hkv + hk) * D + d4 * 4;
        *reinterpret_cast<bf16x4*>(op) = pack4(sum[0] * f, sum[1] * f, sum[2] * f, sum[3] * f);
    }
}

// delta, then dK/dV (+ fix-up), then dQ (+ merge), all on the caller's stream.  Running dQ beside
// dK/dV on a second stream was measured: once each kernel keeps every compute unit busy to its end
// the two only get in each other's way (their workgroups cannot share a compute unit's LDS), and the
// step was 4 % slower.
wlb_status launch_bwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, const void* o, const float* lse, const void* d_o, void* dq,
                      void* dk, void* dv, char* ws, size_t off_delta, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    BwdParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.o = (const __bf16*)o; p.d_o = (const __bf16*)d_o; p.lse = lse;
    p.delta = (float*)(ws + off_delta);
    p.lse2 = (float*)(ws + off_delta + align_up(sizeof(float) * (size_t)d.hq * d.n_q, 256));
    p.dq = (__bf16*)dq; p.dk = (__bf16*)dk; p.dv = (__bf16*)dv;
    p.row_lo = (const int32_t*)(ws + L.off_row_lo);
    p.row_hi = (const int32_t*)(ws + L.off_row_hi);
    p.group = (const int32_t*)(ws + L.off_group);
    p.group_real = (const int32_t*)(ws + L.off_group_real);
    p.key_order = (const int32_t*)(ws + L.off_key_order);
    p.key_range = (const int32_t*)(ws + L.off_key_range);
    p.key_ways = (const int32_t*)(ws + L.off_key_ways);
    p.key_item_base = (const int32_t*)(ws + L.off_key_item_base);
    p.key_slot_base = (const int32_t*)(ws + L.off_key_slot_base);
    p.dkv_counters = (int32_t*)(ws + L.off_dkv_counters);
    p.partial = (float*)(ws + off_delta + 2 * align_up(sizeof(float) * (size_t)d.hq * d.n_q, 256));
    p.sched.prefix = (const long long*)(ws + L.off_fwd_prefix);
    p.sched.order = (const int32_t*)(ws + L.off_fwd_order);
    p.sched.n_tiles = L.n_fwd_tiles; p.sched.hkv = d.hkv; p.sched.G = d.hq / d.hkv; p.sched.n_gangs = L.row_gangs;
    gang_weights(1, p.sched.weight);
    p.row_partial = (float*)((char*)p.partial + dkv_partial_bytes(d, L));
    p.block_hull = (const int32_t*)(ws + L.off_block_hull);
    p.tile_short = (const int32_t*)(ws + L.off_tile_short);
    p.n_blocks32 = L.n_blocks32;
    p.gang_clock = (unsigned long long*)(ws + L.off_gang_clock) + 2 * (size_t)L.row_gangs * (d.hq / d.hkv);
    p.n_q = d.n_q; p.t_kv = d.t_kv; p.hq = d.hq; p.hkv = d.hkv;
    p.n_groups = L.n_groups; p.n_tiles = L.n_fwd_tiles; p.n_key_tiles = L.n_key_tiles;
    p.scale = d.scale;
    p.scale_log2e = d.scale * 1.4426950408889634f;

    // workgroups per query tile in the delta pass: enough to fill the GPU, at most one per 256 lanes of the tile
    const size_t tile_iters = (size_t)kFwdTileRows * d.hq * (d.head_dim / 8) / 256;
    const size_t delta_split = std::max<size_t>(1, std::min(tile_iters, (8 * (size_t)compute_units() + L.n_fwd_tiles - 1) / L.n_fwd_tiles));
    const unsigned grid_delta = (unsigned)(delta_split * L.n_fwd_tiles);
    const unsigned grid_dq = (unsigned)L.row_gangs * (unsigned)(d.hq / d.hkv);
    const unsigned grid_dq_items = (unsigned)((L.n_fwd_tiles + 7) / 8) * 8u * (unsigned)d.hq;
    const bool gangs = use_row_gangs(d, L);
    // one workgroup per compute unit, each taking item after item
    const unsigned grid_dkv = (unsigned)std::min(L.dkv_max_items, compute_units());   // one workgroup per compute unit, each taking item after item
    const unsigned grid_fix = (unsigned)(L.n_key_tiles * d.hkv);
    const bool do_delta = !(d.flags & WLB_ATTN_BWD_SKIP_DELTA);
    const bool do_dq = !(d.flags & WLB_ATTN_BWD_SKIP_DQ);
    const bool do_dkv = !(d.flags & WLB_ATTN_BWD_SKIP_DKV);
    p.use_short = use_short_path(d, L) ? 1 : 0;
    // the short-hull dQ kernel forms delta for its own rows (and runs before dK/dV, which reads it);
    // when it does not run, the delta pass covers every row
    p.delta_skips_short = (p.use_short && do_dq) ? 1 : 0;
    // Order: delta, then dK/dV (+ fix-up), then dQ (+ merge) -- except when short-hull units run inside the
    // dQ launch: they leave delta for their rows, which dK/dV reads, so dQ goes first.
    auto run = [&](auto dtag) {
        constexpr int D = decltype(dtag)::value;
        if (do_delta) delta_kernel<D><<<grid_delta, 256, 0, stream>>>(p);
        auto dkv = [&] {
            if (!do_dkv) return;
            dkv_kernel<D><<<grid_dkv, 512, 0, stream>>>(p);
            dkv_fixup_kernel<D><<<grid_fix * kMergeSplit, 256, 0, stream>>>(p);
        };
        if (gangs) {
            dkv();
            if (do_dq) {
                dq_kernel<D><<<grid_dq, 256, 0, stream>>>(p);
                dq_merge_kernel<D><<<grid_dq * kMergeSplit, 256, 0, stream>>>(p);
            }
        } else if (p.use_short) {
            if (do_dq) dq_items_kernel<D><<<grid_dq_items, 256, 0, stream>>>(p);
            dkv();
        } else {
            dkv();
            if (do_dq) dq_items_kernel<D><<<grid_dq_items, 256, 0, stream>>>(p);
        }
    };
    if (d.head_dim == 128) run(std::integral_constant<int, 128>{});
    else run(std::integral_constant<int, 64>{});
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "backward launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

}  // namespace wlb
