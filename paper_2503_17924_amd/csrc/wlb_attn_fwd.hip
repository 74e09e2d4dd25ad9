// Forward document-masked attention for gfx950 (paper Sections 1 and 3.2 define the mask:
// causal inside a document, nothing across documents; Section 2.1 the data flow: one
// context-parallel rank's query rows against the whole packed sequence's K/V).
//
// A piece of work = one query tile of 128 local rows x one query head (or a part of its key
// range), run by a workgroup of four wavefronts of 32 rows.  Two schedules hand out the pieces:
// a fixed set of workgroups that each walk a share of all the work (RowSched in wlb_device.h),
// or one workgroup per tile and head.  A wavefront keeps its bf16 Q operands, the running row
// max / sum and the transposed output accumulator O^T[d][q] in registers.  Scores are computed transposed, S^T = K Q^T,
// with the 32x32x16 bf16 MFMA: a lane then holds one query column and 16 key rows per block,
// so the row max/sum are in-register reductions plus one exchange between the two lane
// halves, and the exponentiated block is already laid out as the B operand of
// O^T += V^T P^T.  The V^T operand comes from the row-major V tile through LDS transpose
// reads.  K and V tiles of 64 keys are copied global->LDS asynchronously, double buffered.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "wlb_device.h"
#include "wlb_internal.h"

namespace wlb {

struct FwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int32_t* row_lo; const int32_t* row_hi; const int32_t* group;
    RowSched sched;            // which query tiles, heads and key ranges a workgroup works on
    float* partial;            // partial results of the tiles cut at a gang boundary
    const int32_t* block_hull; const int32_t* tile_short;   // short-hull path (see fwd_short_unit)
    unsigned long long* gang_clock;   // [workgroup][2]: real-time counter at the start / end of a gang kernel's workgroup
    int n_q, t_kv, hq, hkv, n_groups, n_tiles, n_blocks32, use_short;
    float scale_log2e, scale;
};

// One piece of work: key tiles [pc.a, pc.b) of the pc.c the query tile pc.tile sees, for query head
// pc.hk * G + pc.member.  A whole tile (pc.slot < 0) writes O and LSE; a part writes its
// unnormalised accumulator, row sums and reference exponents as a partial result.
template <int D>
__device__ __forceinline__ void fwd_piece(const FwdParams& p, char* smem, const RowPiece& pc) {
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
        // this piece's part of the tile's key tiles; the first kRowItemOverhead units of a tile's
        // stretch of the work line stand for its fixed cost and hold no key tile
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
    TileDma<D, 32, NW> dma_half;
    dma_half.init(wave, lane, kv_row);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    auto tile_ptr = [&](int which) { return smem_base + (uint32_t)(which * TILEB); };
    if (jb < je) {
        dma_half.issue(krs, tile_ptr(1), jb * BN, wave);            // keys [64jb, 64jb+32) for the first scores
        dma.issue(krs, tile_ptr(0), jb * BN + 32, wave);            // shifted K tile jb
        dma.issue(vrs, tile_ptr(2), jb * BN, wave);                 // V tile jb
    }

    const int row = tile * BM + wave * 32 + l32;
    const bool in = row < p.n_q;
    const int rc = in ? row : p.n_q - 1;
    const int lo = in ? p.row_lo[rc] : kPadLo;
    const int hi = in ? p.row_hi[rc] : 0;
    // Key tiles this wavefront needs no element-wise mask for: only outside [fb, fe) does it mask.  Inside,
    // the rows of the wavefront's first document see every key; rows of later documents in the same
    // wavefront (a tile that straddles a document boundary has one such wavefront) see none of them and
    // stay switched off as whole lanes until the range ends (`parked`).
    bool parked;
    unmasked_tiles<BN>(lo, hi, hi > 0, fb, fe, parked);
    bf16x8 qf[KS];
    {
        const __bf16* qp = p.q + ((size_t)rc * p.hq + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    int kaddr[KS], vaddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            vaddr[db][t] = key * ROWB + swz<CPR>(key, dch) * 16 + (j16 & 1) * 8;
        }

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float cs = p.scale_log2e;

    // ---- LDS addresses: per-lane registers that already contain the tile base, so that inside
    // the (two-fold unrolled) tile loop every access is register + immediate
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] += smem_base;
#pragma unroll
    for (int db = 0; db < DB; ++db) { vaddr[db][0] += smem_base; vaddr[db][1] += smem_base; }

    auto scores = [&](int imm) __attribute__((always_inline)) {
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(kaddr[ks] + imm));
            s = mfma32(a, qf[ks], s);
        }
        return s;
    };
    auto block_max = [&](const f32x16& s) __attribute__((always_inline)) {
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
        return fmaxf(mx, xhalf(mx));
    };
    // The exponentials are taken against a reference m that follows the running row max lazily:
    // it moves only when a block's max exceeds it by more than kSlack (in log2 units), which keeps
    // every exponential below 2^kSlack and makes the rescaling of the accumulator a rare event.
    constexpr float kSlack = 8.0f;
    float mc = 0.f;                 // m * scale*log2(e), 0 while m is still -inf
    // mc + kSlack: a block max (scaled) above this forces an update.  A parked lane sees no key yet: its
    // limit is +inf so that the scores it computes meanwhile never ask for an update, and its bias (added
    // to the reference of the exponentials) is +inf so that they contribute nothing.
    float lim = parked ? INFINITY : -INFINITY;
    float bias_base = parked ? INFINITY : 0.f;
    // rare path, outside the straight-line block: mask a block of a partial tile, recompute its max
    auto mask_block = [&](f32x16& s, int key0) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = key0 + (r >> 2) * 8 + half * 4 + (r & 3);
            s[r] = (key >= lo && key < hi) ? s[r] : -INFINITY;
        }
        return block_max(s);
    };
    // a block outside the fully visible range: when every row sees either all of its 32 keys or none
    // (rows of another document in the same wavefront) whole lanes are switched off; the element-wise
    // mask is left to the blocks a row's interval really cuts (diagonal, document edges)
    // (a lane is switched off by adding +inf to the reference its exponentials are taken against)
    // past the unmasked range the parked lanes take part again with the limit that belongs to their reference
    auto unpark = [&]() __attribute__((always_inline)) {
        lim = parked ? ((m == -INFINITY) ? -INFINITY : mc + kSlack) : lim;
        parked = false;
        bias_base = 0.f;
    };
    if (jb >= fe) unpark();
    float bias_cur = bias_base, bias_next = bias_base;
    auto mask_next = [&](f32x16& s, int key0, float mx) __attribute__((always_inline)) {
        if (key0 >= fe * BN) unpark();
        const bool none = (key0 + 32 <= lo) || (key0 >= hi);
        const bool all = (key0 >= lo) && (key0 + 32 <= hi);
        if (__any(!(none || all))) {
            bias_next = 0.f;
            return mask_block(s, key0);
        }
        // Every row sees all or none of this block.  That stays so up to the next edge of a row's interval
        // (the end of a row that sees the block, the start of one that is still to come): the key tiles
        // from the next one up to that edge become the unmasked range, with the rows that see nothing
        // parked.  A wavefront that holds rows of two chunks of one document (or of two documents)
        // crosses the keys between them at full speed this way.
        int edge = none ? (lo >= key0 + 32 ? lo : kPadLo) : hi;
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) edge = min(edge, __shfl_xor(edge, o));
        const int j_next = key0 / BN + 1, j_edge = uniform(edge / BN);
        if (j_edge > j_next) {
            fb = uniform(j_next);
            fe = j_edge;
            parked = none;
            bias_base = none ? INFINITY : 0.f;
            lim = none ? INFINITY : lim;
        }
        bias_next = none ? INFINITY : 0.f;
        return none ? -INFINITY : mx;
    };
    // rare path: move the reference up to the running max and rescale what has been accumulated
    auto move_reference = [&](float mx) __attribute__((always_inline)) {
        mx = parked ? -INFINITY : mx;
        const float m_new = fmaxf(m, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(fmaf(m, cs, -m_use * cs));     // m = -inf gives 0 (nothing accumulated yet)
        const float a2 = (m == -INFINITY) ? 0.f : alpha;
        m = m_new;
        mc = m_use * cs;
        lim = parked ? INFINITY : ((m_new == -INFINITY) ? -INFINITY : mc + kSlack);
        l *= a2;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] *= a2;
    };

    f32x16 s_cur;
    if (jb < je) {
        wait_vmem();
        __syncthreads();
        s_cur = scores(TILEB);                                        // K buffer 1, rows 0..31
        float mx = block_max(s_cur);
        if ((jb < fb) || (jb >= fe)) mx = mask_block(s_cur, jb * BN);
        move_reference(mx);
        __syncthreads();                                              // K buffer 1 may now be overwritten
    }

    // one 32-key block: a single straight-line region (next block's scores and this block's
    // accumulation on the MFMA pipe, this block's exponentials and the next block's max on the
    // vector ALU), followed by the two rare fix-ups
    auto block_step = [&](int kimm, int vimm, int next_key0, bool next_partial) __attribute__((always_inline)) {
        f32x16 s_next = scores(kimm);
        float rs = 0.f;
        const float mcb = mc + bias_cur;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float e = fast_exp2(fmaf(s_cur[r], cs, -mcb));
            s_cur[r] = e;
            rs += e;
        }
        l += rs;
        bf16x8 pf[2];
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
            pf[cc] = pack8(s_cur[8 * cc + 0], s_cur[8 * cc + 1], s_cur[8 * cc + 2], s_cur[8 * cc + 3],
                           s_cur[8 * cc + 4], s_cur[8 * cc + 5], s_cur[8 * cc + 6], s_cur[8 * cc + 7]);
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x4 v0 = lds_read_tr4_at(vaddr[db][0] + vimm + cc * 16 * ROWB);
                const bf16x4 v1 = lds_read_tr4_at(vaddr[db][1] + vimm + cc * 16 * ROWB);
                acc[db] = mfma32(cat4(v0, v1), pf[cc], acc[db]);
            }
        float mx = block_max(s_next);
        if (next_partial) {
            asm volatile("");
            mx = mask_next(s_next, next_key0, mx);
        }
        if (__any(mx * cs > lim)) {
            asm volatile("");
            move_reference(mx);
        }
        s_cur = s_next;
        bias_cur = bias_next;
        bias_next = bias_base;
    };
    auto tile_step = [&](int j, auto cur_tag) __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_tag)::value;
        if (j + 1 < je) {
            dma.issue(krs, tile_ptr(cur ^ 1), (j + 1) * BN + 32, wave);
            dma.issue(vrs, tile_ptr(2 + (cur ^ 1)), (j + 1) * BN, wave);
        }
        const bool part0 = (j < fb) || (j >= fe);
        block_step(cur * TILEB, (2 + cur) * TILEB, j * BN + 32, part0);
        const bool part1 = (j + 1 < fb) || (j + 1 >= fe);        // the first step may have set a new range
        block_step(cur * TILEB + 32 * ROWB, (2 + cur) * TILEB + 32 * ROWB, (j + 1) * BN, part1);
        wait_vmem();
        __syncthreads();
    };
    // The compiler's wait-count bookkeeping does not see the asynchronous copies.  Draining the
    // vector-memory counter here, on every path into the loop, keeps it from placing counted waits
    // for the Q operand loads inside the loop, where they would wait for the copies in flight.
    wait_vmem();
    for (int j = jb; j < je; j += 2) {
        tile_step(j, std::integral_constant<int, 0>{});
        if (j + 1 < je) tile_step(j + 1, std::integral_constant<int, 1>{});
    }

    const float lt = l + xhalf(l);
    if (pc.slot >= 0) {
        // part of a tile: accumulator [row][d], row sums and reference exponents (-inf: no key seen)
        float* part = p.partial + (size_t)pc.slot * (BM * D + 2 * BM);
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
            if (half == 0) {
                part[BM * D + rl] = lt;
                part[BM * D + BM + rl] = (m == -INFINITY) ? -INFINITY : mc;
            }
        }
        return;
    }
    const bool live = in && (hi > 0) && (lt > 0.f);
    const float inv = live ? 1.0f / lt : 0.f;
    if (in) {
        __bf16* op = p.o + ((size_t)row * p.hq + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = db * 32 + r4 * 8 + half * 4;
                bf16x4 out;
                if (live) out = pack4(acc[db][r4 * 4 + 0] * inv, acc[db][r4 * 4 + 1] * inv,
                                      acc[db][r4 * 4 + 2] * inv, acc[db][r4 * 4 + 3] * inv);
                else out = pack4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<bf16x4*>(op + d) = out;
            }
        // the look-ahead block past the last tile is fully masked, so m is the true row max
        if (half == 0) p.lse[(size_t)h * p.n_q + row] = live ? m * p.scale + __logf(lt) : -INFINITY;
    }
}

// Two workgroups per CU (two wavefronts per SIMD).  Work advances in blocks of 32 keys, each
// one straight-line region: the MFMA pipe computes the scores of block i+1 and accumulates
// O^T += V^T P^T of block i while the vector ALU exponentiates block i and reduces the row max
// of block i+1 (on gfx950 the two overlap only inside one wavefront's instruction stream).
// To let the score MFMAs run one block ahead without a third buffer, the K tiles are shifted
// by half a tile against the V tiles: K tile j holds keys [64j+32, 64j+96), V tile j holds
// keys [64j, 64j+64).  A workgroup walks its gang's share of the work line piece by piece.
template <int D>
__global__ void __launch_bounds__(256, 2) fwd_kernel(const FwdParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[4 * 64 * D * 2];   // K0 | K1 | V0 | V1
    const unsigned long long t_start = wall_clock64();
    RowWalk walk;
    walk.start(p.sched, (int)blockIdx.x);
    RowPiece pc;
    while (walk.next(p.sched, pc)) fwd_piece<D>(p, smem, pc);
    if (threadIdx.x == 0) {
        p.gang_clock[2 * blockIdx.x] = t_start;
        p.gang_clock[2 * blockIdx.x + 1] = wall_clock64();
    }
}

// Short-hull tiles (documents of a few dozen tokens, where a tile's rows see only the keys next to
// them: the short-chunk case of paper Section 5.2).  There the general piece of work is bound by
// latency: per (tile, head) it fetches K/V, waits, and computes a handful of blocks.  A short-hull
// unit is one block of 32 rows and one KV head, run by a workgroup of the one-workgroup-per-item
// launch: it copies the (at most 96) keys the block sees into LDS
// once -- K and V, in one shot -- and its four wavefronts then work independently, one query head
// each at a time (heads w, w+4, ... of the KV head), with no further barrier.  Per head a wavefront
// loads its 32 Q rows as whole rows and passes them through a staging tile of its own into the MFMA
// operand layout (loading the operand straight from global memory would touch 32 rows x 32 bytes per
// instruction), computes the scores of the up to three 32-key blocks, the exact row maximum, the
// exponentials and O^T += V^T P^T, and sends O through the staging tile so that it leaves in whole
// rows as well.  Eight wavefronts per compute unit keep Q loads and O stores in flight; K/V
// traffic is one LDS fill per 32 rows and KV head instead of one per head.
template <int D>
struct ShortTile {
    static constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, ROWB = D * 2;
    static constexpr int HULL = kShortHullKeys, NB = HULL / 32, NW = 4;
    static constexpr int STAGE = kShortBlockRows * ROWB;              // one wavefront's staging tile: 32 rows
    static constexpr int LDS_BYTES = 2 * HULL * ROWB + NW * STAGE;    // K window | V window | staging tiles
    static constexpr int RPI = 64 / CPR;                              // rows moved by one 64 x 16-byte instruction
};

template <int D>
__device__ __forceinline__ void fwd_short_unit(const FwdParams& p, char* smem, int blk, int hk) {
    using T = ShortTile<D>;
    constexpr int NW = T::NW, KS = T::KS, DB = T::DB, CPR = T::CPR, ROWB = T::ROWB, HULL = T::HULL, NB = T::NB;
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
    const buf_rsrc_t q_buf = make_buf(p.q, (uint32_t)p.n_q * q_row_bytes), o_buf = make_buf(p.o, (uint32_t)p.n_q * q_row_bytes);
    const int row_voff = RowBlock<D>::lane_off(lane, q_row_bytes);
    auto head_soff = [&](int hs) { return uniform((uint32_t)row0 * q_row_bytes + (uint32_t)(hk * G + hs) * ROWB); };

    if (h_hi <= h_lo) {
        // no real row in this block: O = 0, LSE = -inf for every head of the KV head
        RowBlock<D> zero;
#pragma unroll
        for (int i = 0; i < RowBlock<D>::N; ++i) zero.v[i] = i32x4{0, 0, 0, 0};
        for (int hs = wave; hs < G; hs += NW) {
            zero.store(o_buf, row_voff, head_soff(hs), q_row_bytes);
            if (in && half == 0) p.lse[(size_t)(hk * G + hs) * p.n_q + row] = -INFINITY;
        }
        return;
    }
    const int kstart = h_lo & ~31;
    const int nblk = (h_hi - kstart + 31) >> 5;          // 1 .. NB (the schedule marks the tile short only then)

    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t stage = uniform(smem_base + 2 * HULL * ROWB + (uint32_t)wave * T::STAGE);
    const uint32_t kv_row = (uint32_t)p.hkv * D;
    const uint32_t kv_bytes = ((uint32_t)p.t_kv * kv_row - (uint32_t)hk * D) * 2u;
    BufRsrc krs, vrs;
    krs.init(p.k + (size_t)hk * D, kv_bytes);
    vrs.init(p.v + (size_t)hk * D, kv_bytes);
    TileDma<D, 32 * NW, NW> dma;                          // wavefront w copies the 32-key block w
    static_assert(TileDma<D, 32 * NW, NW>::PER * TileDma<D, 32 * NW, NW>::RPI == 32, "one 32-key block per wavefront");
    dma.init(wave, lane, kv_row);
    if (wave < nblk) {
        dma.issue(krs, smem_base, kstart, wave);
        dma.issue(vrs, smem_base + HULL * ROWB, kstart, wave);
    }

    const int lo = in ? p.row_lo[rc] : kPadLo;
    const int hi = in ? p.row_hi[rc] : 0;
    const bool real = hi > 0;

    int kaddr[KS], vaddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            vaddr[db][t] = smem_base + HULL * ROWB + key * ROWB + swz<CPR>(key, dch) * 16 + (j16 & 1) * 8;
        }
    const float cs = p.scale_log2e;

    wait_vmem();
    __syncthreads();              // the key window is in LDS; from here on the wavefronts do not meet again

#pragma nounroll
    for (int hs = wave; hs < G; hs += NW) {
        const int h = hk * G + hs;
        // this head's Q rows: whole rows into registers, then through the staging tile into the operand layout
        // (eight wavefronts per compute unit cover each other's load latency)
        {
            RowBlock<D> q_rows;
            q_rows.load(q_buf, row_voff, head_soff(hs), q_row_bytes);
            q_rows.to_tile(stage, lane);
        }
        bf16x8 qf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(stage + kaddr[ks]));

        f32x16 s[NB];
        float mx = -INFINITY;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = -INFINITY;
            if (b < nblk) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(smem_base + kaddr[ks] + b * 32 * ROWB));
                    s[b] = mfma32(a, qf[ks], s[b]);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kstart + b * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    s[b][r] = (key >= lo && key < hi) ? s[b][r] : -INFINITY;
                    mx = fmaxf(mx, s[b][r]);
                }
            }
        }
        mx = fmaxf(mx, xhalf(mx));
        const float mc = (mx == -INFINITY) ? 0.f : mx * cs;
        f32x16 acc[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
        float l = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = fast_exp2(fmaf(s[b][r], cs, -mc));
                    s[b][r] = e;
                    l += e;
                }
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const bf16x8 pf = pack8(s[b][8 * cc + 0], s[b][8 * cc + 1], s[b][8 * cc + 2], s[b][8 * cc + 3],
                                            s[b][8 * cc + 4], s[b][8 * cc + 5], s[b][8 * cc + 6], s[b][8 * cc + 7]);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const int off = (b * 32 + cc * 16) * ROWB;
                        const bf16x4 v0 = lds_read_tr4_at(vaddr[db][0] + off);
                        const bf16x4 v1 = lds_read_tr4_at(vaddr[db][1] + off);
                        acc[db] = mfma32(cat4(v0, v1), pf, acc[db]);
                    }
                }
            }
        }
        const float lt = l + xhalf(l);
        const bool live = real && (lt > 0.f);
        const float inv = live ? 1.0f / lt : 0.f;
        // O rows through the staging tile (its Q rows are in registers by now): written in the
        // accumulator's layout, read back and stored as whole rows
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *reinterpret_cast<WLB_LDS bf16x4*>((uintptr_t)(stage + l32 * ROWB + swz<CPR>(l32, db * 4 + r4) * 16 + half * 8)) =
                    pack4(acc[db][r4 * 4 + 0] * inv, acc[db][r4 * 4 + 1] * inv, acc[db][r4 * 4 + 2] * inv, acc[db][r4 * 4 + 3] * inv);
        RowBlock<D> o_rows;
        o_rows.from_tile(stage, lane);
        o_rows.store(o_buf, row_voff, head_soff(hs), q_row_bytes);
        if (in && half == 0) p.lse[(size_t)h * p.n_q + row] = live ? mx * p.scale + __logf(lt) : -INFINITY;
        wait_lds();                                 // the staging tile has been read back
    }
}

// The other schedule: one workgroup per (query tile in order, query head), dispatched heaviest
// first.  With many tiles per workgroup slot the hardware's dynamic dispatch balances the load by
// itself and adapts to whatever makes workgroups differ in speed; the gangs' fixed shares win when
// there are only a few tiles per slot (long documents spread over many context-parallel ranks).
template <int D>
__global__ void __launch_bounds__(256, 2) fwd_items_kernel(const FwdParams p) {
    constexpr int kLds = ShortTile<D>::LDS_BYTES > 4 * 64 * D * 2 ? ShortTile<D>::LDS_BYTES : 4 * 64 * D * 2;
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
        // a short-hull tile: its four blocks of 32 rows are units of their own, each for all heads of the
        // KV head; the tile's workgroups of this KV head share them out by member
        constexpr int per_tile = kFwdTileRows / kShortBlockRows;
        for (int j = pc.member; j < per_tile; j += G) {
            const int blk = pc.tile * per_tile + j;
            if (blk < p.n_blocks32) fwd_short_unit<D>(p, smem, blk, pc.hk);
        }
        return;
    }
    pc.c = (int)(ld_const64(p.sched.prefix + rank + 1) - ld_const64(p.sched.prefix + rank));
    pc.a = 0; pc.b = pc.c; pc.slot = -1;
    fwd_piece<D>(p, smem, pc);
}

// Combines the partial results of a query tile that was cut at gang boundaries.  One workgroup per
// (gang, member): it acts if its gang's last piece is the first part of a tile, and then takes
// that part and the following gangs' first pieces.  With reference exponents e_i (log2 units), row
// sums l_i and accumulators A_i:  E = max e_i,  L = sum l_i 2^(e_i - E),  O = sum A_i 2^(e_i - E) / L,
// LSE = (E + log2 L) ln 2.
template <int D>
__global__ void __launch_bounds__(256) fwd_merge_kernel(const FwdParams p) {
    constexpr int BM = kFwdTileRows, PF = BM * D + 2 * BM, V4 = D / 4;
    const RowSched& s = p.sched;
    // kMergeSplit workgroups share a tile's rows: the work is a few dependent loads per element, so
    // the launch needs many wavefronts in flight rather than long loops
    const int job = (int)blockIdx.x / kMergeSplit, quarter = (int)blockIdx.x % kMergeSplit;
    const int gang = job / s.G, member = job % s.G;
    RowCut cut;
    if (!cut.find(s, gang)) return;
    const int tile = cut.tile;
    const int h = cut.hk * s.G + member;
    auto part = [&](int slot) { return p.partial + ((size_t)slot * s.G + member) * PF; };
    const float* first = part(cut.first_slot());
    constexpr int CAP = 32;
    __shared__ int s_slots[CAP], s_count;
    const int n_later = gather_later_parts<CAP>(cut, s_slots, &s_count);
    auto later_parts = [&](auto f) __attribute__((always_inline)) {
        if (n_later <= CAP) {
            for (int i = 0; i < n_later; ++i) f(part(s_slots[i]));
        } else {
            cut.later_parts([&](int slot) { f(part(slot)); });
        }
    };
    constexpr int PER = BM * V4 / kMergeSplit;
    for (int e = quarter * PER + threadIdx.x; e < (quarter + 1) * PER; e += 256) {
        const int rl = e / V4, d4 = e % V4;
        const int row = tile * BM + rl;
        if (row >= p.n_q) continue;
        float E = first[BM * D + BM + rl];
        later_parts([&](const float* pp) { E = fmaxf(E, pp[BM * D + BM + rl]); });
        float L = 0.f;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        auto add = [&](const float* pp) __attribute__((always_inline)) {
            const float ei = pp[BM * D + BM + rl];
            if (ei == -INFINITY) return;
            const float wgt = fast_exp2(ei - E);
            L += wgt * pp[BM * D + rl];
            o += wgt * *reinterpret_cast<const f32x4*>(pp + (size_t)rl * D + d4 * 4);
        };
        if (E > -INFINITY) {
            add(first);
            later_parts(add);
        }
        const bool live = p.row_hi[row] > 0 && L > 0.f;
        const float inv = live ? 1.0f / L : 0.f;
        *reinterpret_cast<bf16x4*>(p.o + ((size_t)row * p.hq + h) * D + d4 * 4) =
            live ? pack4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv) : pack4(0.f, 0.f, 0.f, 0.f);
        if (d4 == 0) p.lse[(size_t)h * p.n_q + row] = live ? (E + __log2f(L)) * 0.6931471805599453f : -INFINITY;
    }
}

wlb_status launch_fwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, void* o, float* lse, char* ws, size_t off_row_partial, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    FwdParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.o = (__bf16*)o; p.lse = lse;
    p.row_lo = (const int32_t*)(ws + L.off_row_lo);
    p.row_hi = (const int32_t*)(ws + L.off_row_hi);
    p.group = (const int32_t*)(ws + L.off_group);
    p.sched.prefix = (const long long*)(ws + L.off_fwd_prefix);
    p.sched.order = (const int32_t*)(ws + L.off_fwd_order);
    p.sched.n_tiles = L.n_fwd_tiles; p.sched.hkv = d.hkv; p.sched.G = d.hq / d.hkv; p.sched.n_gangs = L.row_gangs;
    gang_weights(0, p.sched.weight);
    p.partial = (float*)(ws + off_row_partial);
    p.n_q = d.n_q; p.t_kv = d.t_kv; p.hq = d.hq; p.hkv = d.hkv;
    p.n_groups = L.n_groups; p.n_tiles = L.n_fwd_tiles;
    p.block_hull = (const int32_t*)(ws + L.off_block_hull);
    p.tile_short = (const int32_t*)(ws + L.off_tile_short);
    p.n_blocks32 = L.n_blocks32;
    p.use_short = use_short_path(d, L) ? 1 : 0;
    p.gang_clock = (unsigned long long*)(ws + L.off_gang_clock);
    p.scale = d.scale;
    p.scale_log2e = d.scale * 1.4426950408889634f;
    if (use_row_gangs(d, L)) {
        const unsigned grid = (unsigned)L.row_gangs * (unsigned)(d.hq / d.hkv);
        if (d.head_dim == 128) {
            fwd_kernel<128><<<grid, 256, 0, stream>>>(p);
            fwd_merge_kernel<128><<<grid * kMergeSplit, 256, 0, stream>>>(p);
        } else {
            fwd_kernel<64><<<grid, 256, 0, stream>>>(p);
            fwd_merge_kernel<64><<<grid * kMergeSplit, 256, 0, stream>>>(p);
        }
    } else {
        const unsigned grid = (unsigned)((L.n_fwd_tiles + 7) / 8) * 8u * (unsigned)d.hq;
        if (d.head_dim == 128) fwd_items_kernel<128><<<grid, 256, 0, stream>>>(p);
        else fwd_items_kernel<64><<<grid, 256, 0, stream>>>(p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "forward launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

}  // namespace wlb
