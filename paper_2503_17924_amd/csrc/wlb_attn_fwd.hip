// Forward document-masked attention for gfx950 (paper Sections 1 and 3.2 define the mask:
// causal inside a document, nothing across documents; Section 2.1 the data flow: one
// context-parallel rank's query rows against the whole packed sequence's K/V).
//
// One workgroup = one query tile of 128 local rows x one query head.  Each wavefront owns
// QB blocks of 32 rows and keeps, per block, the bf16 Q operands, the running row max and sum
// and the transposed output accumulator O^T[d][q] in registers.  K and V tiles of 64 keys are
// copied global->LDS asynchronously, double buffered, one barrier per tile.  Scores are
// computed transposed, S^T = K Q^T, with the 32x32x16 bf16 MFMA: a lane then holds one query
// column and 16 key rows per block, so the row max/sum are in-register reductions plus one
// exchange between the two lane halves, and the exponentiated block is already laid out as
// the B operand of O^T += V^T P^T.  The V^T operand comes from the row-major V tile through
// LDS transpose reads.
#include <hip/hip_runtime.h>

#include "wlb_device.h"
#include "wlb_internal.h"

namespace wlb {

struct FwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int32_t* row_lo; const int32_t* row_hi; const int32_t* group; const int32_t* order;
    int n_q, t_kv, hq, hkv, n_groups, n_tiles;
    float scale_log2e, scale;
    int exp_flags;
};

template <int D, int QB, int NW>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) fwd_kernel(const FwdParams p) {
    constexpr int BM = 32 * QB * NW;
    static_assert(BM == kFwdTileRows, "tile rows must match the schedule");
    constexpr int BN = 64;
    constexpr int KS = D / 16;         // contraction steps of S^T = K Q^T
    constexpr int DB = D / 32;         // 32-row blocks of O^T
    constexpr int CPR = D / 8;         // 16-byte chunks per row
    constexpr int ROWB = D * 2;        // bytes per LDS row
    constexpr int TILEB = BN * ROWB;   // bytes per tile

    // K0 | K1 | V0 | V1: double-buffered, unpadded, chunk-swizzled tiles
    __shared__ __attribute__((aligned(1024))) char smem[4 * TILEB];

    // ---- which (tile, head) is this workgroup: 8 consecutive blocks go to the 8 XCDs, so XCD x
    // works through ranks x, x+8, ...; the heads of one KV group follow each other on one XCD.
    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    int y = blockIdx.x >> 3;
    const int hh = y % G; y /= G;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_tiles) return;
    const int tile = p.order[rank];
    const int h = hk * G + hh;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;

    // ---- hull and fully visible range of this tile (two groups of 64 rows)
    int k_lo = kPadLo, k_hi = 0, max_lo = 0, min_hi = kPadLo;
    for (int j = 0; j < BM / kGroupRows; ++j) {
        const int g = tile * (BM / kGroupRows) + j;
        if (g < p.n_groups) {
            const int4 d = reinterpret_cast<const int4*>(p.group)[g];
            if (d.y > d.x) { k_lo = min(k_lo, d.x); k_hi = max(k_hi, d.y); max_lo = max(max_lo, d.z); min_hi = min(min_hi, d.w); }
        }
    }
    int jb = 0, je = 0, fb = 0, fe = 0;
    if (k_hi > k_lo) {
        jb = k_lo / BN; je = (k_hi + BN - 1) / BN;
        fb = (max_lo + BN - 1) / BN; fe = min_hi / BN;
        if (fe < fb) fe = fb;
    }

    // ---- start the first K/V tile copy before anything else
    const uint32_t kv_row = (uint32_t)p.hkv * D;
    const uint32_t kv_bytes = ((uint32_t)p.t_kv * kv_row - (uint32_t)hk * D) * 2u;
    BufRsrc krs, vrs;
    krs.init(p.k + (size_t)hk * D, kv_bytes);
    vrs.init(p.v + (size_t)hk * D, kv_bytes);
    TileDma<D, BN, NW> dma;
    dma.init(wave, lane, kv_row);
    auto tile_ptr = [&](int which) { return reinterpret_cast<__bf16*>(smem + which * TILEB); };
    if (jb < je) {
        dma.issue(krs, tile_ptr(0), jb * BN, wave);
        dma.issue(vrs, tile_ptr(2), jb * BN, wave);
    }

    // ---- per-lane rows: Q operands, key interval
    bf16x8 qf[QB][KS];
    int lo[QB], hi[QB], row[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        row[b] = tile * BM + (wave * QB + b) * 32 + l32;
        const bool in = row[b] < p.n_q;
        const int rc = in ? row[b] : p.n_q - 1;
        lo[b] = in ? p.row_lo[rc] : kPadLo;
        hi[b] = in ? p.row_hi[rc] : 0;
        const __bf16* qp = p.q + ((size_t)rc * p.hq + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[b][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    // ---- LDS read offsets (bytes inside a tile).  The swizzle term depends only on the row's
    // low four bits, so the 32-key block / 16-key step enter as compile-time immediates.
    int kaddr[KS], vaddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);      // logical 16-byte chunk
            vaddr[db][t] = key * ROWB + swz<CPR>(key, dch) * 16 + (j16 & 1) * 8;
        }

    f32x16 acc[QB][DB];
    float m[QB], l[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        m[b] = -INFINITY; l[b] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][db][r] = 0.f;
    }
    const float cs = p.scale_log2e;

    for (int j = jb; j < je; ++j) {
        const int cur = (j - jb) & 1;
        wait_vmem();       // this wavefront's share of tile j has landed
        __syncthreads();   // ... and everyone's; everyone is also done reading the other buffer
        if (j + 1 < je) {
            dma.issue(krs, tile_ptr(cur ^ 1), (j + 1) * BN, wave);
            dma.issue(vrs, tile_ptr(2 + (cur ^ 1)), (j + 1) * BN, wave);
        }
        const char* Kc = smem + cur * TILEB;
        const char* Vc = smem + (2 + cur) * TILEB;
        const bool partial = (j < fb) || (j >= fe);
#pragma unroll
        for (int kb = 0; kb < BN / 32; ++kb) {
            // ---- S^T = K Q^T for one block of 32 keys
            f32x16 s[QB];
#pragma unroll
            for (int b = 0; b < QB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kc + kaddr[ks] + kb * 32 * ROWB);
#pragma unroll
                for (int b = 0; b < QB; ++b) s[b] = mfma32(a, qf[b][ks], s[b]);
            }
            if (partial) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j * BN + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
#pragma unroll
                    for (int b = 0; b < QB; ++b)
                        s[b][r] = (key >= lo[b] && key < hi[b]) ? s[b][r] : -INFINITY;
                }
            }
            // ---- online softmax per query column
            bf16x8 pf[QB][2];
#pragma unroll
            for (int b = 0; b < QB; ++b) {
                float mx = fmaxf(s[b][0], s[b][1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[b][r], s[b][r + 1]));
                mx = fmaxf(mx, xhalf(mx));
                const float m_new = fmaxf(m[b], mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = fast_exp2((m[b] - m_use) * cs);
                const float mc = m_use * cs;
                float rs = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = fast_exp2(fmaf(s[b][r], cs, -mc));
                    s[b][r] = e;
                    rs += e;
                }
                l[b] = l[b] * alpha + rs;
                m[b] = m_new;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[b][db][r] *= alpha;
                }
#pragma unroll
                for (int cc = 0; cc < 2; ++cc)
                    pf[b][cc] = pack8(s[b][8 * cc + 0], s[b][8 * cc + 1], s[b][8 * cc + 2], s[b][8 * cc + 3],
                                      s[b][8 * cc + 4], s[b][8 * cc + 5], s[b][8 * cc + 6], s[b][8 * cc + 7]);
            }
            // ---- O^T += V^T P^T.  V^T operand: lane (d = db*32 + l32, half) needs keys
            // {K0 + 4*half + 0..3, K0 + 8 + 4*half + 0..3}: two transpose reads of four keys each
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int koff = (kb * 32 + cc * 16) * ROWB;
                    const bf16x4 v0 = lds_read_tr4(reinterpret_cast<const __bf16*>(Vc + vaddr[db][0] + koff));
                    const bf16x4 v1 = lds_read_tr4(reinterpret_cast<const __bf16*>(Vc + vaddr[db][1] + koff));
                    const bf16x8 a = cat4(v0, v1);
#pragma unroll
                    for (int b = 0; b < QB; ++b) acc[b][db] = mfma32(a, pf[b][cc], acc[b][db]);
                }
            }
        }
    }

    // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const float lt = l[b] + xhalf(l[b]);
        const bool live = (row[b] < p.n_q) && (hi[b] > 0) && (lt > 0.f);
        const float inv = live ? 1.0f / lt : 0.f;
        if (row[b] < p.n_q) {
            __bf16* op = p.o + ((size_t)row[b] * p.hq + h) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d = db * 32 + r4 * 8 + half * 4;
                    bf16x4 out;
                    if (live) out = pack4(acc[b][db][r4 * 4 + 0] * inv, acc[b][db][r4 * 4 + 1] * inv,
                                          acc[b][db][r4 * 4 + 2] * inv, acc[b][db][r4 * 4 + 3] * inv);
                    else out = pack4(0.f, 0.f, 0.f, 0.f);
                    *reinterpret_cast<bf16x4*>(op + d) = out;
                }
            if (half == 0)
                p.lse[(size_t)h * p.n_q + row[b]] = live ? m[b] * p.scale + __logf(lt) : -INFINITY;
        }
    }
}


// ------------------------------------------------------------------------------------------
// Software-pipelined forward: 4 wavefronts x 32 rows, two workgroups per CU (two wavefronts
// per SIMD).  Work advances in blocks of 32 keys.  While the MFMA pipe computes the scores of
// block i+1, the vector ALU exponentiates block i; while it accumulates O^T += V^T P^T for
// block i, the vector ALU reduces the row max of block i+1.  To let the score MFMAs run one
// block ahead without a third buffer, the K tiles are shifted by half a tile against the V
// tiles: K tile j holds keys [64j+32, 64j+96), V tile j holds keys [64j, 64j+64).
template <int D>
__global__ void __launch_bounds__(256, 2) fwd_pipe_kernel(const FwdParams p) {
    constexpr int NW = 4, BM = 128, BN = 64;
    static_assert(BM == kFwdTileRows, "tile rows must match the schedule");
    constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, ROWB = D * 2, TILEB = BN * ROWB;

    __shared__ __attribute__((aligned(1024))) char smem[4 * TILEB];   // K0 | K1 | V0 | V1

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    int y = blockIdx.x >> 3;
    const int hh = y % G; y /= G;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_tiles) return;
    const int tile = p.order[rank];
    const int h = hk * G + hh;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;

    int k_lo = kPadLo, k_hi = 0, max_lo = 0, min_hi = kPadLo;
    for (int j = 0; j < BM / kGroupRows; ++j) {
        const int g = tile * (BM / kGroupRows) + j;
        if (g < p.n_groups) {
            const int4 d = reinterpret_cast<const int4*>(p.group)[g];
            if (d.y > d.x) { k_lo = min(k_lo, d.x); k_hi = max(k_hi, d.y); max_lo = max(max_lo, d.z); min_hi = min(min_hi, d.w); }
        }
    }
    int jb = 0, je = 0, fb = 0, fe = 0;
    if (k_hi > k_lo) {
        jb = k_lo / BN; je = (k_hi + BN - 1) / BN;
        fb = (max_lo + BN - 1) / BN; fe = min_hi / BN;
        if (fe < fb) fe = fb;
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
    auto tile_ptr = [&](int which) { return reinterpret_cast<__bf16*>(smem + which * TILEB); };
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

    // scores of one block of 32 keys; `ka` holds the LDS addresses of the block's K operands
    // for the current buffer, `imm` a compile-time byte offset
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    auto scores = [&](const uint32_t (&ka)[KS], int imm) {
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(ka[ks] + imm));
            s = mfma32(a, qf[ks], s);
        }
        return s;
    };
    // mask (partial tiles only), row max, new running max; returns the rescale factor
    float mc = 0.f;        // running max * scale*log2(e), with -inf replaced by 0
    auto prep = [&](f32x16& s, int key0, bool partial) -> float {
        if (partial) {
            asm volatile("");   // keeps this rare path a real branch (no if-conversion into selects)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + (r >> 2) * 8 + half * 4 + (r & 3);
                s[r] = (key >= lo && key < hi) ? s[r] : -INFINITY;
            }
        }
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
        mx = fmaxf(mx, xhalf(mx));
        const float m_new = fmaxf(m, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2((m - m_use) * cs);
        m = m_new;
        mc = m_use * cs;
        return alpha;
    };

    f32x16 s_cur;
    float alpha = 1.f;
    if (jb < je) {
        wait_vmem();
        __syncthreads();
        uint32_t ka[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) ka[ks] = smem_base + TILEB + kaddr[ks];
        s_cur = scores(ka, 0);                                        // K buffer 1, rows 0..31
        alpha = prep(s_cur, jb * BN, (jb < fb) || (jb >= fe));
        __syncthreads();                                              // K buffer 1 may now be overwritten
    }

    for (int j = jb; j < je; ++j) {
        const int cur = (j - jb) & 1;
        if (j + 1 < je && !(p.exp_flags & 8)) {
            dma.issue(krs, tile_ptr(cur ^ 1), (j + 1) * BN + 32, wave);
            dma.issue(vrs, tile_ptr(2 + (cur ^ 1)), (j + 1) * BN, wave);
        }
        uint32_t ka[KS], va[DB][2];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) ka[ks] = smem_base + cur * TILEB + kaddr[ks];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            va[db][0] = smem_base + (2 + cur) * TILEB + vaddr[db][0];
            va[db][1] = smem_base + (2 + cur) * TILEB + vaddr[db][1];
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            // the running max moved: rescale what has been accumulated so far
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
            }
            // scores of the next block (MFMA) against exponentials of this one (vector ALU)
            f32x16 s_next = scores(ka, kb * 32 * ROWB);
            float rs = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = fast_exp2(fmaf(s_cur[r], cs, -mc));
                s_cur[r] = e;
                rs += e;
            }
            l = l * alpha + rs;
            bf16x8 pf[2];
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
                pf[cc] = pack8(s_cur[8 * cc + 0], s_cur[8 * cc + 1], s_cur[8 * cc + 2], s_cur[8 * cc + 3],
                               s_cur[8 * cc + 4], s_cur[8 * cc + 5], s_cur[8 * cc + 6], s_cur[8 * cc + 7]);
            // O^T += V^T P^T (MFMA) against the row max of the next block (vector ALU)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int voff = (kb * 32 + cc * 16) * ROWB;
                    const bf16x4 v0 = lds_read_tr4_at(va[db][0] + voff);
                    const bf16x4 v1 = lds_read_tr4_at(va[db][1] + voff);
                    acc[db] = mfma32(cat4(v0, v1), pf[cc], acc[db]);
                }
            const int jn = kb == 0 ? j : j + 1;                       // tile of the next block
            alpha = prep(s_next, jn * BN + (kb == 0 ? 32 : 0), (jn < fb) || (jn >= fe));
            s_cur = s_next;
        }
        wait_vmem();
        __syncthreads();
    }

    const float lt = l + xhalf(l);
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

template <int D, int QB, int NW>
static void launch_one(const FwdParams& p, unsigned grid, hipStream_t stream) {
    fwd_kernel<D, QB, NW><<<grid, NW * 64, 0, stream>>>(p);
}

wlb_status launch_fwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, void* o, float* lse, char* ws, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    FwdParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.o = (__bf16*)o; p.lse = lse;
    p.row_lo = (const int32_t*)(ws + L.off_row_lo);
    p.row_hi = (const int32_t*)(ws + L.off_row_hi);
    p.group = (const int32_t*)(ws + L.off_group);
    p.order = (const int32_t*)(ws + L.off_fwd_order);
    p.n_q = d.n_q; p.t_kv = d.t_kv; p.hq = d.hq; p.hkv = d.hkv;
    p.n_groups = L.n_groups; p.n_tiles = L.n_fwd_tiles;
    p.scale = d.scale;
    p.scale_log2e = d.scale * 1.4426950408889634f;
    p.exp_flags = getenv("WLB_EXP") ? atoi(getenv("WLB_EXP")) : 0;
    const unsigned grid = (unsigned)((L.n_fwd_tiles + 7) / 8) * 8u * (unsigned)d.hq;
    static const int variant = getenv("WLB_FWD_VARIANT") ? atoi(getenv("WLB_FWD_VARIANT")) : 2;
    if (variant == 2) {
        if (d.head_dim == 128) fwd_pipe_kernel<128><<<grid, 256, 0, stream>>>(p);
        else fwd_pipe_kernel<64><<<grid, 256, 0, stream>>>(p);
    } else if (d.head_dim == 128) {
        if (variant == 1) launch_one<128, 1, 4>(p, grid, stream);
        else launch_one<128, 2, 2>(p, grid, stream);
    } else {
        if (variant == 1) launch_one<64, 1, 4>(p, grid, stream);
        else launch_one<64, 2, 2>(p, grid, stream);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "forward launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

}  // namespace wlb
