// Backward document-masked attention for gfx950.  The paper measures forward+backward
// latency of the attention kernel (Section 6.4) without restating the derivative; this is the
// standard one: with P = exp(scale*Q K^T - LSE) on the visible (same-document, causal) pairs
// and delta_i = <dO_i, O_i>,
//     dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale * dS K,  dK = scale * dS^T Q,
// dK/dV summed over the query heads that share a KV head.  As in all-gather context
// parallelism (Section 2.1) dK/dV hold only the calling rank's rows' contribution.
//
// Three kernels, no atomics, deterministic:
//   delta_kernel  delta[h][i] = sum_d dO*O (0 for padding rows)
//   dq_kernel     query-stationary, same tiling as the forward: S^T and dP^T per lane column,
//                 dQ^T += K^T dS^T with K^T read from LDS by transpose reads
//   dkv_kernel    key-stationary: a workgroup owns 128 keys of one KV head (32 per wavefront,
//                 their K and V MFMA operands live in registers), streams the row groups that
//                 can see them through LDS for every query head of the KV group, and keeps
//                 dK^T, dV^T in registers until the single final store.
// Q / dO / K tiles that are read both row-wise (b128) and column-wise (transpose reads) are
// stored unpadded with an XOR swizzle of their 16-byte chunks that makes both patterns
// bank-conflict free.
#include <hip/hip_runtime.h>

#include "wlb_device.h"
#include <type_traits>

#include "wlb_internal.h"

namespace wlb {

struct BwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* o; const __bf16* d_o;
    const float* lse; float* delta; float* lse2;
    __bf16* dq; __bf16* dk; __bf16* dv;
    const int32_t* row_lo; const int32_t* row_hi; const int32_t* group; const int32_t* group_real;
    const int32_t* fwd_order; const int32_t* key_order; const int32_t* key_range;
    int n_q, t_kv, hq, hkv, n_groups, n_tiles, n_key_tiles;
    float scale_log2e, scale;
    int exp_flags;
};

// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) delta_kernel(const BwdParams p) {
    constexpr int LPR = D / 8;                       // lanes per (row, head)
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t rh = idx / LPR;                     // row * hq + head
    const int c = (int)(idx % LPR);
    const size_t total = (size_t)p.n_q * p.hq;
    float acc = 0.f;
    if (rh < total) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(p.d_o + rh * D + c * 8);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(p.o + rh * D + c * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (rh < total && c == 0) {
        const int row = (int)(rh / p.hq), h = (int)(rh % p.hq);
        const bool real = p.row_hi[row] > 0;
        p.delta[(size_t)h * p.n_q + row] = real ? acc : 0.f;
        // LSE in log2 units for the dK/dV kernel; +inf makes every probability of a padding row 0
        p.lse2[(size_t)h * p.n_q + row] = real ? p.lse[(size_t)h * p.n_q + row] * 1.4426950408889634f : INFINITY;
    }
}

// ------------------------------------------------------------------------------------------
// dQ: one workgroup = 128 query rows x one head; wavefront = QB blocks of 32 rows.
template <int D, int QB, int NW>
__global__ void __launch_bounds__(NW * 64) dq_kernel(const BwdParams p) {
    constexpr int BM = 32 * QB * NW;
    static_assert(BM == kFwdTileRows, "tile rows must match the schedule");
    constexpr int BN = 64, NT = NW * 64, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int VSTR = D + 8;

    __shared__ __attribute__((aligned(16))) __bf16 Ks[BN * D];       // swizzled
    __shared__ __attribute__((aligned(16))) __bf16 Vs[BN * VSTR];    // padded, row reads only

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    int y = blockIdx.x >> 3;
    const int hh = y % G; y /= G;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_tiles) return;
    const int tile = p.fwd_order[rank];
    const int h = hk * G + hh;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;

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

    bf16x8 qf[QB][KS], dof[QB][KS];
    int lo[QB], hi[QB], row[QB];
    float lsec[QB], dl[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        row[b] = tile * BM + (wave * QB + b) * 32 + l32;
        const bool in = row[b] < p.n_q;
        const int rc = in ? row[b] : p.n_q - 1;
        lo[b] = in ? p.row_lo[rc] : kPadLo;
        hi[b] = in ? p.row_hi[rc] : 0;
        const bool real = hi[b] > 0;
        // padding rows: zero operands and LSE = +inf make P, dS and dQ exactly 0
        lsec[b] = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;
        dl[b] = real ? p.delta[(size_t)h * p.n_q + rc] : 0.f;
        const __bf16* qp = p.q + ((size_t)rc * p.hq + h) * D + half * 8;
        const __bf16* dp = p.d_o + ((size_t)rc * p.hq + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
            bf16x8 g = *reinterpret_cast<const bf16x8*>(dp + ks * 16);
            if (!real) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { a[i] = (__bf16)0.f; g[i] = (__bf16)0.f; }
            }
            qf[b][ks] = a; dof[b][ks] = g;
        }
    }

    f32x16 acc[QB][DB];
#pragma unroll
    for (int b = 0; b < QB; ++b)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][db][r] = 0.f;

    const float cs = p.scale_log2e;
    const size_t kv_row = (size_t)p.hkv * D;
    const __bf16* kbase = p.k + (size_t)hk * D;
    const __bf16* vbase = p.v + (size_t)hk * D;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;

    for (int j = jb; j < je; ++j) {
        __syncthreads();
        for (int ch = tid; ch < BN * CPR; ch += NT) {
            const int r = ch / CPR, cc = ch % CPR;
            const int kr = min(j * BN + r, p.t_kv - 1);
            const i32x4 kk = *reinterpret_cast<const i32x4*>(kbase + (size_t)kr * kv_row + cc * 8);
            const i32x4 vv = *reinterpret_cast<const i32x4*>(vbase + (size_t)kr * kv_row + cc * 8);
            *reinterpret_cast<i32x4*>(&Ks[r * D + swz<CPR>(r, cc) * 8]) = kk;
            *reinterpret_cast<i32x4*>(&Vs[r * VSTR + cc * 8]) = vv;
        }
        __syncthreads();
        const bool partial = (j < fb) || (j >= fe);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 s[QB], dp[QB];
#pragma unroll
            for (int b = 0; b < QB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
            const int kr = kb * 32 + l32;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8*>(&Ks[kr * D + swz<CPR>(kr, ks * 2 + half) * 8]);
                const bf16x8 va = *reinterpret_cast<const bf16x8*>(&Vs[kr * VSTR + ks * 16 + half * 8]);
#pragma unroll
                for (int b = 0; b < QB; ++b) {
                    s[b] = mfma32(ka, qf[b][ks], s[b]);
                    dp[b] = mfma32(va, dof[b][ks], dp[b]);
                }
            }
            bf16x8 dsf[QB][2];
#pragma unroll
            for (int b = 0; b < QB; ++b) {
                float ds[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float pr = fast_exp2(fmaf(s[b][r], cs, -lsec[b]));
                    if (partial) {
                        const int key = j * BN + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                        pr = (key >= lo[b] && key < hi[b]) ? pr : 0.f;
                    }
                    ds[r] = pr * (dp[b][r] - dl[b]);
                }
                dsf[b][0] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
                dsf[b][1] = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
            }
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const int key0 = kb * 32 + cc * 16 + half * 4 + (j16 >> 2);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);       // logical 16-byte chunk
                    const int dsub = (j16 & 1) * 4;                            // element offset inside it
                    const bf16x4 k0v = lds_read_tr4(&Ks[key0 * D + swz<CPR>(key0, dch) * 8 + dsub]);
                    const bf16x4 k1v = lds_read_tr4(&Ks[(key0 + 8) * D + swz<CPR>(key0 + 8, dch) * 8 + dsub]);
                    const bf16x8 a = cat4(k0v, k1v);
#pragma unroll
                    for (int b = 0; b < QB; ++b) acc[b][db] = mfma32(a, dsf[b][cc], acc[b][db]);
                }
            }
        }
    }

#pragma unroll
    for (int b = 0; b < QB; ++b) {
        if (row[b] < p.n_q) {
            const bool real = hi[b] > 0;
            __bf16* op = p.dq + ((size_t)row[b] * p.hq + h) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d = db * 32 + r4 * 8 + half * 4;
                    bf16x4 out;
                    if (real) out = pack4(acc[b][db][r4 * 4 + 0] * p.scale, acc[b][db][r4 * 4 + 1] * p.scale,
                                          acc[b][db][r4 * 4 + 2] * p.scale, acc[b][db][r4 * 4 + 3] * p.scale);
                    else out = pack4(0.f, 0.f, 0.f, 0.f);
                    *reinterpret_cast<bf16x4*>(op + d) = out;
                }
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
__global__ void __launch_bounds__(256, 2) dq_pipe_kernel(const BwdParams p) {
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
    const int tile = p.fwd_order[rank];
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
    auto tile_ptr = [&](int which) { return reinterpret_cast<__bf16*>(smem + which * TILEB); };
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
    // padding rows: zero operands and LSE = +inf make P, dS and dQ exactly 0
    const float lsec = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;
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
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
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
        if (j + 1 < je && !(p.exp_flags & 8)) {
            dma.issue(krs, tile_ptr(cur ^ 1), (j + 1) * BN, wave);
            dma.issue(vrs, tile_ptr(2 + (cur ^ 1)), (j + 1) * BN, wave);
        }
        constexpr int kb_base = cur * TILEB, vb_base = (2 + cur) * TILEB;
        const bool partial = (j < fb) || (j >= fe);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(kb_base + naddr[ks] + kb * 32 * ROWB));
                const bf16x8 va = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(vb_base + naddr[ks] + kb * 32 * ROWB));
                s = mfma32(ka, qf[ks], s);
                dp = mfma32(va, dof[ks], dp);
            }
            float ds[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pr = fast_exp2(fmaf(s[r], cs, -lsec));
                ds[r] = pr * (dp[r] - dl);
            }
            if (partial) {
                asm volatile("");   // keep the mask a branch
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j * BN + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    ds[r] = (key >= lo && key < hi) ? ds[r] : 0.f;
                }
            }
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
        }
    };
    for (int j = jb; j < je; j += 2) {
        tile_step(j, std::integral_constant<int, 0>{});
        if (j + 1 < je) tile_step(j + 1, std::integral_constant<int, 1>{});
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

// ------------------------------------------------------------------------------------------
// dK/dV: one workgroup = 128 keys x one KV head; wavefront w owns keys [k0+32w, k0+32w+32).
// The row groups that can see the tile stream through LDS, one (group, query head) stage at a
// time: Q and dO rows by asynchronous global->LDS copies into the buffer not being computed
// on, LSE / delta / key intervals through registers one stage ahead.  One barrier per stage.
template <int D>
__global__ void __launch_bounds__(256) dkv_kernel(const BwdParams p) {
    constexpr int BNK = kBwdKeyTile, GR = kGroupRows, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int ROWB = D * 2, TILEB = GR * ROWB;
    static_assert(BNK == 128 && GR == 64, "tiling");

    __shared__ __attribute__((aligned(1024))) char smem[4 * TILEB];          // Q0 | Q1 | dO0 | dO1, swizzled
    __shared__ __attribute__((aligned(16))) float lse_s[2][GR];              // LSE * log2(e); +inf for padding rows
    __shared__ __attribute__((aligned(16))) float dl_s[2][GR];
    __shared__ __attribute__((aligned(16))) int lo_s[2][GR];
    __shared__ __attribute__((aligned(16))) int hi_s[2][GR];

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    const int y = blockIdx.x >> 3;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_key_tiles) return;
    const int kt = p.key_order[rank];
    const int k0 = kt * BNK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    const int kw0 = k0 + wave * 32;            // this wavefront's first key
    const int mykey = kw0 + l32;

    // K and V operands of this wavefront's 32 keys (B operands: column = key, 8 consecutive d)
    bf16x8 kf[KS], vf[KS];
    {
        const int kr = min(mykey, p.t_kv - 1);
        const __bf16* kp = p.k + ((size_t)kr * p.hkv + hk) * D + half * 8;
        const __bf16* vp = p.v + ((size_t)kr * p.hkv + hk) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
            vf[ks] = *reinterpret_cast<const bf16x8*>(vp + ks * 16);
        }
    }
    f32x16 dk_acc[DB], dv_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }

    const float cs = p.scale_log2e;
    const int g_end = p.key_range[2 * kt + 1];
    const int k1 = min(k0 + BNK, p.t_kv);

    // first group at or after g whose hull touches this key tile (g_end if none)
    auto next_group = [&](int g) {
        for (; g < g_end; ++g) {
            const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
            if (gd.y > gd.x && gd.x < k1 && gd.y > k0) break;
        }
        return g;
    };

    const uint32_t q_row = (uint32_t)p.hq * D;
    const uint32_t q_total = (uint32_t)p.n_q * q_row * 2u;
    TileDma<D, GR, 4> dma;
    dma.init(wave, lane, q_row);
    auto tile_ptr = [&](int which) { return reinterpret_cast<__bf16*>(smem + which * TILEB); };
    auto issue_stage = [&](int g, int h, int buf) {
        BufRsrc qrs, ors;
        qrs.init(p.q + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        ors.init(p.d_o + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        dma.issue(qrs, tile_ptr(buf), g * GR, wave);
        dma.issue(ors, tile_ptr(2 + buf), g * GR, wave);
    };
    // per-row scalars of a stage, fetched by the first 64 threads one stage ahead
    float r_lse = INFINITY, r_dl = 0.f;
    int r_lo = kPadLo, r_hi = 0;
    auto load_small = [&](int g, int h) {
        if (tid < GR) {
            const int rowi = g * GR + tid;
            const bool inr = rowi < p.n_q;
            const int rc = inr ? rowi : p.n_q - 1;
            r_hi = inr ? p.row_hi[rc] : 0;
            const bool real = r_hi > 0;
            r_lo = real ? p.row_lo[rc] : kPadLo;
            r_lse = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;
            r_dl = real ? p.delta[(size_t)h * p.n_q + rc] : 0.f;
        }
    };

    // LDS offsets (bytes inside a tile) of the two access patterns
    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int qq = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = qq * ROWB + swz<CPR>(qq, dch) * 16 + (j16 & 1) * 8;
        }
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;

    int g = next_group(p.key_range[2 * kt]);
    int hh = 0, buf = 0;
    if (g < g_end) {
        issue_stage(g, hk * G, 0);
        load_small(g, hk * G);
    }
    while (g < g_end) {
        // next stage
        int gn = g, hn = hh + 1;
        if (hn == G) { hn = 0; gn = next_group(g + 1); }
        const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
        const bool full = (gd.z <= k0) && (k0 + BNK <= gd.w);              // every real row sees every key
        const bool wave_live = (gd.x < kw0 + 32) && (gd.y > kw0);
        const bool has_pads = p.group_real[g] < min(GR, p.n_q - g * GR);

        if (tid < GR) { lse_s[buf][tid] = r_lse; dl_s[buf][tid] = r_dl; lo_s[buf][tid] = r_lo; hi_s[buf][tid] = r_hi; }
        wait_vmem();
        __syncthreads();      // stage (g, hh) is in LDS; everyone has left the other buffer
        if (gn < g_end) {
            issue_stage(gn, hk * G + hn, buf ^ 1);
            load_small(gn, hk * G + hn);
        }
        if (has_pads) {
            // padding rows may hold anything: clear them so they cannot poison the MFMAs
            const int r = tid >> 2, part = tid & 3;
            if (hi_s[buf][r] == 0) {
                const i32x4 z = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < CPR / 4; ++i) {
                    *reinterpret_cast<i32x4*>(smem + buf * TILEB + r * ROWB + (part * (CPR / 4) + i) * 16) = z;
                    *reinterpret_cast<i32x4*>(smem + (2 + buf) * TILEB + r * ROWB + (part * (CPR / 4) + i) * 16) = z;
                }
            }
            __syncthreads();
        }
        if (wave_live) {
            const uint32_t qb_base = smem_base + buf * TILEB, ob_base = smem_base + (2 + buf) * TILEB;
#pragma unroll 1
            for (int qb = 0; qb < GR / 32; ++qb) {
                // S[q][k] = Q K^T, dP[q][k] = dO V^T : lane = key column, register = query row
                f32x16 s, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 qa = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(qb_base + naddr[ks] + qb * 32 * ROWB));
                    const bf16x8 ga = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(ob_base + naddr[ks] + qb * 32 * ROWB));
                    s = mfma32(qa, kf[ks], s);
                    dp = mfma32(ga, vf[ks], dp);
                }
                float pr[16], ds[16];
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int qrow = qb * 32 + r4 * 8 + half * 4;
                    const f32x4 ls = *reinterpret_cast<const f32x4*>(&lse_s[buf][qrow]);
                    const f32x4 dl = *reinterpret_cast<const f32x4*>(&dl_s[buf][qrow]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) pr[r4 * 4 + i] = fast_exp2(fmaf(s[r4 * 4 + i], cs, -ls[i]));
                    if (!full) {
                        asm volatile("");   // keep the mask a branch
                        const i32x4 l4 = *reinterpret_cast<const i32x4*>(&lo_s[buf][qrow]);
                        const i32x4 h4 = *reinterpret_cast<const i32x4*>(&hi_s[buf][qrow]);
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            pr[r4 * 4 + i] = (mykey >= l4[i] && mykey < h4[i]) ? pr[r4 * 4 + i] : 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) ds[r4 * 4 + i] = pr[r4 * 4 + i] * (dp[r4 * 4 + i] - dl[i]);
                }
                bf16x8 pf[2], dsf[2];
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    pf[cc] = pack8(pr[8 * cc + 0], pr[8 * cc + 1], pr[8 * cc + 2], pr[8 * cc + 3], pr[8 * cc + 4],
                                   pr[8 * cc + 5], pr[8 * cc + 6], pr[8 * cc + 7]);
                    dsf[cc] = pack8(ds[8 * cc + 0], ds[8 * cc + 1], ds[8 * cc + 2], ds[8 * cc + 3], ds[8 * cc + 4],
                                    ds[8 * cc + 5], ds[8 * cc + 6], ds[8 * cc + 7]);
                }
                // dV^T[d][k] += dO^T[d][q] P[q][k];  dK^T[d][k] += Q^T[d][q] dS[q][k]
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const int qoff = (qb * 32 + cc * 16) * ROWB;
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const bf16x8 ga = cat4(lds_read_tr4_at(ob_base + taddr[db][0] + qoff),
                                               lds_read_tr4_at(ob_base + taddr[db][1] + qoff));
                        const bf16x8 qa = cat4(lds_read_tr4_at(qb_base + taddr[db][0] + qoff),
                                               lds_read_tr4_at(qb_base + taddr[db][1] + qoff));
                        dv_acc[db] = mfma32(ga, pf[cc], dv_acc[db]);
                        dk_acc[db] = mfma32(qa, dsf[cc], dk_acc[db]);
                    }
                }
            }
        }
        g = gn; hh = hn; buf ^= 1;
    }

    if (mykey < p.t_kv) {
        __bf16* kp = p.dk + ((size_t)mykey * p.hkv + hk) * D;
        __bf16* vp = p.dv + ((size_t)mykey * p.hkv + hk) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = db * 32 + r4 * 8 + half * 4;
                *reinterpret_cast<bf16x4*>(kp + d) =
                    pack4(dk_acc[db][r4 * 4 + 0] * p.scale, dk_acc[db][r4 * 4 + 1] * p.scale,
                          dk_acc[db][r4 * 4 + 2] * p.scale, dk_acc[db][r4 * 4 + 3] * p.scale);
                *reinterpret_cast<bf16x4*>(vp + d) = pack4(dv_acc[db][r4 * 4 + 0], dv_acc[db][r4 * 4 + 1],
                                                           dv_acc[db][r4 * 4 + 2], dv_acc[db][r4 * 4 + 3]);
            }
    }
}

// ------------------------------------------------------------------------------------------
// dK/dV with role-split wavefronts: one workgroup = 128 keys x one KV head, eight wavefronts.
// Wavefronts 0-3 ("score" role) hold the K operands of 32 keys each: they compute
// S = Q K^T, P = exp(scale*S - LSE) (masked), hand P (bf16) to their partner through LDS and
// accumulate dV^T += dO^T P.  Wavefronts 4-7 ("gradient" role) hold the V operands of the same
// keys: they compute dP = dO V^T, take P from the partner, form dS = P o (dP - delta) and
// accumulate dK^T += Q^T dS.  Partners sit on the same SIMD, so each SIMD always has an MFMA
// stream and a vector-ALU stream to overlap; every wavefront needs about half the registers
// of an unsplit one, which is what allows two per SIMD.
// Stages (row group, query head) stream through LDS exactly as in dkv_kernel; per stage:
//   barrier 1 (tiles landed) -> phase 1 (S,P | dP) -> barrier 2 (P visible) -> phase 2 (dV | dS,dK).
template <int D>
__global__ void __launch_bounds__(512) dkv_split_kernel(const BwdParams p) {
    constexpr int BNK = kBwdKeyTile, GR = kGroupRows, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int ROWB = D * 2, TILEB = GR * ROWB, NW = 8;
    static_assert(BNK == 128 && GR == 64, "tiling");

    __shared__ __attribute__((aligned(1024))) char smem[4 * TILEB];          // Q0 | Q1 | dO0 | dO1, swizzled
    __shared__ __attribute__((aligned(1024))) char pbuf[4 * 2 * 2 * 1024];   // P: [key block][row block][half of 16 rows][lane] x 16 B
    __shared__ __attribute__((aligned(16))) float lse_s[2][GR];
    __shared__ __attribute__((aligned(16))) float dl_s[2][GR];
    __shared__ __attribute__((aligned(16))) int lo_s[2][GR];
    __shared__ __attribute__((aligned(16))) int hi_s[2][GR];

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    const int y = blockIdx.x >> 3;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_key_tiles) return;
    const int kt = p.key_order[rank];
    const int k0 = kt * BNK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int role = wave >> 2, kblk = wave & 3;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    const int kw0 = k0 + kblk * 32;
    const int mykey = kw0 + l32;

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

    const float cs = p.scale_log2e;
    const int g_end = p.key_range[2 * kt + 1];
    const int k1 = min(k0 + BNK, p.t_kv);
    auto next_group = [&](int g) {
        for (; g < g_end; ++g) {
            const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
            if (gd.y > gd.x && gd.x < k1 && gd.y > k0) break;
        }
        return g;
    };

    const uint32_t q_row = (uint32_t)p.hq * D;
    const uint32_t q_total = (uint32_t)p.n_q * q_row * 2u;
    TileDma<D, GR, NW> dma;
    dma.init(wave, lane, q_row);
    auto tile_ptr = [&](int which) { return reinterpret_cast<__bf16*>(smem + which * TILEB); };
    auto issue_stage = [&](int g, int h, int buf) {
        BufRsrc qrs, ors;
        qrs.init(p.q + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        ors.init(p.d_o + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        dma.issue(qrs, tile_ptr(buf), g * GR, wave);
        dma.issue(ors, tile_ptr(2 + buf), g * GR, wave);
    };
    float r_lse = INFINITY, r_dl = 0.f;
    int r_lo = kPadLo, r_hi = 0;
    auto load_small = [&](int g, int h) {
        if (tid < GR) {
            const int rowi = g * GR + tid;
            const bool inr = rowi < p.n_q;
            const int rc = inr ? rowi : p.n_q - 1;
            r_hi = inr ? p.row_hi[rc] : 0;
            const bool real = r_hi > 0;
            r_lo = real ? p.row_lo[rc] : kPadLo;
            r_lse = real ? p.lse[(size_t)h * p.n_q + rc] * 1.4426950408889634f : INFINITY;
            r_dl = real ? p.delta[(size_t)h * p.n_q + rc] : 0.f;
        }
    };

    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int qq = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = qq * ROWB + swz<CPR>(qq, dch) * 16 + (j16 & 1) * 8;
        }
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t pbuf_lane = (uint32_t)(uintptr_t)(WLB_LDS char*)pbuf + kblk * 4096 + lane * 16;

    int g = next_group(p.key_range[2 * kt]);
    int hh = 0, buf = 0;
    if (g < g_end) {
        issue_stage(g, hk * G, 0);
        load_small(g, hk * G);
    }
    while (g < g_end) {
        int gn = g, hn = hh + 1;
        if (hn == G) { hn = 0; gn = next_group(g + 1); }
        const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
        const bool full = (gd.z <= k0) && (k0 + BNK <= gd.w);
        const bool wave_live = (gd.x < kw0 + 32) && (gd.y > kw0);
        const bool has_pads = p.group_real[g] < min(GR, p.n_q - g * GR);

        if (tid < GR) { lse_s[buf][tid] = r_lse; dl_s[buf][tid] = r_dl; lo_s[buf][tid] = r_lo; hi_s[buf][tid] = r_hi; }
        if (!(p.exp_flags & 2)) wait_vmem();
        __syncthreads();      // barrier 1: stage (g, hh) is in LDS; everyone has left the other buffers and pbuf
        if (gn < g_end && !(p.exp_flags & 4)) {
            issue_stage(gn, hk * G + hn, buf ^ 1);
            load_small(gn, hk * G + hn);
        }
        if (has_pads) {
            const int r = tid >> 3, part = tid & 7;       // 512 threads: 8 per row
            if (hi_s[buf][r] == 0) {
                const i32x4 z = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < CPR / 8; ++i) {
                    *reinterpret_cast<i32x4*>(smem + buf * TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                    *reinterpret_cast<i32x4*>(smem + (2 + buf) * TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                }
            }
            __syncthreads();
        }
        const uint32_t qb_base = smem_base + buf * TILEB, ob_base = smem_base + (2 + buf) * TILEB;

        // ---------------- phase 1
        bf16x8 pf[2][2];          // score role: P as MFMA B operands, [row block][16-row half]
        f32x16 dp[2];             // gradient role: dP
        if (wave_live) {
            if (role == 0) {
                // all 16 Q operands are requested before the first MFMA, the two row blocks'
                // accumulation chains are interleaved
                bf16x8 qa[2][KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        qa[qb][ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(qb_base + naddr[ks] + qb * 32 * ROWB));
                f32x16 s2[2];
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s2[qb][r] = 0.f;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb) s2[qb] = mfma32(qa[qb][ks], bop[ks], s2[qb]);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    const f32x16 s = s2[qb];
                    float pr[16];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int qrow = qb * 32 + r4 * 8 + half * 4;
                        const f32x4 ls = *reinterpret_cast<const f32x4*>(&lse_s[buf][qrow]);
#pragma unroll
                        for (int i = 0; i < 4; ++i) pr[r4 * 4 + i] = fast_exp2(fmaf(s[r4 * 4 + i], cs, -ls[i]));
                        if (!full) {
                            asm volatile("");   // keep the mask a branch
                            const i32x4 l4 = *reinterpret_cast<const i32x4*>(&lo_s[buf][qrow]);
                            const i32x4 h4 = *reinterpret_cast<const i32x4*>(&hi_s[buf][qrow]);
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pr[r4 * 4 + i] = (mykey >= l4[i] && mykey < h4[i]) ? pr[r4 * 4 + i] : 0.f;
                        }
                    }
#pragma unroll
                    for (int cc = 0; cc < 2; ++cc) {
                        pf[qb][cc] = pack8(pr[8 * cc + 0], pr[8 * cc + 1], pr[8 * cc + 2], pr[8 * cc + 3],
                                           pr[8 * cc + 4], pr[8 * cc + 5], pr[8 * cc + 6], pr[8 * cc + 7]);
                        *reinterpret_cast<WLB_LDS bf16x8*>((uintptr_t)(pbuf_lane + (qb * 2 + cc) * 1024)) = pf[qb][cc];
                    }
                }
            } else {
                bf16x8 ga[2][KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        ga[qb][ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(ob_base + naddr[ks] + qb * 32 * ROWB));
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dp[qb][r] = 0.f;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb) dp[qb] = mfma32(ga[qb][ks], bop[ks], dp[qb]);
            }
        }
        if (!(p.exp_flags & 1)) __syncthreads();      // barrier 2: P of this stage is visible to the partners

        // ---------------- phase 2
        if (wave_live) {
            if (role == 0) {
                // four steps of 16 rows; the transposed dO operands of step i+1 are requested
                // before the MFMAs of step i are issued
                bf16x4 tv[2][DB][2];
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int t = 0; t < 2; ++t) tv[0][db][t] = lds_read_tr4_at(ob_base + taddr[db][t]);
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    if (st + 1 < 4) {
#pragma unroll
                        for (int db = 0; db < DB; ++db)
#pragma unroll
                            for (int t = 0; t < 2; ++t)
                                tv[(st + 1) & 1][db][t] = lds_read_tr4_at(ob_base + taddr[db][t] + (st + 1) * 16 * ROWB);
                    }
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        acc[db] = mfma32(cat4(tv[st & 1][db][0], tv[st & 1][db][1]), pf[st >> 1][st & 1], acc[db]);
                }
            } else {
                bf16x4 tv[2][DB][2];
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int t = 0; t < 2; ++t) tv[0][db][t] = lds_read_tr4_at(qb_base + taddr[db][t]);
                bf16x8 dsf[4];
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const int qb = st >> 1, cc = st & 1;
                    const bf16x8 pv = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(pbuf_lane + st * 1024));
                    float ds[8];
#pragma unroll
                    for (int r2 = 0; r2 < 2; ++r2) {
                        const int qrow = qb * 32 + (cc * 2 + r2) * 8 + half * 4;
                        const f32x4 dl = *reinterpret_cast<const f32x4*>(&dl_s[buf][qrow]);
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            ds[r2 * 4 + i] = (float)pv[r2 * 4 + i] * (dp[qb][cc * 8 + r2 * 4 + i] - dl[i]);
                    }
                    dsf[st] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
                }
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    if (st + 1 < 4) {
#pragma unroll
                        for (int db = 0; db < DB; ++db)
#pragma unroll
                            for (int t = 0; t < 2; ++t)
                                tv[(st + 1) & 1][db][t] = lds_read_tr4_at(qb_base + taddr[db][t] + (st + 1) * 16 * ROWB);
                    }
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        acc[db] = mfma32(cat4(tv[st & 1][db][0], tv[st & 1][db][1]), dsf[st], acc[db]);
                }
            }
        }
        g = gn; hh = hn; buf ^= 1;
    }

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
}

// ------------------------------------------------------------------------------------------
// dK/dV, software-pipelined.  One workgroup = 128 keys x one KV head, four wavefronts of 32
// keys (their K and V MFMA operands live in registers), one wavefront per SIMD.  Measured on
// gfx950, MFMA and vector-ALU work overlap only inside one wavefront, so the loop is arranged
// as a pipeline over blocks of 32 query rows: while the vector ALU turns the scores of block i
// into P and dS, the MFMA pipe accumulates dV^T, dK^T of block i-1.  Stages (64 rows of one
// query head: Q, dO, LSE, delta, key intervals) arrive in a ring of four LDS buffers by
// asynchronous copies issued two stages ahead; one barrier per stage.
template <int D>
__global__ void __launch_bounds__(256) dkv_ring_kernel(const BwdParams p) {
    constexpr int BNK = kBwdKeyTile, GR = kGroupRows, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int ROWB = D * 2, TILEB = GR * ROWB, NBUF = 4, NW = 4;
    constexpr int SMALLB = 4 * GR * 4;                       // lse2 | delta | lo | hi, 64 dwords each
    static_assert(BNK == 128 && GR == 64, "tiling");
    using Dma = TileDma<D, GR, NW>;
    constexpr int BATCH = 2 * Dma::PER + 1;                  // vector-memory operations per wavefront and stage

    __shared__ __attribute__((aligned(1024))) char smem[NBUF * 2 * TILEB];   // per slot: Q tile | dO tile, swizzled
    __shared__ __attribute__((aligned(1024))) char small[NBUF * SMALLB];

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    const int y = blockIdx.x >> 3;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    if (rank >= p.n_key_tiles) return;
    const int kt = p.key_order[rank];
    const int k0 = kt * BNK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    const int kw0 = k0 + wave * 32;
    const int mykey = kw0 + l32;

    bf16x8 kf[KS], vf[KS];
    {
        const int kr = min(mykey, p.t_kv - 1);
        const __bf16* kp = p.k + ((size_t)kr * p.hkv + hk) * D + half * 8;
        const __bf16* vp = p.v + ((size_t)kr * p.hkv + hk) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
            vf[ks] = *reinterpret_cast<const bf16x8*>(vp + ks * 16);
        }
    }
    f32x16 dk_acc[DB], dv_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }

    const float cs = p.scale_log2e;
    const int g_end = p.key_range[2 * kt + 1];
    const int k1 = min(k0 + BNK, p.t_kv);
    auto next_group = [&](int g) {
        for (; g < g_end; ++g) {
            const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
            if (gd.y > gd.x && gd.x < k1 && gd.y > k0) break;
        }
        return g;
    };
    // successor of stage (g, hh); g == g_end marks the end
    auto succ = [&](int& g, int& hh) {
        if (++hh == G) { hh = 0; g = next_group(g + 1); }
    };

    const uint32_t q_row = (uint32_t)p.hq * D;
    const uint32_t q_total = (uint32_t)p.n_q * q_row * 2u;
    Dma dma;
    dma.init(wave, lane, q_row);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t small_base = (uint32_t)(uintptr_t)(WLB_LDS char*)small;
    // every wavefront issues the same number of copies per stage: its share of the Q and dO
    // tiles plus one of the four 64-entry scalar arrays
    auto issue_stage = [&](int g, int h, int slot) {
        BufRsrc qrs, ors, srs;
        qrs.init(p.q + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        ors.init(p.d_o + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        dma.issue(qrs, reinterpret_cast<__bf16*>(smem + slot * 2 * TILEB), g * GR, wave);
        dma.issue(ors, reinterpret_cast<__bf16*>(smem + slot * 2 * TILEB + TILEB), g * GR, wave);
        const void* base = wave == 0 ? (const void*)(p.lse2 + (size_t)h * p.n_q)
                         : wave == 1 ? (const void*)(p.delta + (size_t)h * p.n_q)
                         : wave == 2 ? (const void*)p.row_lo : (const void*)p.row_hi;
        srs.init(base, (uint32_t)p.n_q * 4u);
        srs.make_uniform();
        dma_issue_256(srs.r, __builtin_amdgcn_readfirstlane(small_base + slot * SMALLB + wave * GR * 4), lane * 4,
                      __builtin_amdgcn_readfirstlane((uint32_t)(g * GR) * 4u));
    };

    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int qq = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = qq * ROWB + swz<CPR>(qq, dch) * 16 + (j16 & 1) * 8;
        }

    // P and dS of the previous block (MFMA B operands) and where its rows sit in LDS
    bf16x8 pf_old[2], dsf_old[2];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int i = 0; i < 8; ++i) { pf_old[cc][i] = (__bf16)0.f; dsf_old[cc][i] = (__bf16)0.f; }
    uint32_t back_q = smem_base, back_o = smem_base + TILEB;      // first unit: zero operands against stage 0's tile

    // dV^T, dK^T += (dO^T, Q^T of the previous block) x (P, dS of the previous block), 16-row step cc
    auto back_step = [&](int cc) {
        bf16x8 ga[DB], qa[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            ga[db] = cat4(lds_read_tr4_at(back_o + taddr[db][0] + cc * 16 * ROWB),
                          lds_read_tr4_at(back_o + taddr[db][1] + cc * 16 * ROWB));
            qa[db] = cat4(lds_read_tr4_at(back_q + taddr[db][0] + cc * 16 * ROWB),
                          lds_read_tr4_at(back_q + taddr[db][1] + cc * 16 * ROWB));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            dv_acc[db] = mfma32(ga[db], pf_old[cc], dv_acc[db]);
            dk_acc[db] = mfma32(qa[db], dsf_old[cc], dk_acc[db]);
        }
    };

    // one pipeline unit: scores and dP of block (slot, qb), then its P/dS on the vector ALU
    // against the previous block's dV/dK MFMAs
    auto unit = [&](int slot, int qb, bool live, auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const uint32_t fq = smem_base + slot * 2 * TILEB + qb * 32 * ROWB, fo = fq + TILEB;
        const uint32_t sm = small_base + slot * SMALLB + (qb * 32 + half * 4) * 4;
        bf16x8 pf_new[2], dsf_new[2];
        if (live) {
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
            bf16x8 qa[KS], ga[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                qa[ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(fq + naddr[ks]));
                ga[ks] = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(fo + naddr[ks]));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = mfma32(qa[ks], kf[ks], s);
                dp = mfma32(ga[ks], vf[ks], dp);
            }
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                float pr[8], ds[8];
#pragma unroll
                for (int r2 = 0; r2 < 2; ++r2) {
                    const int r4 = cc * 2 + r2;
                    const f32x4 ls = *reinterpret_cast<const WLB_LDS f32x4*>((uintptr_t)(sm + r4 * 32));
                    const f32x4 dl = *reinterpret_cast<const WLB_LDS f32x4*>((uintptr_t)(sm + GR * 4 + r4 * 32));
#pragma unroll
                    for (int i = 0; i < 4; ++i) pr[r2 * 4 + i] = fast_exp2(fmaf(s[r4 * 4 + i], cs, -ls[i]));
                    if (MASK) {
                        const i32x4 l4 = *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)(sm + 2 * GR * 4 + r4 * 32));
                        const i32x4 h4 = *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)(sm + 3 * GR * 4 + r4 * 32));
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            pr[r2 * 4 + i] = (mykey >= l4[i] && mykey < h4[i]) ? pr[r2 * 4 + i] : 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) ds[r2 * 4 + i] = pr[r2 * 4 + i] * (dp[r4 * 4 + i] - dl[i]);
                }
                pf_new[cc] = pack8(pr[0], pr[1], pr[2], pr[3], pr[4], pr[5], pr[6], pr[7]);
                dsf_new[cc] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
                back_step(cc);
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { pf_new[cc][i] = (__bf16)0.f; dsf_new[cc][i] = (__bf16)0.f; }
                back_step(cc);
            }
        }
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) { pf_old[cc] = pf_new[cc]; dsf_old[cc] = dsf_new[cc]; }
        back_q = fq; back_o = fo;
    };

    // ---- stage ring: s (computing), s+1 (landed or landing), s+2 (issued at the top of s)
    int g0 = next_group(p.key_range[2 * kt]), h0 = 0;           // stage s
    int g1 = g0, h1 = h0;                                       // stage s+1
    if (g0 < g_end) {
        issue_stage(g0, hk * G + h0, 0);
        succ(g1, h1);
        if (g1 < g_end) issue_stage(g1, hk * G + h1, 1);
    }
    int g2 = g1, h2 = h1;                                       // stage s+2
    int slot = 0;
    while (g0 < g_end) {
        if (g1 < g_end) succ(g2, h2); else g2 = g_end;
        const int4 gd = reinterpret_cast<const int4*>(p.group)[g0];
        const bool full = (gd.z <= k0) && (k0 + BNK <= gd.w);
        const bool live = (gd.x < kw0 + 32) && (gd.y > kw0);
        const bool has_pads = p.group_real[g0] < min(GR, p.n_q - g0 * GR);

        // stage s has landed once at most the copies of stage s+1 are outstanding
        if (g1 < g_end) wait_vmem_le<BATCH>(); else wait_vmem();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the previous block's LDS reads have returned
        __syncthreads();
        if (g2 < g_end) issue_stage(g2, hk * G + h2, (slot + 2) % NBUF);
        if (has_pads) {
            // padding rows may hold anything: clear them so they cannot poison the MFMAs
            const int r = tid >> 2, part = tid & 3;
            const int hi_r = *reinterpret_cast<const int*>(small + slot * SMALLB + 3 * GR * 4 + r * 4);
            if (hi_r == 0 && g0 * GR + r < p.n_q) {
                const i32x4 z = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < CPR / 4; ++i) {
                    *reinterpret_cast<i32x4*>(smem + slot * 2 * TILEB + r * ROWB + (part * (CPR / 4) + i) * 16) = z;
                    *reinterpret_cast<i32x4*>(smem + slot * 2 * TILEB + TILEB + r * ROWB + (part * (CPR / 4) + i) * 16) = z;
                }
            }
            __syncthreads();
        }
        if (full) {
            unit(slot, 0, live, std::false_type{});
            unit(slot, 1, live, std::false_type{});
        } else {
            unit(slot, 0, live, std::true_type{});
            unit(slot, 1, live, std::true_type{});
        }
        g0 = g1; h0 = h1; g1 = g2; h1 = h2;
        slot = (slot + 1) % NBUF;
    }
    // drain: the last block's dV/dK
    back_step(0);
    back_step(1);

    if (mykey < p.t_kv) {
        __bf16* kp = p.dk + ((size_t)mykey * p.hkv + hk) * D;
        __bf16* vp = p.dv + ((size_t)mykey * p.hkv + hk) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = db * 32 + r4 * 8 + half * 4;
                *reinterpret_cast<bf16x4*>(kp + d) =
                    pack4(dk_acc[db][r4 * 4 + 0] * p.scale, dk_acc[db][r4 * 4 + 1] * p.scale,
                          dk_acc[db][r4 * 4 + 2] * p.scale, dk_acc[db][r4 * 4 + 3] * p.scale);
                *reinterpret_cast<bf16x4*>(vp + d) = pack4(dv_acc[db][r4 * 4 + 0], dv_acc[db][r4 * 4 + 1],
                                                           dv_acc[db][r4 * 4 + 2], dv_acc[db][r4 * 4 + 3]);
            }
    }
}

// ------------------------------------------------------------------------------------------
// dK/dV with two kinds of wavefront.  One workgroup = 128 keys x one KV head, eight
// wavefronts, two per SIMD.  Wavefronts 0-3 own dV^T of 32 keys each: S = Q K^T, P, then
// dV^T += dO^T P.  Wavefronts 4-7 own dK^T of the same keys: S and dP = dO V^T, dS, then
// dK^T += Q^T dS.  S is computed by both kinds (10*D instead of 8*D MFMA flops per pair); in
// return neither needs more than half the accumulator registers of a combined wavefront, two
// fit on a SIMD, nothing is exchanged between them and one barrier per stage suffices.
// Measured on gfx950, MFMA and vector-ALU work overlap only inside one wavefront, so each
// wavefront runs a pipeline over blocks of 32 query rows: while its vector ALU turns the
// scores of block i into P (dS), its MFMAs accumulate block i-1.  Stages (64 rows of one query
// head: Q, dO, LSE, delta, key intervals) arrive in a ring of four LDS buffers by asynchronous
// copies issued two stages ahead.
template <int D, int ROLE>
__device__ __forceinline__ void dkv_duo_body(const BwdParams& p, char* smem, char* small) {
    constexpr int BNK = kBwdKeyTile, GR = kGroupRows, KS = D / 16, DB = D / 32, CPR = D / 8;
    constexpr int ROWB = D * 2, TILEB = GR * ROWB, NBUF = 4, NW = 8;
    constexpr int SMALLB = 4 * GR * 4;                       // lse2 | delta | lo | hi, 64 dwords each
    static_assert(BNK == 128 && GR == 64, "tiling");
    using Dma = TileDma<D, GR, NW>;
    constexpr int BATCH = 2 * Dma::PER;                      // tile copies per wavefront and stage (+1 scalar array on wavefronts 0-3)

    const int G = p.hq / p.hkv;
    const int x = blockIdx.x & 7;
    const int y = blockIdx.x >> 3;
    const int hk = y % p.hkv;
    const int c = y / p.hkv;
    const int rank = c * 8 + x;
    const int kt = p.key_order[rank];
    const int k0 = kt * BNK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int j16 = lane & 15, gi = (lane >> 4) & 1;
    constexpr int role = ROLE;                       // role 0: dV, role 1: dK
    const int kblk = wave & 3;
    const int kw0 = k0 + kblk * 32;
    const int mykey = kw0 + l32;

    bf16x8 kf[KS], vf[KS];
    {
        const int kr = min(mykey, p.t_kv - 1);
        const __bf16* kp = p.k + ((size_t)kr * p.hkv + hk) * D + half * 8;
        const __bf16* vp = p.v + ((size_t)kr * p.hkv + hk) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
            if (role == 1) vf[ks] = *reinterpret_cast<const bf16x8*>(vp + ks * 16);
        }
    }
    f32x16 acc[DB];      // dV^T (role 0) or dK^T (role 1)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    const float cs = p.scale_log2e;
    const int g_end = p.key_range[2 * kt + 1];
    const int k1 = min(k0 + BNK, p.t_kv);
    auto next_group = [&](int g) {
        for (; g < g_end; ++g) {
            const int4 gd = reinterpret_cast<const int4*>(p.group)[g];
            if (gd.y > gd.x && gd.x < k1 && gd.y > k0) break;
        }
        return g;
    };
    // successor of stage (g, hh); g == g_end marks the end
    auto succ = [&](int& g, int& hh) {
        if (++hh == G) { hh = 0; g = next_group(g + 1); }
    };

    const uint32_t q_row = (uint32_t)p.hq * D;
    const uint32_t q_total = (uint32_t)p.n_q * q_row * 2u;
    Dma dma;
    dma.init(wave, lane, q_row);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(WLB_LDS char*)smem;
    const uint32_t small_base = (uint32_t)(uintptr_t)(WLB_LDS char*)small;
    // every wavefront issues the same number of copies per stage: its share of the Q and dO
    // tiles plus one of the four 64-entry scalar arrays
    auto issue_stage = [&](int g, int h, int slot) {
        BufRsrc qrs, ors, srs;
        qrs.init(p.q + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        ors.init(p.d_o + (size_t)h * D, q_total - (uint32_t)h * ROWB);
        dma.issue(qrs, reinterpret_cast<__bf16*>(smem + slot * 2 * TILEB), g * GR, wave);
        dma.issue(ors, reinterpret_cast<__bf16*>(smem + slot * 2 * TILEB + TILEB), g * GR, wave);
        if (wave < 4) {
            const void* base = wave == 0 ? (const void*)(p.lse2 + (size_t)h * p.n_q)
                             : wave == 1 ? (const void*)(p.delta + (size_t)h * p.n_q)
                             : wave == 2 ? (const void*)p.row_lo : (const void*)p.row_hi;
            srs.init(base, (uint32_t)p.n_q * 4u);
            srs.make_uniform();
            dma_issue_256(srs.r, __builtin_amdgcn_readfirstlane(small_base + slot * SMALLB + wave * GR * 4), lane * 4,
                          __builtin_amdgcn_readfirstlane((uint32_t)(g * GR) * 4u));
        }
    };

    int naddr[KS], taddr[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) naddr[ks] = l32 * ROWB + swz<CPR>(l32, ks * 2 + half) * 16;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int qq = t * 8 + half * 4 + (j16 >> 2);
            const int dch = db * 4 + gi * 2 + ((j16 & 3) >> 1);
            taddr[db][t] = qq * ROWB + swz<CPR>(qq, dch) * 16 + (j16 & 1) * 8;
        }

    // P and dS of the previous block (MFMA B operands) and where its rows sit in LDS
    bf16x8 b_old[2];      // P (role 0) or dS (role 1) of the previous block
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int i = 0; i < 8; ++i) b_old[cc][i] = (__bf16)0.f;
    // rows of the previous block in LDS: dO tile for dV, Q tile for dK (first unit: zero operands, stage 0's tile)
    uint32_t back_t = smem_base + (role == 0 ? TILEB : 0);

    // acc += (dO^T or Q^T of the previous block) x (P or dS of the previous block), 16-row step cc
    auto back_step = [&](int cc) {
        bf16x8 ta[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
            ta[db] = cat4(lds_read_tr4_at(back_t + taddr[db][0] + cc * 16 * ROWB),
                          lds_read_tr4_at(back_t + taddr[db][1] + cc * 16 * ROWB));
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma32(ta[db], b_old[cc], acc[db]);
    };

    // one pipeline unit: scores (and dP) of block (slot, qb), then its P (dS) on the vector ALU
    // against the previous block's accumulation MFMAs
    auto unit = [&](int slot, int qb, bool live, auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const uint32_t fq = smem_base + slot * 2 * TILEB + qb * 32 * ROWB, fo = fq + TILEB;
        const uint32_t sm = small_base + slot * SMALLB + (qb * 32 + half * 4) * 4;
        bf16x8 b_new[2];
        if (live) {
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
            if (role == 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 qa = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(fq + naddr[ks]));
                    s = mfma32(qa, kf[ks], s);
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 qa = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(fq + naddr[ks]));
                    const bf16x8 ga = *reinterpret_cast<const WLB_LDS bf16x8*>((uintptr_t)(fo + naddr[ks]));
                    s = mfma32(qa, kf[ks], s);
                    dp = mfma32(ga, vf[ks], dp);
                }
            }
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                float pr[8];
#pragma unroll
                for (int r2 = 0; r2 < 2; ++r2) {
                    const int r4 = cc * 2 + r2;
                    const f32x4 ls = *reinterpret_cast<const WLB_LDS f32x4*>((uintptr_t)(sm + r4 * 32));
#pragma unroll
                    for (int i = 0; i < 4; ++i) pr[r2 * 4 + i] = fast_exp2(fmaf(s[r4 * 4 + i], cs, -ls[i]));
                    if (MASK) {
                        const i32x4 l4 = *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)(sm + 2 * GR * 4 + r4 * 32));
                        const i32x4 h4 = *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)(sm + 3 * GR * 4 + r4 * 32));
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            pr[r2 * 4 + i] = (mykey >= l4[i] && mykey < h4[i]) ? pr[r2 * 4 + i] : 0.f;
                    }
                    if (role == 1) {
                        const f32x4 dl = *reinterpret_cast<const WLB_LDS f32x4*>((uintptr_t)(sm + GR * 4 + r4 * 32));
#pragma unroll
                        for (int i = 0; i < 4; ++i) pr[r2 * 4 + i] *= dp[r4 * 4 + i] - dl[i];
                    }
                }
                b_new[cc] = pack8(pr[0], pr[1], pr[2], pr[3], pr[4], pr[5], pr[6], pr[7]);
                back_step(cc);
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int i = 0; i < 8; ++i) b_new[cc][i] = (__bf16)0.f;
                back_step(cc);
            }
        }
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) b_old[cc] = b_new[cc];
        back_t = role == 0 ? fo : fq;
    };

    // ---- stage ring: s (computing), s+1 (landed or landing), s+2 (issued at the top of s)
    int g0 = next_group(p.key_range[2 * kt]), h0 = 0;           // stage s
    int g1 = g0, h1 = h0;                                       // stage s+1
    if (g0 < g_end) {
        issue_stage(g0, hk * G + h0, 0);
        succ(g1, h1);
        if (g1 < g_end) issue_stage(g1, hk * G + h1, 1);
    }
    int g2 = g1, h2 = h1;                                       // stage s+2
    int slot = 0;
    while (g0 < g_end) {
        if (g1 < g_end) succ(g2, h2); else g2 = g_end;
        const int4 gd = reinterpret_cast<const int4*>(p.group)[g0];
        const bool full = (gd.z <= k0) && (k0 + BNK <= gd.w);
        const bool live = (gd.x < kw0 + 32) && (gd.y > kw0);
        const bool has_pads = p.group_real[g0] < min(GR, p.n_q - g0 * GR);

        // stage s has landed once at most the copies of stage s+1 are outstanding
        if (g1 >= g_end) wait_vmem();
        else if (wave < 4) wait_vmem_le<BATCH + 1>();
        else wait_vmem_le<BATCH>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the previous block's LDS reads have returned
        __syncthreads();
        if (g2 < g_end) issue_stage(g2, hk * G + h2, (slot + 2) % NBUF);
        if (has_pads) {
            // padding rows may hold anything: clear them so they cannot poison the MFMAs
            const int r = tid >> 3, part = tid & 7;
            const int hi_r = *reinterpret_cast<const int*>(small + slot * SMALLB + 3 * GR * 4 + r * 4);
            if (hi_r == 0 && g0 * GR + r < p.n_q) {
                const i32x4 z = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < CPR / 8; ++i) {
                    *reinterpret_cast<i32x4*>(smem + slot * 2 * TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                    *reinterpret_cast<i32x4*>(smem + slot * 2 * TILEB + TILEB + r * ROWB + (part * (CPR / 8) + i) * 16) = z;
                }
            }
            __syncthreads();
        }
        if (full) {
            unit(slot, 0, live, std::false_type{});
            unit(slot, 1, live, std::false_type{});
        } else {
            unit(slot, 0, live, std::true_type{});
            unit(slot, 1, live, std::true_type{});
        }
        g0 = g1; h0 = h1; g1 = g2; h1 = h2;
        slot = (slot + 1) % NBUF;
    }
    // drain: the last block's dV/dK
    back_step(0);
    back_step(1);

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
}

template <int D>
__global__ void __launch_bounds__(512) dkv_duo_kernel(const BwdParams p) {
    constexpr int TILEB = kGroupRows * D * 2;
    __shared__ __attribute__((aligned(1024))) char smem[4 * 2 * TILEB];   // per slot: Q tile | dO tile, swizzled
    __shared__ __attribute__((aligned(1024))) char small[4 * 4 * kGroupRows * 4];
    const int rank = ((int)(blockIdx.x >> 3) / p.hkv) * 8 + (int)(blockIdx.x & 7);
    if (rank >= p.n_key_tiles) return;
    if (threadIdx.x < 256) dkv_duo_body<D, 0>(p, smem, small);
    else dkv_duo_body<D, 1>(p, smem, small);
}

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
    p.fwd_order = (const int32_t*)(ws + L.off_fwd_order);
    p.key_order = (const int32_t*)(ws + L.off_key_order);
    p.key_range = (const int32_t*)(ws + L.off_key_range);
    p.n_q = d.n_q; p.t_kv = d.t_kv; p.hq = d.hq; p.hkv = d.hkv;
    p.n_groups = L.n_groups; p.n_tiles = L.n_fwd_tiles; p.n_key_tiles = L.n_key_tiles;
    p.scale = d.scale;
    p.scale_log2e = d.scale * 1.4426950408889634f;
    p.exp_flags = getenv("WLB_EXP") ? atoi(getenv("WLB_EXP")) : 0;

    const size_t n_lanes = (size_t)d.n_q * d.hq * (d.head_dim / 8);
    const unsigned grid_delta = (unsigned)((n_lanes + 255) / 256);
    const unsigned grid_dq = (unsigned)((L.n_fwd_tiles + 7) / 8) * 8u * (unsigned)d.hq;
    const unsigned grid_dkv = (unsigned)((L.n_key_tiles + 7) / 8) * 8u * (unsigned)d.hkv;
    const bool do_delta = !(d.flags & WLB_ATTN_BWD_SKIP_DELTA);
    const bool do_dq = !(d.flags & WLB_ATTN_BWD_SKIP_DQ);
    const bool do_dkv = !(d.flags & WLB_ATTN_BWD_SKIP_DKV);
    static const int dkv_variant = getenv("WLB_DKV_VARIANT") ? atoi(getenv("WLB_DKV_VARIANT")) : 1;
    if (dkv_variant == 3 && do_dkv) {
        if (do_delta) { if (d.head_dim == 128) delta_kernel<128><<<grid_delta, 256, 0, stream>>>(p); else delta_kernel<64><<<grid_delta, 256, 0, stream>>>(p); }
        if (do_dq) { if (d.head_dim == 128) dq_pipe_kernel<128><<<grid_dq, 256, 0, stream>>>(p); else dq_pipe_kernel<64><<<grid_dq, 256, 0, stream>>>(p); }
        if (d.head_dim == 128) dkv_duo_kernel<128><<<grid_dkv, 512, 0, stream>>>(p);
        else dkv_duo_kernel<64><<<grid_dkv, 512, 0, stream>>>(p);
    } else
    if (dkv_variant == 2 && do_dkv) {
        if (do_delta) { if (d.head_dim == 128) delta_kernel<128><<<grid_delta, 256, 0, stream>>>(p); else delta_kernel<64><<<grid_delta, 256, 0, stream>>>(p); }
        if (do_dq) { if (d.head_dim == 128) dq_pipe_kernel<128><<<grid_dq, 256, 0, stream>>>(p); else dq_pipe_kernel<64><<<grid_dq, 256, 0, stream>>>(p); }
        if (d.head_dim == 128) dkv_ring_kernel<128><<<grid_dkv, 256, 0, stream>>>(p);
        else dkv_ring_kernel<64><<<grid_dkv, 256, 0, stream>>>(p);
    } else
    if (dkv_variant == 1 && do_dkv) {
        if (do_delta) { if (d.head_dim == 128) delta_kernel<128><<<grid_delta, 256, 0, stream>>>(p); else delta_kernel<64><<<grid_delta, 256, 0, stream>>>(p); }
        if (do_dq) { if (d.head_dim == 128) dq_pipe_kernel<128><<<grid_dq, 256, 0, stream>>>(p); else dq_pipe_kernel<64><<<grid_dq, 256, 0, stream>>>(p); }
        if (d.head_dim == 128) dkv_split_kernel<128><<<grid_dkv, 512, 0, stream>>>(p);
        else dkv_split_kernel<64><<<grid_dkv, 512, 0, stream>>>(p);
    } else if (d.head_dim == 128) {
        if (do_delta) delta_kernel<128><<<grid_delta, 256, 0, stream>>>(p);
        if (do_dq) dq_pipe_kernel<128><<<grid_dq, 256, 0, stream>>>(p);
        if (do_dkv) dkv_kernel<128><<<grid_dkv, 256, 0, stream>>>(p);
    } else {
        if (do_delta) delta_kernel<64><<<grid_delta, 256, 0, stream>>>(p);
        if (do_dq) dq_pipe_kernel<64><<<grid_dq, 256, 0, stream>>>(p);
        if (do_dkv) dkv_kernel<64><<<grid_dkv, 256, 0, stream>>>(p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "backward launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

}  // namespace wlb
