// Forward document-masked attention for gfx950 (paper Sections 1 and 3.2 define the mask:
// causal inside a document, nothing across documents; Section 2.1 the data flow: one
// context-parallel rank's query rows against the whole packed sequence's K/V).
//
// One workgroup = one query tile of 128 local rows x one query head.  Each wavefront owns
// QB blocks of 32 rows and keeps, per block, the bf16 Q operands, the running row max and sum
// and the transposed output accumulator O^T[d][q] in registers.  K and V tiles of 64 keys are
// staged in LDS.  Scores are computed transposed, S^T = K Q^T, with the 32x32x16 bf16 MFMA: a
// lane then holds one query column and 16 key rows per block, so the row max/sum are
// in-register reductions plus one exchange between the two lane halves, and the
// exponentiated block is already laid out as the B operand of O^T += V^T P^T.  The V^T
// operand comes from the row-major V tile through LDS transpose reads.
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
};

template <int D, int QB, int NW>
__global__ void __launch_bounds__(NW * 64) fwd_kernel(const FwdParams p) {
    constexpr int BM = 32 * QB * NW;
    static_assert(BM == kFwdTileRows, "tile rows must match the schedule");
    constexpr int BN = 64;
    constexpr int NT = NW * 64;
    constexpr int KS = D / 16;         // contraction steps of S^T = K Q^T
    constexpr int DB = D / 32;         // 32-row blocks of O^T
    constexpr int KSTR = D + 8;        // LDS row strides (elements): K rows 16 B apart in banks,
    constexpr int VSTR = D + 32;       // V rows 64 B apart (four rows of a transpose read disjoint)
    constexpr int CPR = D / 8;         // 16-byte chunks per row

    __shared__ __attribute__((aligned(16))) __bf16 Ks[BN * KSTR];
    __shared__ __attribute__((aligned(16))) __bf16 Vs[BN * VSTR];

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
    const size_t kv_row = (size_t)p.hkv * D;
    const __bf16* kbase = p.k + (size_t)hk * D;
    const __bf16* vbase = p.v + (size_t)hk * D;

    for (int j = jb; j < je; ++j) {
        __syncthreads();   // everyone is done reading the previous tile
        for (int ch = tid; ch < BN * CPR; ch += NT) {
            const int r = ch / CPR, cc = ch % CPR;
            const int kr = min(j * BN + r, p.t_kv - 1);
            const i32x4 kk = *reinterpret_cast<const i32x4*>(kbase + (size_t)kr * kv_row + cc * 8);
            const i32x4 vv = *reinterpret_cast<const i32x4*>(vbase + (size_t)kr * kv_row + cc * 8);
            *reinterpret_cast<i32x4*>(&Ks[r * KSTR + cc * 8]) = kk;
            *reinterpret_cast<i32x4*>(&Vs[r * VSTR + cc * 8]) = vv;
        }
        __syncthreads();

        // ---- S^T = K Q^T for two blocks of 32 keys
        f32x16 s[2][QB];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int b = 0; b < QB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][b][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(kb * 32 + l32) * KSTR + ks * 16 + half * 8]);
#pragma unroll
                for (int b = 0; b < QB; ++b) s[kb][b] = mfma32(a, qf[b][ks], s[kb][b]);
            }
        }

        const bool partial = (j < fb) || (j >= fe);
        if (partial) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j * BN + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
#pragma unroll
                    for (int b = 0; b < QB; ++b)
                        s[kb][b][r] = (key >= lo[b] && key < hi[b]) ? s[kb][b][r] : -INFINITY;
                }
        }

        // ---- online softmax per query column, then O^T += V^T P^T
        bf16x8 pf[QB][2][2];
#pragma unroll
        for (int b = 0; b < QB; ++b) {
            float mx = s[0][b][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][b][r]);
            mx = fmaxf(mx, xhalf(mx));
            const float m_new = fmaxf(m[b], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2((m[b] - m_use) * cs);
            const float mc = m_use * cs;
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = fast_exp2(fmaf(s[kb][b][r], cs, -mc));
                    s[kb][b][r] = e;
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
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc)
                    pf[b][kb][cc] = pack8(s[kb][b][8 * cc + 0], s[kb][b][8 * cc + 1], s[kb][b][8 * cc + 2],
                                          s[kb][b][8 * cc + 3], s[kb][b][8 * cc + 4], s[kb][b][8 * cc + 5],
                                          s[kb][b][8 * cc + 6], s[kb][b][8 * cc + 7]);
        }

        // V^T operand: lane (d = db*32 + l32, half) needs keys {K0 + 4*half + 0..3, K0 + 8 + 4*half + 0..3}
        {
            const int j16 = lane & 15, gi = (lane >> 4) & 1;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const int key0 = kb * 32 + cc * 16 + half * 4 + (j16 >> 2);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const int d0 = db * 32 + gi * 16 + (j16 & 3) * 4;
                        const bf16x4 v0 = lds_read_tr4(&Vs[key0 * VSTR + d0]);
                        const bf16x4 v1 = lds_read_tr4(&Vs[(key0 + 8) * VSTR + d0]);
                        const bf16x8 a = cat4(v0, v1);
#pragma unroll
                        for (int b = 0; b < QB; ++b) acc[b][db] = mfma32(a, pf[b][kb][cc], acc[b][db]);
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
    const unsigned grid = (unsigned)((L.n_fwd_tiles + 7) / 8) * 8u * (unsigned)d.hq;
    if (d.head_dim == 128) fwd_kernel<128, 2, 2><<<grid, 128, 0, stream>>>(p);
    else fwd_kernel<64, 2, 2><<<grid, 128, 0, stream>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "forward launch: %s", hipGetErrorString(e));
    return WLB_OK;
}

}  // namespace wlb
