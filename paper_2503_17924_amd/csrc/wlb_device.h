// Device-side helpers shared by the gfx950 kernels of libwlb: vector types, MFMA wrappers,
// LDS transpose reads, bf16 packing.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace wlb {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

#define WLB_LDS __attribute__((address_space(3)))

// D[32x32] += A[32x16] * B[16x32], bf16 inputs, fp32 accumulate, one wavefront.
// Lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32];
// accumulator register i of lane l is D[(i/4)*8 + (l/32)*4 + i%4][l%32].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane i passes the
// address of 4 consecutive 16-bit values M[i][0..3]; lane j receives M[4e + j/4][j%4] for
// e = 0..3.  With lane i pointing at row (r0 + i/4), columns c0 + 4*(i%4) .. +3 of a row-major
// tile X, lane j therefore receives X[r0+e][c0+j]: four rows of one column.
__device__ __forceinline__ bf16x4 lds_read_tr4(const __bf16* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((WLB_LDS s16x4*)(uintptr_t)(uint32_t)(uintptr_t)p);
    return __builtin_bit_cast(bf16x4, r);
}

// same, from a 32-bit LDS address
__device__ __forceinline__ bf16x4 lds_read_tr4_at(uint32_t lds_addr) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((WLB_LDS s16x4*)(uintptr_t)lds_addr);
    return __builtin_bit_cast(bf16x4, r);
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// exchange a value with the lane 32 away (both directions in one instruction)
__device__ __forceinline__ float xhalf(float x) {
    int xi = __builtin_bit_cast(int, x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    int other = (threadIdx.x & 32) ? r[0] : r[1];
    return __builtin_bit_cast(float, other);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5,
                                        float a6, float a7) {
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

__device__ __forceinline__ bf16x4 pack4(float a0, float a1, float a2, float a3) {
    bf16x4 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    return r;
}

// tells the compiler that a value is the same in every lane (moves it to a scalar register)
__device__ __forceinline__ uint32_t uniform(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Loads through the constant address space: with a wave-uniform address they become scalar
// loads (counted by lgkmcnt, not vmcnt, so they do not interfere with the asynchronous tile
// copies).  Only for data no kernel writes while this one runs (the schedule tables).
#define WLB_CONST __attribute__((address_space(4)))
__device__ __forceinline__ int ld_const(const int32_t* p) {
    return *reinterpret_cast<const WLB_CONST int*>((uintptr_t)p);
}
__device__ __forceinline__ int4 ld_const4(const int32_t* p) {
    const i32x4 v = *reinterpret_cast<const WLB_CONST i32x4*>((uintptr_t)p);
    return int4{v[0], v[1], v[2], v[3]};
}

__device__ __forceinline__ long long ld_const64(const long long* p) {
    return *reinterpret_cast<const WLB_CONST long long*>((uintptr_t)p);
}

// ------------------------------------------------------------------------------------------
// Work schedule of the forward and dQ kernels.  The query tiles in order (heaviest first), each
// repeated for every KV head, form one line of work measured in key tiles (each tile's stretch
// begins with a few units that stand for its fixed cost).  A launch has n_gangs gangs of G = hq / hkv workgroups (one per query head of a KV
// head); the gangs take consecutive shares of the line, so a gang's load does not depend on the
// tiles' sizes.  The shares are weighted: those of the first half of the gangs are larger than those
// of the second half (with two workgroups per compute unit the workgroups of the first half of the
// launch are the older wavefronts of their SIMDs, win issue arbitration and advance faster), and a
// caller that has measured how fast each XCD of its GPU runs can weight them by XCD as well
// (wlb_attn_set_gang_weights).  A tile cut by a share's end is continued by
// the next gang; the pieces of such a tile leave fp32 partial results that a merge kernel
// combines.  Workgroup b is member (b / 8) % G of gang ((b / 8) / G) * 8 + b % 8: consecutive
// workgroups go to consecutive XCDs, so a gang's members share an XCD (and its L2 copy of K/V).
struct RowSched {
    const long long* prefix;   // [n_tiles + 1] cost of the query tiles before order rank r
    const int32_t* order;      // [n_tiles]
    int n_tiles, hkv, G, n_gangs;
    // relative share of a gang, by the half of the launch it belongs to and by its XCD (gang g runs on XCD
    // g % 8): weight[0][x] for the first n_gangs / 2 gangs, weight[1][x] for the rest
    int weight[2][8];
    // sum of the weights of the gangs before g (indices fixed at compile time: the table stays in scalar registers)
    __device__ __forceinline__ long long weight_before(int g) const {
        const int g0 = g < n_gangs / 2 ? g : n_gangs / 2;      // of them, those in the first half
        long long cum = 0;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int n0 = (g0 + 7 - x) >> 3, n = (g + 7 - x) >> 3;   // gangs i < g0 (i < g) with i % 8 == x
            cum += (long long)n0 * weight[0][x] + (long long)(n - n0) * weight[1][x];
        }
        return cum;
    }
    // first unit of gang g's share of a line of W units (g = n_gangs: W)
    __device__ __forceinline__ long long share_begin(long long W, int g) const {
        return W * weight_before(g) / weight_before(n_gangs);
    }
};
struct RowPiece {
    int tile, hk, member;
    int a, b, c;               // units [a, b) of the tile's c
    int slot;                  // partial result index, -1 for a whole tile (a == 0 and b == c)
};
struct RowWalk {
    long long pos, end;
    int r, hk, gang, member;
    __device__ __forceinline__ void start(const RowSched& s, int block) {
        const int x = block & 7, i = block >> 3;
        member = i % s.G;
        gang = (i / s.G) * 8 + x;
        const long long W = s.hkv * ld_const64(s.prefix + s.n_tiles);
        pos = s.share_begin(W, gang);
        end = s.share_begin(W, gang + 1);
        r = 0; hk = 0;
        if (pos >= end) return;
        locate(s, pos, r, hk);
    }
    // the (order rank, KV head) whose stretch of the line contains unit u < W
    __device__ static __forceinline__ void locate(const RowSched& s, long long u, int& r, int& hk) {
        int lo = 0, hi = s.n_tiles;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s.hkv * ld_const64(s.prefix + mid) <= u) lo = mid; else hi = mid;
        }
        const long long p0 = ld_const64(s.prefix + lo), c = ld_const64(s.prefix + lo + 1) - p0;
        r = lo;
        hk = (int)((u - s.hkv * p0) / c);
    }
    __device__ __forceinline__ bool next(const RowSched& s, RowPiece& pc) {
        if (pos >= end) return false;
        const long long p0 = ld_const64(s.prefix + r);
        const int c = (int)(ld_const64(s.prefix + r + 1) - p0);
        const long long st = s.hkv * p0 + (long long)hk * c;
        pc.tile = ld_const(s.order + r);
        pc.hk = hk; pc.member = member; pc.c = c;
        pc.a = (int)(pos - st);
        pc.b = (int)((end - st < c) ? end - st : c);
        // a piece that starts inside a tile is its gang's first, one that ends inside a tile its last
        pc.slot = (pc.a == 0 && pc.b == c) ? -1 : ((pc.a > 0 ? 2 * gang : 2 * gang + 1) * s.G + member);
        pos = st + c;
        if (++hk == s.hkv) { hk = 0; ++r; }
        return true;
    }
};

// For the merge kernels: the query tile whose first part is gang `gang`'s last piece, if there is
// one, and the partial results of its parts.  Partial slot 2g holds gang g's first piece when it
// starts inside a tile, slot 2g + 1 its last piece when that ends inside a tile (times G members).
struct RowCut {
    const RowSched* s;
    long long W, tile_end;
    int gang, tile, hk;
    // false: this gang's last piece is a whole tile or continues a tile begun by an earlier gang
    __device__ __forceinline__ bool find(const RowSched& sched, int g) {
        s = &sched; gang = g;
        W = sched.hkv * ld_const64(sched.prefix + sched.n_tiles);
        const long long w0 = sched.share_begin(W, g), w1 = sched.share_begin(W, g + 1);
        if (w0 >= w1) return false;
        int r;
        RowWalk::locate(sched, w1 - 1, r, hk);
        const long long p0 = ld_const64(sched.prefix + r);
        const long long c = ld_const64(sched.prefix + r + 1) - p0;
        const long long st = sched.hkv * p0 + hk * c;
        if (st < w0 || w1 - st >= c) return false;
        tile_end = st + c;
        tile = ld_const(sched.order + r);
        return true;
    }
    // slot index (before the member) of the first part
    __device__ __forceinline__ int first_slot() const { return 2 * gang + 1; }
    // calls f(slot index) for the first piece of every later gang whose (non-empty) share begins inside the tile
    template <class F>
    __device__ __forceinline__ void later_parts(F f) const {
        for (int g2 = gang + 1; g2 < s->n_gangs; ++g2) {
            const long long b0 = s->share_begin(W, g2), b1 = s->share_begin(W, g2 + 1);
            if (b0 >= tile_end) break;
            if (b1 > b0) f(2 * g2);
        }
    }
};

// The slot indices of a cut tile's later parts, found once per workgroup (each step of RowCut::later_parts
// costs two 64-bit divisions, and the merge kernels need the list for every element they combine): thread 0
// walks them and leaves up to CAP of them in shared memory.  Returns their number; above CAP the caller
// falls back to RowCut::later_parts.  Every thread of the workgroup must call it.
template <int CAP>
__device__ __forceinline__ int gather_later_parts(const RowCut& cut, int* s_slots, int* s_count) {
    if (threadIdx.x == 0) {
        int n = 0;
        cut.later_parts([&](int slot) {
            if (n < CAP) s_slots[n] = slot;
            ++n;
        });
        *s_count = n;
    }
    __syncthreads();
    return *s_count;
}

// XOR swizzle of the 16-byte chunks of an unpadded row-major LDS tile whose rows hold CPR
// chunks: logical chunk cc of row r is stored at chunk swz(r, cc).  It makes both access patterns
// of the kernels bank-conflict free: 16 rows x one chunk (b128 MFMA operand reads) and 4 rows x 4
// consecutive chunks (transpose reads).  An LDS access covers 256 bytes per cycle.  With 256-byte
// rows (head_dim 128) a row is one such line and the 16 rows of a read must land in 16 different
// chunk positions: row bits 0-1 go to chunk bits 2-3 and row bits 2-3 to chunk bits 0-1.  With
// 128-byte rows (head_dim 64) two rows share a line -- the row's lowest bit already selects the
// half -- so row bits 1-3 take that part: bit 1 to chunk bit 2, bits 2-3 to chunk bits 0-1.
template <int CPR>
__host__ __device__ __forceinline__ constexpr int swz(int r, int cc) {
    static_assert(CPR == 8 || CPR == 16, "rows of 128 or 256 bytes");
    return CPR == 16 ? cc ^ (((r & 3) << 2) | ((r >> 2) & 3))
                     : cc ^ ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

// Asynchronous global -> LDS copy of a tile of ROWS rows x D bf16 (rows contiguous in LDS,
// 16-byte chunks swizzled), issued by all NW wavefronts of a workgroup.  Each instruction is a
// buffer load that moves 64 x 16 bytes straight into LDS without passing through registers;
// lane i's 16 bytes land at (instruction's LDS base) + 16*i, so the swizzle is applied on the
// global side.  The buffer descriptor bounds the tensor: rows past its end read as zeros, so
// ragged last tiles need no clamping.  Completion: wait_vmem() + workgroup barrier.
struct BufRsrc {
    i32x4 r;   // buffer descriptor: base address, stride 0, num_records = bytes, raw 32-bit format
    __device__ __forceinline__ void init(const void* base, uint32_t bytes) {
        const uint64_t a = (uint64_t)(uintptr_t)base;
        r[0] = (int)(uint32_t)a;
        r[1] = (int)(uint32_t)((a >> 32) & 0xffffu);
        r[2] = (int)bytes;
        r[3] = 0x00020000;
    }
    // for descriptors whose base was chosen per wavefront: move the (wave-uniform) words to scalar registers
    __device__ __forceinline__ void make_uniform() {
        r[0] = __builtin_amdgcn_readfirstlane(r[0]);
        r[1] = __builtin_amdgcn_readfirstlane(r[1]);
        r[2] = __builtin_amdgcn_readfirstlane(r[2]);
    }
};

// One buffer_load_dwordx4 ... lds: 64 lanes x 16 bytes from (descriptor base + soff + voff)
// into LDS at lds_addr + 16*lane.  Written as inline assembly so that the compiler does not
// serialise later LDS reads of OTHER buffers behind this copy; the callers order reads of the
// destination buffer themselves (wait_vmem + barrier).  The statement writes m0 (the LDS base of
// the copy) and says so in its clobber list; the compiler's remark that m0 is a reserved
// register is expected and switched off for these two statements.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_issue_1k(const i32x4& rsrc, uint32_t lds_addr, int voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

template <int D, int ROWS, int NW>
struct TileDma {
    static constexpr int CPR = D / 8;         // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;      // rows per instruction
    static constexpr int NI = ROWS / RPI;     // instructions per tile
    static constexpr int PER = NI / NW;       // instructions per wavefront
    static_assert(NI % NW == 0, "tile must split evenly over the wavefronts");
    int voff[PER];                            // per-lane byte offsets inside the instruction's rows
    uint32_t row_bytes;

    __device__ __forceinline__ void init(int wave, int lane, uint32_t stride_elems) {
        row_bytes = stride_elems * 2;
#pragma unroll
        for (int n = 0; n < PER; ++n) {
            const int blk = wave * PER + n;
            const int ri = lane / CPR;
            const int cc = swz<CPR>(blk * RPI + ri, lane % CPR);   // source chunk for this LDS slot
            voff[n] = ri * (int)row_bytes + cc * 16;
        }
    }
    // rows row0 .. row0+ROWS-1 of the tensor -> the tile at LDS byte address lds_tile (ROWS * D * 2
    // bytes).  `wave` must be wave-uniform in the compiler's eyes (take it through uniform()), so
    // that the LDS address and the row offset are computed on the scalar unit.
    __device__ __forceinline__ void issue(const BufRsrc& rs, uint32_t lds_tile, int row0, int wave) const {
#pragma unroll
        for (int n = 0; n < PER; ++n) {
            const int blk = wave * PER + n;
            const uint32_t soff = (uint32_t)(row0 + blk * RPI) * row_bytes;
            dma_issue_1k(rs.r, uniform(lds_tile + (uint32_t)blk * 1024u), voff[n], uniform(soff));
        }
    }
};

// 64 lanes x 4 bytes (one dword per lane, consecutive in LDS) from descriptor base + soff + 4*lane
__device__ __forceinline__ void dma_issue_256(const i32x4& rsrc, uint32_t lds_addr, int voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

#pragma clang diagnostic pop

// wait until at most N of this wavefront's most recent vector-memory operations are outstanding
template <int N>
__device__ __forceinline__ void wait_vmem_le() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)
// every LDS access this wavefront has issued is complete (before a copy overwrites what was read)
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xC07F); }    // lgkmcnt(0)

// ------------------------------------------------------------------------------------------
// Whole-row moves for the short-hull kernels: rows row0 .. row0+31 of one head of a
// [n][heads][D] bf16 tensor travel between global memory, registers and a 32-row LDS tile
// (swizzled like the K/V tiles) as complete rows -- every instruction covers RPI whole rows,
// 64 lanes x 16 bytes -- through a bounds-checked buffer descriptor of the whole tensor, so rows
// past its end load as zeros and are not stored, without a branch.
typedef __amdgpu_buffer_rsrc_t buf_rsrc_t;
__device__ __forceinline__ buf_rsrc_t make_buf(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
template <int D>
struct RowBlock {
    static constexpr int CPR = D / 8, ROWB = D * 2, RPI = 64 / CPR, N = 32 / RPI;
    i32x4 v[N];
    // lane's byte offset inside an instruction's rows, and the instructions' scalar offsets:
    // row0 * row_bytes + head * ROWB + i * RPI * row_bytes
    static __device__ __forceinline__ int lane_off(int lane, uint32_t row_bytes) { return (lane / CPR) * (int)row_bytes + (lane % CPR) * 16; }
    __device__ __forceinline__ void load(buf_rsrc_t rs, int voff, uint32_t soff0, uint32_t row_bytes) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, (int)(soff0 + i * RPI * row_bytes), 0));
    }
    __device__ __forceinline__ void store(buf_rsrc_t rs, int voff, uint32_t soff0, uint32_t row_bytes) const {
#pragma unroll
        for (int i = 0; i < N; ++i) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) unsigned, v[i]), rs, voff, (int)(soff0 + i * RPI * row_bytes), 0);
    }
    __device__ __forceinline__ void to_tile(uint32_t tile, int lane) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int r = i * RPI + lane / CPR, c = lane % CPR;
            *reinterpret_cast<WLB_LDS i32x4*>((uintptr_t)(tile + r * ROWB + swz<CPR>(r, c) * 16)) = v[i];
        }
    }
    __device__ __forceinline__ void from_tile(uint32_t tile, int lane) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int r = i * RPI + lane / CPR, c = lane % CPR;
            v[i] = *reinterpret_cast<const WLB_LDS i32x4*>((uintptr_t)(tile + r * ROWB + swz<CPR>(r, c) * 16));
        }
    }
};

constexpr int kPadLo = 0x7fffffff;  // row_lo of a padding row (row_hi = 0): no key satisfies lo <= k < hi

// Key tiles (of BN keys) a wavefront of 32 rows needs no element-wise mask for.  The rows are split by the
// start of their key interval [lo, hi): the rows that share the smallest start (the first document in the
// wavefront) see every key of the tiles [fb, fe); the other real rows (`other`: rows of later documents
// that share the wavefront) see none of them and are switched off as whole lanes there.  A wavefront of one
// document gets the range all its rows see in full and no lane with `other` set; neither does one whose
// range is empty.  Both halves of the
// wavefront hold the same 32 rows, so the reductions run over the 32 lanes of a half.
template <int BN>
__device__ __forceinline__ void unmasked_tiles(int lo, int hi, bool real, int& fb, int& fe, bool& other) {
    int lo_min = real ? lo : kPadLo;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) lo_min = min(lo_min, __shfl_xor(lo_min, o));
    const bool first = real && lo == lo_min;
    other = real && !first;
    int end = first ? hi : (other ? lo : kPadLo);      // the range ends where a first-document row stops seeing keys
#pragma unroll                                         // or another document's keys begin
    for (int o = 16; o > 0; o >>= 1) end = min(end, __shfl_xor(end, o));
    const int b = lo_min == kPadLo ? 0 : (lo_min + BN - 1) / BN;
    const int e = end == kPadLo ? 0 : end / BN;
    fb = __builtin_amdgcn_readfirstlane(b);
    fe = __builtin_amdgcn_readfirstlane(e < b ? b : e);
    if (fe == fb) other = false;       // no such tile: every block is classified on its own
}

}  // namespace wlb
