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

constexpr int kPadLo = 0x7fffffff;  // row_lo of a padding row (row_hi = 0): no key satisfies lo <= k < hi

}  // namespace wlb
