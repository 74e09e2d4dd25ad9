// Measurement aid: the dense bf16 MFMA rate this GPU sustains, so that the attention kernels'
// useful TFLOP/s can be quoted against a measured ceiling next to the published peak (the
// attention kernels are MFMA bound for long documents; paper Section 5.2 discusses kernel
// efficiency in achieved TFLOPs).  A launch issues nothing but 32x32x16 bf16 MFMAs on register
// operands: two wavefronts per SIMD, four independent accumulator chains each.  On MI355X the
// sustained rate depends on the operand values (all-ones runs measurably faster than random
// data, which is what attention sees), so the caller picks the operand kind.
#include <hip/hip_runtime.h>

#include "wlb_device.h"
#include "wlb_internal.h"

namespace wlb {

constexpr int kCalibBlocks = 512, kCalibThreads = 256, kCalibMfmaPerIter = 32;

__device__ __forceinline__ uint32_t calib_hash(uint32_t h) {
    h *= 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    return h;
}

__global__ void __launch_bounds__(kCalibThreads, 2) calib_mfma_kernel(float* sink, int n_iter, int random_operands) {
    bf16x8 a[8], b[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = calib_hash(threadIdx.x * 64u + s * 8u + i + blockIdx.x * 1315423911u);
            a[s][i] = random_operands ? (__bf16)(((int)(h & 0xffff) - 32768) * (1.f / 32768.f)) : (__bf16)1.0f;
            b[s][i] = random_operands ? (__bf16)(((int)(h >> 16) - 32768) * (1.f / 32768.f)) : (__bf16)1.0f;
        }
    f32x16 c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[j][r] = 0.f;
    for (int it = 0; it < n_iter; ++it) {
#pragma unroll
        for (int u = 0; u < kCalibMfmaPerIter / 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) c[j] = mfma32(a[(u + j) & 7], b[(u + 2 * j) & 7], c[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[j][r];
    if (s == 12345.678f) sink[0] = s;      // keeps the accumulators live; practically never true
}

// Second measurement aid: the rate at which fp32 tiles are added into device memory with atomics.  A backward
// pass in one kernel (dQ, dK and dV from one computation of S and dP: 10*D executed flops per pair instead of the
// 14*D of the two-kernel backward) keeps dK/dV of its key tile in registers and has to add a 64 x 128 fp32 dQ tile
// to memory for every (row group, head) it streams; this kernel does nothing but such additions -- one workgroup
// per compute unit, each adding tile after tile (agent-scope atomic add without return value, 32 per lane and
// tile) -- into tiles of its own or into tiles all workgroups share.
constexpr int kAtomicTileFloats = 64 * 128, kAtomicThreads = 256;

__global__ void __launch_bounds__(kAtomicThreads) calib_atomic_kernel(float* buf, int n_tiles, int n_iter, int shared) {
    for (int it = 0; it < n_iter; ++it) {
        const int tile = shared ? (int)((blockIdx.x * 7u + (unsigned)it) % (unsigned)n_tiles)
                                : (int)((blockIdx.x + (unsigned)it * gridDim.x) % (unsigned)n_tiles);
        float* t = buf + (size_t)tile * kAtomicTileFloats;
#pragma unroll 8
        for (int i = threadIdx.x; i < kAtomicTileFloats; i += kAtomicThreads)
            __hip_atomic_fetch_add(t + i, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace wlb

extern "C" wlb_status wlb_calib_atomic_add(int32_t shared, int32_t n_iter, float* buf, size_t buf_bytes, double* bytes_added,
                                           void* stream) {
    using namespace wlb;
    const size_t tile_bytes = sizeof(float) * kAtomicTileFloats;
    if (!buf || !bytes_added || n_iter < 1 || n_iter > (1 << 20) || buf_bytes < tile_bytes || buf_bytes / tile_bytes > (1u << 30))
        return fail(WLB_ERR_INVALID_ARG, "wlb_calib_atomic_add: null pointer, n_iter=%d outside [1, 2^20] or a buffer under one tile", n_iter);
    const int n_tiles = (int)(buf_bytes / tile_bytes), grid = compute_units();
    calib_atomic_kernel<<<grid, kAtomicThreads, 0, (hipStream_t)stream>>>(buf, n_tiles, n_iter, shared != 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "calibration launch: %s", hipGetErrorString(e));
    *bytes_added = (double)grid * n_iter * (double)tile_bytes;
    return WLB_OK;
}

extern "C" wlb_status wlb_calib_mfma(int32_t random_operands, int32_t n_iter, float* sink, double* flops, void* stream) {
    using namespace wlb;
    if (!sink || !flops || n_iter < 1 || n_iter > (1 << 20))
        return fail(WLB_ERR_INVALID_ARG, "wlb_calib_mfma: null pointer or n_iter=%d outside [1, 2^20]", n_iter);
    calib_mfma_kernel<<<kCalibBlocks, kCalibThreads, 0, (hipStream_t)stream>>>(sink, n_iter, random_operands != 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(WLB_ERR_HIP, "calibration launch: %s", hipGetErrorString(e));
    *flops = (double)kCalibBlocks * (kCalibThreads / 64) * (double)n_iter * kCalibMfmaPerIter * (2.0 * 32 * 32 * 16);
    return WLB_OK;
}
