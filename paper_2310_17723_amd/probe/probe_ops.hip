// Diagnostics, not on the hot path: the ceilings the kernels are measured against, taken on the machine at
// hand.  hero_probe_mfma_i8 runs a register-only loop of v_mfma_i32_32x32x32_i8 (one 512-thread workgroup per CU,
// two waves per SIMD, eight independent accumulators per wave, nothing else in the loop), whose rate is the
// matrix cores' rate at the clock the chip sustains under that load.  The clock depends on how many operand bits
// toggle, so the operands are either near-constant or random bytes.  hero_probe_copy is a plain device copy.
#include "hero_common.h"

namespace {

__device__ __forceinline__ unsigned lcg(unsigned& s) { s = s * 1664525u + 1013904223u; return s ^ (s >> 13) ^ (s << 7); }

__global__ __launch_bounds__(512) void probe_mfma_i8_kernel(int random_bytes, int iters, int* sink) {
    typedef int v16i_t __attribute__((ext_vector_type(16)));
    unsigned seed = threadIdx.x * 7919u + blockIdx.x * 104729u + 1u;
    v4i fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) fa[i][j] = random_bytes ? (int)lcg(seed) : 0x01010101;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[i][j] = random_bytes ? (int)lcg(seed) : 0x01010101;
    v16i_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            acc[n & 7] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[(n >> 2) & 1], fa[n & 3], acc[n & 7], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 0x7fffffff) sink[0] = s;                     // keeps the loop alive; never true for these operands' sums
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace

extern "C" hero_status hero_probe_mfma_i8(int random_bytes, int64_t iters, int32_t* sink, double* ops, void* stream) {
    if (iters <= 0 || iters > 0x7fffffffLL) return HERO_ERR_SHAPE;
    if (!sink) return HERO_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return HERO_ERR_LAUNCH;
    hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3((unsigned)cus), dim3(512), 0, (hipStream_t)stream, random_bytes, (int)iters, sink);
    if (ops) *ops = (double)cus * 8.0 * (double)iters * 16.0 * 65536.0;      // 8 waves x 16 instructions x 2*32*32*32 per iteration
    return hero_launch_status();
}

extern "C" hero_status hero_probe_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (bytes < 0 || bytes % 16 != 0) return HERO_ERR_SHAPE;
    if (bytes == 0) return HERO_OK;
    if (!src || !dst) return HERO_ERR_NULL;
    if (!hero_aligned16(src) || !hero_aligned16(dst)) return HERO_ERR_ALIGN;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const v4i*)src, (v4i*)dst, bytes / 16);
    return hero_launch_status();
}
