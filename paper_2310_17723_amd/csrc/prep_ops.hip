// Model-load-time operators of the method, on the GPU (not on the hot path):
//   hero_absmax_cols       the calibration statistic behind the FWQ / SQ scales (paper Sec. 2.1: these
//                          scales are fixed by a calibration pass before inference; Sec. 3: the range
//                          recorded over calibration batches, no truncation)
//   hero_weight_fold_quant scale folding (Sec. 2.2.2: W~_q = W_q / S_q, W~_o = S_attn W_o / S_o;
//                          Sec. 2.2.3: W~_2 = S_a W_2 / S_x2) followed by the column-wise weight
//                          quantization W = W_int8 Diag(S_w) of Sec. 2.1, codes stored [N][K]
//                          (each output column's K values contiguous: the GEMM's operand layout);
//                          hero_weight_fold_quant_fp8: the same with E4M3 codes and scale max / 448.
// Both are bandwidth-trivial one-off passes; they are written for exactness (the fold runs in fp64,
// multiply then divide, one cast to fp32, IEEE division by the scale, round half to even) so that the
// codes are bit-identical to the definition's.
#include "hero_common.h"

namespace {

// ---- column-wise max |x| over the rows, merged into a running maximum --------------------------
// Non-negative floats order like their bit patterns, so the merge is an integer atomic max.
template <int DT>
__global__ __launch_bounds__(256) void absmax_cols_kernel(const void* x, int64_t ldx, int64_t T, int D, float* col_absmax,
                                                          int rows_per_block) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= D) return;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block, r1 = min(r0 + rows_per_block, T);
    float m = 0.0f;
    for (int64_t r = r0; r < r1; ++r) {
        float v;
        if (DT == HERO_F32) v = ((const float*)x)[r * ldx + col];
        else v = hp_to_f32<DT>(((const uint16_t*)x)[r * ldx + col]);
        m = fmaxf(m, fabsf(v));                                   // NaN inputs are ignored by fmaxf
    }
    atomicMax(reinterpret_cast<int*>(col_absmax) + col, __float_as_int(m));
}

// ---- fold + column-wise quantization ------------------------------------------------------------
__device__ __forceinline__ float folded(const float* W, int64_t ldw, const float* row_mult, const float* col_div, int k, int n) {
    double v = (double)W[(int64_t)k * ldw + n];
    if (row_mult) v = (double)row_mult[k] * v;
    if (col_div) v = v / (double)col_div[n];
    return (float)v;
}

// pass 1: amax[n] = max_k |W~[k][n]|  (amax zero-filled before)
__global__ __launch_bounds__(256) void fold_absmax_kernel(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                                          int K, int N, float* amax, int rows_per_block) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const int k0 = blockIdx.y * rows_per_block, k1 = min(k0 + rows_per_block, K);
    float m = 0.0f;
    for (int k = k0; k < k1; ++k) m = fmaxf(m, fabsf(folded(W, ldw, row_mult, col_div, k, n)));
    atomicMax(reinterpret_cast<int*>(amax) + n, __float_as_int(m));
}

// pass 2: codes, transposed through LDS: a 64 x 64 tile is read along n (coalesced), written along k
// F8: E4M3 codes with scale max / 448 (the FP8 variant of Sec. 2.1) instead of INT8 codes with scale max / 127
template <bool F8>
__global__ __launch_bounds__(256) void fold_quant_kernel(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                                         int K, int N, const float* amax, int8_t* Wt, int64_t ldwt) {
    __shared__ int8_t tile[64][64 + 4];                           // [n][k]
    const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tn = threadIdx.x & 63, tk = threadIdx.x >> 6;       // 4 k-rows per sweep
    const int n = n0 + tn;
    float sc = 1.0f;
    if (n < N) { const float a = amax[n]; sc = a == 0.0f ? 1.0f : __fdiv_rn(a, F8 ? 448.0f : 127.0f); }
    for (int kk = tk; kk < 64; kk += 4) {
        const int k = k0 + kk;
        int code = 0;
        if (n < N && k < K) {
            const float w = folded(W, ldw, row_mult, col_div, k, n);
            if (F8) code = (int)(fp8x4_sat(__fdiv_rn(w, sc), 0.0f, 0.0f, 0.0f) & 0xffu);
            else code = quant_code_div(w, sc);
        }
        tile[tn][kk] = (int8_t)code;
    }
    __syncthreads();
    const int wk = threadIdx.x & 63, wn = threadIdx.x >> 6;
    for (int nn = wn; nn < 64; nn += 4)
        if (n0 + nn < N && k0 + wk < K) Wt[(int64_t)(n0 + nn) * ldwt + k0 + wk] = tile[nn][wk];
}

// pass 3: amax -> scale, in place
__global__ void amax_to_scale_kernel(float* s, int N, float qmax) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n < N) { const float a = s[n]; s[n] = a == 0.0f ? 1.0f : __fdiv_rn(a, qmax); }
}

__global__ void fill_f32_kernel(float* p, int n, float v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

extern "C" hero_status hero_absmax_cols(const void* x, hero_dtype x_dt, int64_t ldx, int64_t T, int64_t D,
                                        float* col_absmax, void* stream) {
    if (T < 0 || D <= 0 || D > 0x7fffffffLL || ldx < D) return HERO_ERR_SHAPE;
    if (x_dt != HERO_F32 && x_dt != HERO_BF16 && x_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (T == 0) return HERO_OK;
    if (!x || !col_absmax) return HERO_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    // enough row ranges to occupy the chip, at least 64 rows each
    int64_t ranges = (2048 + (D + 255) / 256 - 1) / ((D + 255) / 256);
    int64_t rpb = (T + ranges - 1) / ranges;
    if (rpb < 64) rpb = 64;
    ranges = (T + rpb - 1) / rpb;
    if (ranges > 65535) { ranges = 65535; rpb = (T + ranges - 1) / ranges; }
    const dim3 grid((unsigned)((D + 255) / 256), (unsigned)ranges);
    if (x_dt == HERO_F32) hipLaunchKernelGGL((absmax_cols_kernel<HERO_F32>), grid, dim3(256), 0, st, x, ldx, T, (int)D, col_absmax, (int)rpb);
    else if (x_dt == HERO_BF16) hipLaunchKernelGGL((absmax_cols_kernel<HERO_BF16>), grid, dim3(256), 0, st, x, ldx, T, (int)D, col_absmax, (int)rpb);
    else hipLaunchKernelGGL((absmax_cols_kernel<HERO_F16>), grid, dim3(256), 0, st, x, ldx, T, (int)D, col_absmax, (int)rpb);
    return hero_launch_status();
}

namespace {
hero_status weight_fold_quant_entry(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                    int64_t K, int64_t N, int8_t* Wt, int64_t ldwt, float* col_scale, bool fp8, void* stream) {
    if (K <= 0 || N <= 0 || K > 0x7fffffffLL || N > 0x7fffffffLL || ldw < N || ldwt < K) return HERO_ERR_SHAPE;
    if ((N + 63) / 64 > 0x7fffffffLL || (K + 63) / 64 > 65535) return HERO_ERR_SHAPE;
    if (!W || !Wt || !col_scale) return HERO_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, col_scale, (int)N, 0.0f);
    int64_t ranges = (2048 + (N + 255) / 256 - 1) / ((N + 255) / 256);
    int64_t rpb = (K + ranges - 1) / ranges;
    if (rpb < 32) rpb = 32;
    ranges = (K + rpb - 1) / rpb;
    if (ranges > 65535) { ranges = 65535; rpb = (K + ranges - 1) / ranges; }
    hipLaunchKernelGGL(fold_absmax_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)ranges), dim3(256), 0, st,
                       W, ldw, row_mult, col_div, (int)K, (int)N, col_scale, (int)rpb);
    const dim3 qgrid((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64));
    if (fp8) hipLaunchKernelGGL(fold_quant_kernel<true>, qgrid, dim3(256), 0, st, W, ldw, row_mult, col_div, (int)K, (int)N, col_scale, Wt, ldwt);
    else hipLaunchKernelGGL(fold_quant_kernel<false>, qgrid, dim3(256), 0, st, W, ldw, row_mult, col_div, (int)K, (int)N, col_scale, Wt, ldwt);
    hipLaunchKernelGGL(amax_to_scale_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, col_scale, (int)N, fp8 ? 448.0f : 127.0f);
    return hero_launch_status();
}
}  // namespace

extern "C" hero_status hero_weight_fold_quant(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                              int64_t K, int64_t N, int8_t* Wt, int64_t ldwt, float* col_scale, void* stream) {
    return weight_fold_quant_entry(W, ldw, row_mult, col_div, K, N, Wt, ldwt, col_scale, false, stream);
}

extern "C" hero_status hero_weight_fold_quant_fp8(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                                  int64_t K, int64_t N, void* Wt, int64_t ldwt, float* col_scale, void* stream) {
    return weight_fold_quant_entry(W, ldw, row_mult, col_div, K, N, (int8_t*)Wt, ldwt, col_scale, true, stream);
}
