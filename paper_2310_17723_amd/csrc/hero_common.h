// Shared device/host helpers of libhero (gfx950 only).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/hero.h"
#include "../../include/hero_debug.h"

#define HERO_WAVE 64

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

static inline bool hero_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// library-internal: 16-bit operands (dt = HERO_BF16 / HERO_F16) through the persistent GEMM kernels (int8_gemm.hip)
hero_status hero_hp_gemm_large(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                               const float* bias, const void* residual, int64_t ldr, int gelu,
                               void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, hipStream_t st, int tile);

static inline hero_status hero_launch_status() {
    return hipGetLastError() == hipSuccess ? HERO_OK : HERO_ERR_LAUNCH;
}

// ---- internal to the library (not part of the C ABI): the GeMM^quant entry points with a hint for callers that know
// what their chain reads next (hero_layer_fwd: the next module's weight matrix).  The large-problem kernels request
// that memory while they run, so that it waits in the cache hierarchy when the next kernel starts; the other kernels
// ignore the hint; no result depends on it.  Defined in int8_gemm.hip.
hero_status hero_int8_gemm_prefetching(const int8_t* A, int64_t lda, const float* a_row_scale,
                                       const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                       const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                       hero_epilogue epi, const float* out_col_scale,
                                       void* C, hero_dtype c_dt, int64_t ldc,
                                       int64_t M, int64_t N, int64_t K,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       const void* prefetch, size_t prefetch_bytes);

hero_status hero_fp8_gemm_prefetching(const void* A, int64_t lda, const float* a_row_scale,
                                      const void* Bt, int64_t ldb, const float* b_col_scale,
                                      const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                      hero_epilogue epi, const float* out_col_scale,
                                      void* C, hero_dtype c_dt, int64_t ldc,
                                      int64_t M, int64_t N, int64_t K, void* stream,
                                      const void* prefetch, size_t prefetch_bytes);

// ---- 16-bit float storage (round to nearest even) -------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
// v_cvt_pk_bf16_f32 (round to nearest even), one instruction for two values
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    const v2f v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    return (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)f);
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
    // The value is first rounded to fp32 and then to fp16.  The empty asm keeps the
    // compiler from merging a preceding multiply/fma with the conversion into one
    // mixed-precision instruction, which would round only once.
    asm volatile("" : "+v"(f));
    return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)f);      // v_cvt_f16_f32: RNE
}
template <int DT> __device__ __forceinline__ float hp_to_f32(uint32_t h) {
    return DT == HERO_BF16 ? bf16_bits_to_f32(h) : f16_bits_to_f32(h);
}
template <int DT> __device__ __forceinline__ uint32_t f32_to_hp(float f) {
    return DT == HERO_BF16 ? f32_to_bf16_bits(f) : f32_to_f16_bits(f);
}
// two values -> one dword of 16-bit floats (lo in bits 0..15)
template <int DT> __device__ __forceinline__ uint32_t pack2_hp(float lo, float hi) {
    if constexpr (DT == HERO_BF16) return f32x2_to_bf16x2(lo, hi);
    else return f32_to_f16_bits(lo) | (f32_to_f16_bits(hi) << 16);
}

// ---- the quantization primitive ---------------------------------------------------------
// code = sat_[-127,127](rne(x / s)) with IEEE fp32 division (never a reciprocal multiply).
__device__ __forceinline__ int quant_code_div(float x, float s) {
    float q = __builtin_rintf(__fdiv_rn(x, s));
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}
// sat(rne(y)) for an already scaled value.
__device__ __forceinline__ int round_sat_i8(float y) {
    float q = __builtin_rintf(y);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}
__device__ __forceinline__ uint32_t pack4_i8(int a, int b, int c, int d) {
    return (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8) | ((uint32_t)(c & 0xff) << 16) | ((uint32_t)d << 24);
}
// Round-half-even + two's-complement byte in ONE add: for |y| < 2^22 the fp32 sum y + 1.5*2^23 has
// ulp 1, so the adder rounds y to the nearest integer (ties to even) and the low byte of the sum's
// bit pattern is that integer mod 256.  Callers clamp y to the code range first (clamping before
// or after rounding is the same thing because the bounds are integers).
__device__ __forceinline__ uint32_t rne_low_byte(float y) { return __float_as_uint(y + 12582912.0f); }
// low bytes of four such sums -> one dword (v_perm_b32 x2 + v_or)
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3) {
    return __builtin_amdgcn_perm(r1, r0, 0x0c0c0400u) | __builtin_amdgcn_perm(r3, r2, 0x04000c0cu);
}
// four already-scaled values -> sat_[-127,127](rne(.)) packed as int8
__device__ __forceinline__ uint32_t quant4_sat(float y0, float y1, float y2, float y3) {
    return pack_low_bytes(rne_low_byte(__builtin_amdgcn_fmed3f(y0, -127.0f, 127.0f)),
                          rne_low_byte(__builtin_amdgcn_fmed3f(y1, -127.0f, 127.0f)),
                          rne_low_byte(__builtin_amdgcn_fmed3f(y2, -127.0f, 127.0f)),
                          rne_low_byte(__builtin_amdgcn_fmed3f(y3, -127.0f, 127.0f)));
}
// four fp32 values -> four OCP E4M3 bytes (round to nearest even), saturated to +-448
__device__ __forceinline__ uint32_t fp8x4_sat(float y0, float y1, float y2, float y3) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(y0, -448.0f, 448.0f), __builtin_amdgcn_fmed3f(y1, -448.0f, 448.0f), 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(y2, -448.0f, 448.0f), __builtin_amdgcn_fmed3f(y3, -448.0f, 448.0f), w, true);
    return (uint32_t)w;
}
// E4M3 x E4M3 at the full matrix rate: v_mfma_f32_32x32x64_f8f6f4, K = 64 per instruction, each lane half carries
// 32 bytes of its row (here: two 16-byte fragments side by side; any K grouping shared by both operands is the
// same contraction).  Unit scales.
__device__ __forceinline__ v16f mfma_wide_f8(v4i a_lo, v4i a_hi, v4i b_lo, v4i b_hi, v16f c) {
    const v8i a = {a_lo[0], a_lo[1], a_lo[2], a_lo[3], a_hi[0], a_hi[1], a_hi[2], a_hi[3]};
    const v8i b = {b_lo[0], b_lo[1], b_lo[2], b_lo[3], b_hi[0], b_hi[1], b_hi[2], b_hi[3]};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}
// erf-form GELU in fp32:  GELU(x) = x Phi(x) = max(x,0) - |x| Phi(-|x|).
// Phi(-z) = 2^P(z) with P a degree-6 polynomial: a weighted least-squares fit of log2 Phi(-z) on
// [0,6] (beyond 6, Phi(-z) < 1e-9 and z is clamped).  Evaluated in fp32 the absolute error of
// GELU is below 1.1e-7 for every x, i.e. the same order as the fp32 rounding of the erf form.
// Cost: 1 min, 6 fma, 1 exp2, 1 max, 1 fma.
__device__ __forceinline__ float gelu_erf(float x) {
    const float z = fminf(fabsf(x), 6.0f);
    float p = 3.309558087e-05f;
    p = fmaf(p, z, -7.692443905e-04f);
    p = fmaf(p, z, 8.080800064e-03f);
    p = fmaf(p, z, -5.341223627e-02f);
    p = fmaf(p, z, -4.587708712e-01f);
    p = fmaf(p, z, -1.151201725e+00f);
    p = fmaf(p, z, -9.999930859e-01f);
    const float q = __builtin_amdgcn_exp2f(p);          // Phi(-|x|)
    return fmaf(-fabsf(x), q, fmaxf(x, 0.0f));
}

// ---- wave reductions (64 lanes) ---------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
