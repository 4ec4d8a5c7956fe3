// CPU oracle for the ZeroQuant-HERO W8A8 layer operators.
//
// TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and
// the benchmark's cpu_baseline leg may build, load or call this file.  It shares no
// code, header, table or helper with the HIP library; every routine is the paper's
// definition written out in the plainest way (one loop nest per equation, fp64 for
// LayerNorm / softmax / GELU, exact integers for the contractions), so that it can be
// checked against the paper by eye.  All pointers are HOST pointers.
//
// Conventions (paper Sec. 2.1 only says "symmetric uniform INT8"; the rest is this
// build's reading, listed with its reasons in the design document):
//   * codes in [-127,127]; round half to even; IEEE fp32 division by the scale;
//   * dynamic scale = absmax / 127.0f; an all-zero row gets scale 1.0f;
//   * softmax codes are unsigned 0..255 with zero-point 0 (Sec. 2.2.2: softmax
//     output is "asymmetric" because it has no negative values).
//
// Parity pins live in tests/test_oracle_*.py (brute force, closed forms, invariants,
// numpy/scipy/torch library routines).  No function here is "parity unpinned".

#include <cmath>
#include <limits>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

enum { ORC_I8 = 0, ORC_U8 = 1, ORC_I32 = 2, ORC_F16 = 3, ORC_BF16 = 4, ORC_F32 = 5, ORC_F8 = 6 };
enum { ORC_EPI_RAW_I32 = 0, ORC_EPI_DEQUANT = 1, ORC_EPI_DEQUANT_GELU = 2,
       ORC_EPI_REQUANT = 3, ORC_EPI_GELU_REQUANT = 4 };
enum { ORC_MASK_NONE = 0, ORC_MASK_PADDING = 1, ORC_MASK_CAUSAL = 2 };

// ---------------------------------------------------------------------------------
// 16-bit float formats (storage only).  Round to nearest, ties to even.
// ---------------------------------------------------------------------------------
static inline uint32_t f32_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
static inline float bits_f32(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

uint16_t orc_f32_to_bf16(float f) {
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}
float orc_bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

uint16_t orc_f32_to_f16(float f) {
    // Through the exact value: find the nearest binary16 by scaling into an integer
    // number of half-precision ulps and rounding that integer half-to-even in fp64.
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    double a = std::fabs((double)f);
    if (std::isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);        // rounds to infinity
    if (a < std::ldexp(1.0, -14)) {                              // subnormal: ulp = 2^-24
        double n = std::nearbyint(a * std::ldexp(1.0, 24));      // 0..1024
        return (uint16_t)(sign | (uint16_t)n);                   // 1024 == smallest normal
    }
    int e; std::frexp(a, &e);                                    // a = m * 2^e, m in [0.5,1)
    int E = e - 1;                                               // a in [2^E, 2^(E+1))
    double n = std::nearbyint(a * std::ldexp(1.0, 10 - E));      // 1024..2048
    if (n >= 2048.0) { n = 1024.0; E += 1; }
    return (uint16_t)(sign | (uint16_t)(((E + 15) << 10) + ((int)n - 1024)));
}
float orc_f16_to_f32(uint16_t h) {
    int s = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    double v;
    if (e == 0) v = std::ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = std::ldexp((double)(m + 1024), e - 25);
    return (float)(s ? -v : v);
}

void orc_f32_to_bf16_n(const float* x, int64_t n, uint16_t* y) { for (int64_t i = 0; i < n; ++i) y[i] = orc_f32_to_bf16(x[i]); }
void orc_f32_to_f16_n(const float* x, int64_t n, uint16_t* y) { for (int64_t i = 0; i < n; ++i) y[i] = orc_f32_to_f16(x[i]); }
void orc_f16_to_f32_n(const uint16_t* x, int64_t n, float* y) { for (int64_t i = 0; i < n; ++i) y[i] = orc_f16_to_f32(x[i]); }

static inline float load_hp(const void* p, int dt, int64_t idx) {
    if (dt == ORC_BF16) return orc_bf16_to_f32(((const uint16_t*)p)[idx]);
    if (dt == ORC_F16) return orc_f16_to_f32(((const uint16_t*)p)[idx]);
    return ((const float*)p)[idx];
}
static inline void store_hp(void* p, int dt, int64_t idx, float v) {
    if (dt == ORC_BF16) ((uint16_t*)p)[idx] = orc_f32_to_bf16(v);
    else if (dt == ORC_F16) ((uint16_t*)p)[idx] = orc_f32_to_f16(v);
    else ((float*)p)[idx] = v;
}

// ---------------------------------------------------------------------------------
// O1.  The quantization primitive (Sec. 2.1, "symmetric uniform INT8").
// ---------------------------------------------------------------------------------
static inline int8_t sat_i8(float r) {          // r already rounded to an integer value
    if (r > 127.0f) return 127;
    if (r < -127.0f) return -127;
    return (int8_t)r;
}
static inline int8_t quant_code(float x, float s) {
    volatile float qf = x / s;                  // IEEE fp32 division, kept in fp32
    return sat_i8(std::nearbyintf(qf));         // default rounding mode: half to even
}
static inline float dyn_scale(float absmax) {
    if (absmax == 0.0f) return 1.0f;
    volatile float s = absmax / 127.0f;
    return s;
}

// Token-wise quantization (TWQ, Sec. 2.1): X = S_x X_int8, S_x in R^{n x 1}, computed
// on the fly from each row's absolute maximum.
void orc_quant_twq(const float* x, int64_t M, int64_t D, int8_t* q, float* s) {
    for (int64_t i = 0; i < M; ++i) {
        float amax = 0.0f;
        for (int64_t j = 0; j < D; ++j) amax = std::max(amax, std::fabs(x[i * D + j]));
        float sc = dyn_scale(amax);
        s[i] = sc;
        for (int64_t j = 0; j < D; ++j) q[i * D + j] = quant_code(x[i * D + j], sc);
    }
}

// Feature-wise (FWQ, S_x in R^{1 x d}) and static (SQ, scalar S_x) quantization with
// calibrated scales (Sec. 2.1).  col_scale == NULL selects the scalar.
void orc_quant_static(const float* x, int64_t M, int64_t D, const float* col_scale,
                      float scalar_scale, int8_t* q) {
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < D; ++j)
            q[i * D + j] = quant_code(x[i * D + j], col_scale ? col_scale[j] : scalar_scale);
}

// O2.  Column-wise weight quantization (Sec. 2.1: W = W_int8 Diag(S_w), S_w in
// R^{1 x m}).  W is the mathematical [K][N] matrix, row-major; the codes are written
// "column-major", i.e. Wt[n][k], each output column's K values contiguous.
void orc_weight_quant(const float* W, int64_t K, int64_t N, int8_t* Wt, float* s) {
    for (int64_t n = 0; n < N; ++n) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) amax = std::max(amax, std::fabs(W[k * N + n]));
        float sc = dyn_scale(amax);
        s[n] = sc;
        for (int64_t k = 0; k < K; ++k) Wt[n * K + k] = quant_code(W[k * N + n], sc);
    }
}

// ---------------------------------------------------------------------------------
// O3.  The integer contraction  acc[i][j] = sum_k A[i][k] * Bt[j][k].
// ---------------------------------------------------------------------------------
void orc_gemm_i32(const int8_t* A, int64_t lda, const int8_t* Bt, int64_t ldb,
                  int64_t M, int64_t N, int64_t K, int32_t* C) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)A[i * lda + k] * (int32_t)Bt[j * ldb + k];
            C[i * N + j] = acc;
        }
}
// Same sum carried in 64 bits: shows that the 32-bit one never wrapped.
void orc_gemm_i64(const int8_t* A, int64_t lda, const int8_t* Bt, int64_t ldb,
                  int64_t M, int64_t N, int64_t K, int64_t* C) {
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)A[i * lda + k] * (int64_t)Bt[j * ldb + k];
            C[i * N + j] = acc;
        }
}

// GELU, exact erf form (the paper only names "GELU", Sec. 2.2.3), in fp64.
double orc_gelu(double x) { return 0.5 * x * (1.0 + std::erf(x / std::sqrt(2.0))); }

// ---------------------------------------------------------------------------------
// O4.  GeMM^quant: INT8 GEMM with dequantization and the static FWQ/SQ scales fused
// behind it (Sec. 2.2.2, the paragraph on fusing dequantization and scaling factors
// into the INT8 GeMM, and the "Round(GeMM^quant(...))" equation; Sec. 2.2.3 for
// GELU^quant).  fp32 arithmetic in one fixed order:
//     t = float(acc);  t = t * a_row_scale[i];  y = fma(t, b_col_scale[j], bias[j])
// DEQUANT:       y (+ residual) -> bf16/f16/f32
// DEQUANT_GELU:  GELU(y) -> bf16/f16/f32
// REQUANT:       sat(rne(y)) -> i8           (the folded scale makes this a bare Round)
// GELU_REQUANT:  sat(rne(GELU(y) / out_col_scale[j])) -> i8
// Returns 0, or -1 on an invalid combination.
// ---------------------------------------------------------------------------------
int orc_int8_gemm(const int8_t* A, int64_t lda, const float* a_row_scale,
                  const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                  const float* bias, const void* residual, int res_dt, int64_t ldr,
                  int epi, const float* out_col_scale,
                  void* C, int c_dt, int64_t ldc, int64_t M, int64_t N, int64_t K) {
    if (epi == ORC_EPI_RAW_I32 && c_dt != ORC_I32) return -1;
    if ((epi == ORC_EPI_REQUANT || epi == ORC_EPI_GELU_REQUANT) && c_dt != ORC_I8) return -1;
    if ((epi == ORC_EPI_DEQUANT || epi == ORC_EPI_DEQUANT_GELU) &&
        !(c_dt == ORC_F16 || c_dt == ORC_BF16 || c_dt == ORC_F32)) return -1;
    if (epi == ORC_EPI_GELU_REQUANT && !out_col_scale) return -1;
    if (epi != ORC_EPI_RAW_I32 && !b_col_scale) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)A[i * lda + k] * (int32_t)Bt[j * ldb + k];
            if (epi == ORC_EPI_RAW_I32) { ((int32_t*)C)[i * ldc + j] = acc; continue; }
            volatile float t = (float)acc;
            if (a_row_scale) t = t * a_row_scale[i];
            volatile float y = std::fmaf(t, b_col_scale[j], bias ? bias[j] : 0.0f);
            switch (epi) {
            case ORC_EPI_DEQUANT: {
                float o = y;
                if (residual) { volatile float r = y + load_hp(residual, res_dt, i * ldr + j); o = r; }
                store_hp(C, c_dt, i * ldc + j, o);
                break; }
            case ORC_EPI_DEQUANT_GELU:
                store_hp(C, c_dt, i * ldc + j, (float)orc_gelu((double)y));
                break;
            case ORC_EPI_REQUANT:
                ((int8_t*)C)[i * ldc + j] = sat_i8(std::nearbyintf(y));
                break;
            case ORC_EPI_GELU_REQUANT:
                ((int8_t*)C)[i * ldc + j] = quant_code((float)orc_gelu((double)y), out_col_scale[j]);
                break;
            }
        }
    return 0;
}

// ---------------------------------------------------------------------------------
// O4f.  The FP8 variant (Sec. 2.1: the method "also works for other 8-bit precision formats, like
// FP8").  Format: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals; no
// infinities; largest finite value 448; the all-ones pattern 0x7F / 0xFF is NaN), the 8-bit float
// the gfx950 matrix cores multiply.  Conventions mirror the INT8 ones: round to nearest even,
// SATURATE to +-448, token-wise scale = absmax / 448, static scales folded as before.
//   orc_e4m3_to_f32 / orc_f32_to_e4m3: the format itself.
//   orc_quant_twq_fp8: per row  s = max|x| / 448 (1 for a zero row);  q = e4m3(x / s)  (IEEE fp32 quotient).
//   orc_fp8_gemm: acc = sum_k A[i][k] * Bt[j][k] with every product exact and the sum carried in fp64
//     (the definition: the exact sum, rounded once); t = float(acc) and then the same fp32 epilogue
//     as O4, with e4m3(.) in place of sat(rne(.)) for the 8-bit outputs.
// ---------------------------------------------------------------------------------
float orc_e4m3_to_f32(uint8_t c) {
    const int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    float v;
    if (e == 15 && m == 7) return std::numeric_limits<float>::quiet_NaN();
    if (e == 0) v = std::ldexp((float)m, -9);                       // subnormal: m/8 * 2^-6
    else v = std::ldexp(1.0f + (float)m / 8.0f, e - 7);
    return sign ? -v : v;
}
uint8_t orc_f32_to_e4m3(float x) {
    if (std::isnan(x)) return 0x7F;
    const uint8_t sign = std::signbit(x) ? 0x80 : 0x00;
    const double a = std::fabs((double)x);
    if (a >= 464.0) return sign | 0x7E;                             // beyond the midpoint above 448: saturate
    if (a < std::ldexp(1.0, -6)) {                                  // subnormal range (may round up to 2^-6 = code 8)
        const int q = (int)std::nearbyint(a * 512.0);
        return sign | (uint8_t)q;
    }
    int e2;
    const double fr = std::frexp(a, &e2);                           // a = fr * 2^e2, fr in [0.5, 1)
    int e = e2 - 1;
    int q = (int)std::nearbyint((fr * 2.0 - 1.0) * 8.0);            // ties to even in the default rounding mode
    if (q == 8) { q = 0; ++e; }
    if (e > 8 || (e == 8 && q > 6)) return sign | 0x7E;
    return sign | (uint8_t)(((e + 7) << 3) | q);
}
void orc_e4m3_to_f32_n(const uint8_t* c, int64_t n, float* out) { for (int64_t i = 0; i < n; ++i) out[i] = orc_e4m3_to_f32(c[i]); }
void orc_f32_to_e4m3_n(const float* x, int64_t n, uint8_t* out) { for (int64_t i = 0; i < n; ++i) out[i] = orc_f32_to_e4m3(x[i]); }

void orc_quant_twq_fp8(const float* x, int64_t M, int64_t D, uint8_t* q, float* s) {
    for (int64_t i = 0; i < M; ++i) {
        float amax = 0.0f;
        for (int64_t j = 0; j < D; ++j) amax = std::max(amax, std::fabs(x[i * D + j]));
        volatile float sc = amax == 0.0f ? 1.0f : amax / 448.0f;
        s[i] = sc;
        for (int64_t j = 0; j < D; ++j) { volatile float t = x[i * D + j] / sc; q[i * D + j] = orc_f32_to_e4m3(t); }
    }
}

int orc_fp8_gemm(const uint8_t* A, int64_t lda, const float* a_row_scale,
                 const uint8_t* Bt, int64_t ldb, const float* b_col_scale,
                 const float* bias, const void* residual, int res_dt, int64_t ldr,
                 int epi, const float* out_col_scale,
                 void* C, int c_dt, int64_t ldc, int64_t M, int64_t N, int64_t K) {
    if (epi == ORC_EPI_RAW_I32) return -1;
    if ((epi == ORC_EPI_REQUANT || epi == ORC_EPI_GELU_REQUANT) && c_dt != ORC_F8) return -1;
    if ((epi == ORC_EPI_DEQUANT || epi == ORC_EPI_DEQUANT_GELU) &&
        !(c_dt == ORC_F16 || c_dt == ORC_BF16 || c_dt == ORC_F32)) return -1;
    if (epi == ORC_EPI_GELU_REQUANT && !out_col_scale) return -1;
    if (!b_col_scale) return -1;
    float lut[256];
    for (int c = 0; c < 256; ++c) lut[c] = orc_e4m3_to_f32((uint8_t)c);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += (double)lut[A[i * lda + k]] * (double)lut[Bt[j * ldb + k]];
            volatile float t = (float)acc;
            if (a_row_scale) t = t * a_row_scale[i];
            volatile float y = std::fmaf(t, b_col_scale[j], bias ? bias[j] : 0.0f);
            switch (epi) {
            case ORC_EPI_DEQUANT: {
                float o = y;
                if (residual) { volatile float r = y + load_hp(residual, res_dt, i * ldr + j); o = r; }
                store_hp(C, c_dt, i * ldc + j, o);
                break; }
            case ORC_EPI_DEQUANT_GELU:
                store_hp(C, c_dt, i * ldc + j, (float)orc_gelu((double)y));
                break;
            case ORC_EPI_REQUANT:
                ((uint8_t*)C)[i * ldc + j] = orc_f32_to_e4m3(y);
                break;
            case ORC_EPI_GELU_REQUANT: {
                volatile float gq = (float)orc_gelu((double)y) / out_col_scale[j];
                ((uint8_t*)C)[i * ldc + j] = orc_f32_to_e4m3(gq);
                break; }
            }
        }
    return 0;
}

// ---------------------------------------------------------------------------------
// O5.  LN^quant (Sec. 2.2.2 last equation of the quantized attention flow and the
// paragraph after the W_o fold; Sec. 2.2.3 last equation): LayerNorm of the SUM of its
// inputs, output token-wise quantized.
//   x: i8 [M,D] with a per-row (TWQ) scale, or bf16/f16/f32 without a scale
//   r: optional second addend: i8 with a per-column (FWQ) scale, or bf16/f16/f32
//   gamma == NULL: no LayerNorm, the sum itself is quantized per token
// Sum, mean, biased variance and the normalised value in fp64; the result is cast to
// fp32 once and the TWQ primitive runs in fp32.
// ---------------------------------------------------------------------------------
// y_q_dt selects the 8-bit format of the output (Sec. 2.1: INT8 or FP8): ORC_I8 as above, ORC_F8 for
// token-wise E4M3 codes with scale = max|y| / 448.
static int ln_quant_impl(const void* x, int x_dt, const float* x_row_scale,
                         const void* r, int r_dt, const float* r_col_scale,
                         const float* gamma, const float* beta, float eps,
                         int64_t M, int64_t D,
                         void* y_q_, int y_q_dt, float* y_scale, void* y_hp, int y_hp_dt) {
    int8_t* y_q = (int8_t*)y_q_;
    // 8-bit addends: INT8 codes or E4M3 codes (ORC_F8), each times its scale
    const bool x8 = x_dt == ORC_I8 || x_dt == ORC_F8, r8 = r && (r_dt == ORC_I8 || r_dt == ORC_F8);
    if (x8 && !x_row_scale) return -1;
    if (r8 && !r_col_scale) return -1;
    auto code = [](const void* p, int dt, int64_t idx) -> double {
        return dt == ORC_I8 ? (double)((const int8_t*)p)[idx] : (double)orc_e4m3_to_f32(((const uint8_t*)p)[idx]);
    };
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        std::vector<double> s(D);
        std::vector<float> y32(D);
        for (int64_t j = 0; j < D; ++j) {
            double v = x8 ? (double)x_row_scale[i] * code(x, x_dt, i * D + j) : (double)load_hp(x, x_dt, i * D + j);
            if (r) v += r8 ? (double)r_col_scale[j] * code(r, r_dt, i * D + j) : (double)load_hp(r, r_dt, i * D + j);
            s[j] = v;
        }
        if (gamma) {
            double mu = 0.0;
            for (int64_t j = 0; j < D; ++j) mu += s[j];
            mu /= (double)D;
            double var = 0.0;
            for (int64_t j = 0; j < D; ++j) var += (s[j] - mu) * (s[j] - mu);
            var /= (double)D;
            double rstd = 1.0 / std::sqrt(var + (double)eps);
            for (int64_t j = 0; j < D; ++j)
                y32[j] = (float)((s[j] - mu) * rstd * (double)gamma[j] + (beta ? (double)beta[j] : 0.0));
        } else {
            for (int64_t j = 0; j < D; ++j) y32[j] = (float)s[j];
        }
        float amax = 0.0f;
        for (int64_t j = 0; j < D; ++j) amax = std::max(amax, std::fabs(y32[j]));
        if (y_q_dt == ORC_F8) {
            volatile float scf = amax == 0.0f ? 1.0f : amax / 448.0f;
            y_scale[i] = scf;
            for (int64_t j = 0; j < D; ++j) {
                volatile float t = y32[j] / scf;
                ((uint8_t*)y_q_)[i * D + j] = orc_f32_to_e4m3(t);
                if (y_hp) store_hp(y_hp, y_hp_dt, i * D + j, y32[j]);
            }
            continue;
        }
        float sc = dyn_scale(amax);
        y_scale[i] = sc;
        for (int64_t j = 0; j < D; ++j) {
            y_q[i * D + j] = quant_code(y32[j], sc);
            if (y_hp) store_hp(y_hp, y_hp_dt, i * D + j, y32[j]);
        }
    }
    return 0;
}

int orc_ln_quant(const void* x, int x_dt, const float* x_row_scale,
                 const void* r, int r_dt, const float* r_col_scale,
                 const float* gamma, const float* beta, float eps,
                 int64_t M, int64_t D,
                 int8_t* y_q, float* y_scale, void* y_hp, int y_hp_dt) {
    return ln_quant_impl(x, x_dt, x_row_scale, r, r_dt, r_col_scale, gamma, beta, eps, M, D, y_q, ORC_I8, y_scale, y_hp, y_hp_dt);
}

// LN^quant with a token-wise FP8 (E4M3) output: the same y, scale = max|y| / 448, code = e4m3(y / scale).
int orc_ln_quant_fp8(const void* x, int x_dt, const float* x_row_scale,
                     const void* r, int r_dt, const float* r_col_scale,
                     const float* gamma, const float* beta, float eps,
                     int64_t M, int64_t D,
                     uint8_t* y_q, float* y_scale, void* y_hp, int y_hp_dt) {
    return ln_quant_impl(x, x_dt, x_row_scale, r, r_dt, r_col_scale, gamma, beta, eps, M, D, y_q, ORC_F8, y_scale, y_hp, y_hp_dt);
}

// ---------------------------------------------------------------------------------
// O5b.  Embedding LN^quant (Sec. 2.2.1: S_emb X_emb,int8 = LN^quant(S_xt X_t,int8, X_p, X_s)).
// Per token i:  h[j] = S_xt[tok_ids[i]] * X_t,int8[tok_ids[i]][j] + X_p[pos_ids[i]][j]
//                      (+ X_s[type_ids[i]][j] when a type table is given)
// with the token table in INT8 codes + one TWQ scale per table row and the position / type tables in
// bf16 / f16 / f32; LayerNorm of h over j and the TWQ quantization exactly as in O5 (sum, mean,
// biased variance and the normalised value in fp64, one cast to fp32, TWQ primitive in fp32).
// Returns -2 when an index is out of its table.
// ---------------------------------------------------------------------------------
int orc_embed_ln_quant(const int32_t* tok_ids, const int32_t* pos_ids, const int32_t* type_ids,
                       const int8_t* tok_table, const float* tok_scale, int64_t V,
                       const void* pos_table, int64_t P, const void* type_table, int64_t NT, int pt_dt,
                       const float* gamma, const float* beta, float eps,
                       int64_t T, int64_t D, int8_t* y_q, float* y_scale) {
    if (!tok_ids || !pos_ids || !tok_table || !tok_scale || !pos_table || !gamma) return -1;
    if (type_table && !type_ids) return -1;
    for (int64_t i = 0; i < T; ++i) {
        if (tok_ids[i] < 0 || tok_ids[i] >= V || pos_ids[i] < 0 || pos_ids[i] >= P) return -2;
        if (type_table && (type_ids[i] < 0 || type_ids[i] >= NT)) return -2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        std::vector<double> s(D);
        const int64_t tk = tok_ids[i], ps = pos_ids[i], ty = type_table ? type_ids[i] : 0;
        for (int64_t j = 0; j < D; ++j) {
            double v = (double)tok_scale[tk] * (double)tok_table[tk * D + j];
            v += (double)load_hp(pos_table, pt_dt, ps * D + j);
            if (type_table) v += (double)load_hp(type_table, pt_dt, ty * D + j);
            s[j] = v;
        }
        double mu = 0.0;
        for (int64_t j = 0; j < D; ++j) mu += s[j];
        mu /= (double)D;
        double var = 0.0;
        for (int64_t j = 0; j < D; ++j) var += (s[j] - mu) * (s[j] - mu);
        var /= (double)D;
        const double rstd = 1.0 / std::sqrt(var + (double)eps);
        std::vector<float> y32(D);
        float amax = 0.0f;
        for (int64_t j = 0; j < D; ++j) {
            y32[j] = (float)((s[j] - mu) * rstd * (double)gamma[j] + (beta ? (double)beta[j] : 0.0));
            amax = std::max(amax, std::fabs(y32[j]));
        }
        const float sc = dyn_scale(amax);
        y_scale[i] = sc;
        for (int64_t j = 0; j < D; ++j) y_q[i * D + j] = quant_code(y32[j], sc);
    }
    return 0;
}

// ---------------------------------------------------------------------------------
// O6.  INT8 attention (Sec. 2.2.2, quantized flow, lines A, Softmax^quant, X_attn;
// and d~ = S_q S_k / sqrt(d)).  Per (batch, head):
//   acc_qk[i][k] exact;  a = float(acc_qk) * d~  (fp32, A is never quantized);
//   keys outside the mask are left out;  p = softmax(a) in fp64;
//   P_u8 = sat_[0,255](rne(float(p) / S_p));  acc_pv[i][e] = sum_k P_u8 * V[k][e] exact;
//   INT8 out:  sat(rne(float(acc_pv) * c[j])),  c[j] = S_p S_v / S_attn[j],  j = h*Dh+e
//   bf16/f16/f32 out:  float(acc_pv) * c[0]     (c[0] = S_p S_v)
// Strides are in elements, ordered (batch, position, head, channel).
// Mask: key k is visible to query i iff  k < kv_len[b] (when kv_len != NULL) and, for
// CAUSAL, k <= i + (kvlen_b - Sq), i.e. the last query sees the last valid key.
// With the PADDING mask in self-attention (Sq == Skv) the positions i >= kv_len[b] are padding as
// queries too: they see no key.  A query with no visible key outputs 0.  p_dump (optional)
// receives the codes [B,H,Sq,Skv].
// ---------------------------------------------------------------------------------
int orc_int8_attn(const int8_t* q, const int64_t* qs, const int8_t* k, const int64_t* ks,
                  const int8_t* v, const int64_t* vs,
                  int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                  float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                  int mask, const int32_t* kv_len,
                  void* out, int out_dt, int64_t ldo, uint8_t* p_dump) {
    if (out_dt == ORC_I8 && out_scale_is_scalar == 0 && !out_col_scale) return -1;
    if (mask == ORC_MASK_PADDING && !kv_len) return -1;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            int64_t len = kv_len ? std::min<int64_t>(kv_len[b], Skv) : Skv;
            std::vector<float> a(Skv);
            std::vector<double> p(Skv);
            std::vector<int32_t> codes(Skv);
            for (int64_t i = 0; i < Sq; ++i) {
                int64_t last = len - 1;                              // last visible key
                if (mask == ORC_MASK_CAUSAL) last = std::min<int64_t>(last, i + (len - Sq));
                if (mask == ORC_MASK_PADDING && Sq == Skv && i >= len) last = -1;   // a padded position asks nothing
                int64_t nvis = last + 1;
                const int8_t* qi = q + b * qs[0] + i * qs[1] + h * qs[2];
                for (int64_t kk = 0; kk < nvis; ++kk) {
                    const int8_t* kr = k + b * ks[0] + kk * ks[1] + h * ks[2];
                    int32_t acc = 0;
                    for (int64_t e = 0; e < Dh; ++e) acc += (int32_t)qi[e * qs[3]] * (int32_t)kr[e * ks[3]];
                    volatile float t = (float)acc * qk_scale;
                    a[kk] = t;
                }
                for (int64_t kk = 0; kk < Skv; ++kk) codes[kk] = 0;
                if (nvis > 0) {
                    double m = a[0];
                    for (int64_t kk = 1; kk < nvis; ++kk) m = std::max(m, (double)a[kk]);
                    double l = 0.0;
                    for (int64_t kk = 0; kk < nvis; ++kk) { p[kk] = std::exp((double)a[kk] - m); l += p[kk]; }
                    for (int64_t kk = 0; kk < nvis; ++kk) {
                        volatile float pf = (float)(p[kk] / l);
                        volatile float qf = pf / p_scale;
                        float rr = std::nearbyintf(qf);
                        codes[kk] = rr > 255.0f ? 255 : (rr < 0.0f ? 0 : (int32_t)rr);
                    }
                }
                if (p_dump)
                    for (int64_t kk = 0; kk < Skv; ++kk)
                        p_dump[((b * H + h) * Sq + i) * Skv + kk] = (uint8_t)codes[kk];
                for (int64_t e = 0; e < Dh; ++e) {
                    int32_t acc = 0;
                    for (int64_t kk = 0; kk < nvis; ++kk)
                        acc += codes[kk] * (int32_t)v[b * vs[0] + kk * vs[1] + h * vs[2] + e * vs[3]];
                    int64_t j = h * Dh + e;
                    int64_t o = (b * Sq + i) * ldo + j;
                    float c = out_scale_is_scalar ? out_col_scale[0] : out_col_scale[j];
                    volatile float y = (float)acc * c;
                    if (out_dt == ORC_I8) ((int8_t*)out)[o] = sat_i8(std::nearbyintf(y));
                    else store_hp(out, out_dt, o, y);
                }
            }
        }
    return 0;
}

// ---------------------------------------------------------------------------------
// O6f.  FP8 attention: the quantized attention flow of Sec. 2.2.2 with E4M3 as the 8-bit format
// (Sec. 2.1).  The same operands, strides, masks and output scales as O6; q, k, v hold E4M3 bytes.
// Per (batch, head), query i, visible keys k:
//   a[k]  = float(sum_e q[i][e] k[k][e]) * d~        every product exact, the sum in fp64, rounded once
//   p     = softmax(a) in fp64
//   P_f8  = e4m3(float(p) / S_p)                     round to nearest even, saturating at 448; probabilities
//           are non-negative, so the codes use the positive half of the format and S_p = 1/448 gives p = 1
//           the largest code
//   acc[e] = sum_k P_f8[k] v[k][e]                   exact products, fp64 sum, rounded once to fp32
//   E4M3 out: e4m3(acc[e] * c[j]), c[j] = S_p S_v / S_attn[j];   16-bit / fp32 out: acc[e] * c[0]
// A query with no visible key outputs 0.  p_dump (optional) receives the codes [B,H,Sq,Skv].
// ---------------------------------------------------------------------------------
int orc_fp8_attn(const uint8_t* q, const int64_t* qs, const uint8_t* k, const int64_t* ks,
                 const uint8_t* v, const int64_t* vs,
                 int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                 float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                 int mask, const int32_t* kv_len,
                 void* out, int out_dt, int64_t ldo, uint8_t* p_dump) {
    if (!out_col_scale) return -1;
    if (mask == ORC_MASK_PADDING && !kv_len) return -1;
    if (out_dt != ORC_F8 && !out_scale_is_scalar) return -1;
    float lut[256];
    for (int c = 0; c < 256; ++c) lut[c] = orc_e4m3_to_f32((uint8_t)c);
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            const int64_t len = kv_len ? std::min<int64_t>(kv_len[b], Skv) : Skv;
            std::vector<float> a(Skv);
            std::vector<double> p(Skv);
            std::vector<uint8_t> codes(Skv);
            for (int64_t i = 0; i < Sq; ++i) {
                int64_t last = len - 1;
                if (mask == ORC_MASK_CAUSAL) last = std::min<int64_t>(last, i + (len - Sq));
                if (mask == ORC_MASK_PADDING && Sq == Skv && i >= len) last = -1;   // a padded position asks nothing
                const int64_t nvis = last + 1;
                const uint8_t* qi = q + b * qs[0] + i * qs[1] + h * qs[2];
                for (int64_t kk = 0; kk < nvis; ++kk) {
                    const uint8_t* kr = k + b * ks[0] + kk * ks[1] + h * ks[2];
                    double acc = 0.0;
                    for (int64_t e = 0; e < Dh; ++e) acc += (double)lut[qi[e * qs[3]]] * (double)lut[kr[e * ks[3]]];
                    volatile float t = (float)acc * qk_scale;
                    a[kk] = t;
                }
                for (int64_t kk = 0; kk < Skv; ++kk) codes[kk] = 0;
                if (nvis > 0) {
                    double m = a[0];
                    for (int64_t kk = 1; kk < nvis; ++kk) m = std::max(m, (double)a[kk]);
                    double l = 0.0;
                    for (int64_t kk = 0; kk < nvis; ++kk) { p[kk] = std::exp((double)a[kk] - m); l += p[kk]; }
                    for (int64_t kk = 0; kk < nvis; ++kk) {
                        volatile float pf = (float)(p[kk] / l);
                        volatile float qf = pf / p_scale;
                        codes[kk] = orc_f32_to_e4m3(qf);
                    }
                }
                if (p_dump)
                    for (int64_t kk = 0; kk < Skv; ++kk)
                        p_dump[((b * H + h) * Sq + i) * Skv + kk] = codes[kk];
                for (int64_t e = 0; e < Dh; ++e) {
                    double acc = 0.0;
                    for (int64_t kk = 0; kk < nvis; ++kk)
                        acc += (double)lut[codes[kk]] * (double)lut[v[b * vs[0] + kk * vs[1] + h * vs[2] + e * vs[3]]];
                    const int64_t j = h * Dh + e, o = (b * Sq + i) * ldo + j;
                    const float c = out_scale_is_scalar ? out_col_scale[0] : out_col_scale[j];
                    volatile float y = (float)acc * c;
                    if (out_dt == ORC_F8) ((uint8_t*)out)[o] = orc_f32_to_e4m3(y);
                    else store_hp(out, out_dt, o, y);
                }
            }
        }
    return 0;
}

// ---------------------------------------------------------------------------------
// O6b.  INT8 attention with an ONLINE Softmax^quant -- a variant, not the equation of Sec. 2.2.2:
// the probabilities are quantized BEFORE they are normalised, block by block, against the running row
// maximum, so one sweep over the keys suffices and the largest weight of a row always has code 255.
// The same operands, masks and output scales as orc_int8_attn; qk_scale is per head.
// Per (batch, head), query i, with the visible keys 0 .. nvis-1 cut into blocks of kv_block keys
// (block t = keys [t*kv_block, (t+1)*kv_block), aligned to key 0):
//   a[k]   = float(acc_qk[i][k]) * d~[h]                                  fp32, as in O6
//   m_t    = max(m_{t-1}, max_{k in t} a[k]),  m_{-1} = -inf              running maximum
//   c[k]   = sat_[0,255](rne(float(255 exp(a[k] - m_t))))                 unsigned codes, k in block t
//   O_t[e] = sum_{k in t} c[k] V[k][e],   L_t = sum_{k in t} c[k]          exact integers
//   O[e]   = sum_t exp(m_t - m_T) O_t[e],  L = sum_t exp(m_t - m_T) L_t    (T = last block; fp64)
//   X_attn = S_v O / L ;  out = sat(rne(float(O[e] / L * c[j] / S_p)))  with c[j] = S_p S_v / S_attn[j] as in
//   O6 (the caller passes the same c and S_p as for the two-pass operator: S_p cancels), or float(.) for a
//   16-bit output with c[0] = S_p S_v.  A query with no visible key outputs 0.
// c_dump (optional) receives the codes [B,H,Sq,Skv].
// ---------------------------------------------------------------------------------
int orc_int8_attn_online(const int8_t* q, const int64_t* qs, const int8_t* k, const int64_t* ks,
                         const int8_t* v, const int64_t* vs,
                         int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, int64_t kv_block,
                         const float* qk_scale_h, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                         int mask, const int32_t* kv_len,
                         void* out, int out_dt, int64_t ldo, uint8_t* c_dump) {
    if (out_dt == ORC_I8 && out_scale_is_scalar == 0 && !out_col_scale) return -1;
    if (mask == ORC_MASK_PADDING && !kv_len) return -1;
    if (kv_block <= 0 || !qk_scale_h) return -1;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            int64_t len = kv_len ? std::min<int64_t>(kv_len[b], Skv) : Skv;
            std::vector<float> a(Skv);
            std::vector<int32_t> codes(Skv);
            std::vector<double> O(Dh);
            for (int64_t i = 0; i < Sq; ++i) {
                int64_t last = len - 1;
                if (mask == ORC_MASK_CAUSAL) last = std::min<int64_t>(last, i + (len - Sq));
                if (mask == ORC_MASK_PADDING && Sq == Skv && i >= len) last = -1;   // a padded position asks nothing
                const int64_t nvis = last + 1;
                const int8_t* qi = q + b * qs[0] + i * qs[1] + h * qs[2];
                for (int64_t kk = 0; kk < nvis; ++kk) {
                    const int8_t* kr = k + b * ks[0] + kk * ks[1] + h * ks[2];
                    int32_t acc = 0;
                    for (int64_t e = 0; e < Dh; ++e) acc += (int32_t)qi[e * qs[3]] * (int32_t)kr[e * ks[3]];
                    volatile float t = (float)acc * qk_scale_h[h];
                    a[kk] = t;
                }
                for (int64_t kk = 0; kk < Skv; ++kk) codes[kk] = 0;
                for (int64_t e = 0; e < Dh; ++e) O[e] = 0.0;
                double L = 0.0, m = -INFINITY;
                for (int64_t k0 = 0; k0 < nvis; k0 += kv_block) {
                    const int64_t k1 = std::min(k0 + kv_block, nvis);
                    double mt = m;
                    for (int64_t kk = k0; kk < k1; ++kk) mt = std::max(mt, (double)a[kk]);
                    const double rescale = (m == -INFINITY) ? 0.0 : std::exp(m - mt);   // exp(m_{t-1} - m_t)
                    int64_t Lt = 0;
                    for (int64_t kk = k0; kk < k1; ++kk) {
                        volatile float w = (float)(255.0 * std::exp((double)a[kk] - mt));
                        float rr = std::nearbyintf(w);
                        codes[kk] = rr > 255.0f ? 255 : (rr < 0.0f ? 0 : (int32_t)rr);
                        Lt += codes[kk];
                    }
                    L = L * rescale + (double)Lt;
                    for (int64_t e = 0; e < Dh; ++e) {
                        int64_t Ot = 0;
                        for (int64_t kk = k0; kk < k1; ++kk)
                            Ot += (int64_t)codes[kk] * (int64_t)v[b * vs[0] + kk * vs[1] + h * vs[2] + e * vs[3]];
                        O[e] = O[e] * rescale + (double)Ot;
                    }
                    m = mt;
                }
                if (c_dump)
                    for (int64_t kk = 0; kk < Skv; ++kk)
                        c_dump[((b * H + h) * Sq + i) * Skv + kk] = (uint8_t)codes[kk];
                for (int64_t e = 0; e < Dh; ++e) {
                    const int64_t j = h * Dh + e;
                    const int64_t o = (b * Sq + i) * ldo + j;
                    const float c = out_scale_is_scalar ? out_col_scale[0] : out_col_scale[j];
                    volatile float y = nvis > 0 ? (float)(O[e] / L * (double)c / (double)p_scale) : 0.0f;
                    if (out_dt == ORC_I8) ((int8_t*)out)[o] = sat_i8(std::nearbyintf(y));
                    else store_hp(out, out_dt, o, y);
                }
            }
        }
    return 0;
}

// ---------------------------------------------------------------------------------
// BF16 side of a switched module (Sec. 2.3, Table 1: a module marked with a cross runs
// in FP16/BF16).  Operands are bf16 values; the sums are carried in fp64 and rounded
// to bf16 once at the end, so this is the value any correct fp32-accumulating kernel
// must approach.
//   C = act(A W + bias) (+ residual),  A [M,K] bf16, Wt [N][K] bf16, C bf16.
// ---------------------------------------------------------------------------------
// dt = ORC_BF16 or ORC_F16: the 16-bit type of operands, residual and result (Sec. 2.3: a switched module runs in
// FP16 / BF16).
int orc_hp_gemm(const uint16_t* A, int64_t lda, const uint16_t* Wt, int64_t ldb,
                const float* bias, const uint16_t* residual, int64_t ldr, int gelu,
                uint16_t* C, int64_t ldc, int64_t M, int64_t N, int64_t K, int dt) {
    if (dt != ORC_BF16 && dt != ORC_F16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t kk = 0; kk < K; ++kk)
                acc += (double)load_hp(A, dt, i * lda + kk) * (double)load_hp(Wt, dt, j * ldb + kk);
            if (bias) acc += (double)bias[j];
            if (gelu) acc = orc_gelu(acc);
            if (residual) acc += (double)load_hp(residual, dt, i * ldr + j);
            store_hp(C, dt, i * ldc + j, (float)acc);
        }
    return 0;
}
int orc_bf16_gemm(const uint16_t* A, int64_t lda, const uint16_t* Wt, int64_t ldb,
                  const float* bias, const uint16_t* residual, int64_t ldr, int gelu,
                  uint16_t* C, int64_t ldc, int64_t M, int64_t N, int64_t K) {
    return orc_hp_gemm(A, lda, Wt, ldb, bias, residual, ldr, gelu, C, ldc, M, N, K, ORC_BF16);
}

// 16-bit attention core: softmax(Q K^T * scale) V in fp64 on bf16 / f16 inputs, output in the same type.
// Same strides and mask rules as orc_int8_attn.
int orc_hp_attn(const uint16_t* q, const int64_t* qs, const uint16_t* k, const int64_t* ks,
                const uint16_t* v, const int64_t* vs,
                int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                int mask, const int32_t* kv_len, uint16_t* out, int64_t ldo, int dt) {
    if (dt != ORC_BF16 && dt != ORC_F16) return -1;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            int64_t len = kv_len ? std::min<int64_t>(kv_len[b], Skv) : Skv;
            std::vector<double> p(Skv);
            for (int64_t i = 0; i < Sq; ++i) {
                int64_t last = len - 1;
                if (mask == ORC_MASK_CAUSAL) last = std::min<int64_t>(last, i + (len - Sq));
                if (mask == ORC_MASK_PADDING && Sq == Skv && i >= len) last = -1;   // a padded position asks nothing
                int64_t nvis = last + 1;
                double m = -INFINITY;
                for (int64_t kk = 0; kk < nvis; ++kk) {
                    double acc = 0.0;
                    for (int64_t e = 0; e < Dh; ++e)
                        acc += (double)load_hp(q, dt, b * qs[0] + i * qs[1] + h * qs[2] + e * qs[3]) *
                               (double)load_hp(k, dt, b * ks[0] + kk * ks[1] + h * ks[2] + e * ks[3]);
                    p[kk] = acc * (double)scale;
                    m = std::max(m, p[kk]);
                }
                double l = 0.0;
                for (int64_t kk = 0; kk < nvis; ++kk) { p[kk] = std::exp(p[kk] - m); l += p[kk]; }
                for (int64_t e = 0; e < Dh; ++e) {
                    double acc = 0.0;
                    for (int64_t kk = 0; kk < nvis; ++kk)
                        acc += p[kk] * (double)load_hp(v, dt, b * vs[0] + kk * vs[1] + h * vs[2] + e * vs[3]);
                    store_hp(out, dt, (b * Sq + i) * ldo + h * Dh + e, nvis > 0 ? (float)(acc / l) : 0.0f);
                }
            }
        }
    return 0;
}
int orc_bf16_attn(const uint16_t* q, const int64_t* qs, const uint16_t* k, const int64_t* ks,
                  const uint16_t* v, const int64_t* vs,
                  int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                  int mask, const int32_t* kv_len, uint16_t* out, int64_t ldo) {
    return orc_hp_attn(q, qs, k, ks, v, vs, B, H, Sq, Skv, Dh, scale, mask, kv_len, out, ldo, ORC_BF16);
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

}  // extern "C"
