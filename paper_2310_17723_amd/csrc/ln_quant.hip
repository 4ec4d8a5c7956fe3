// hero_ln_quant: LN^quant, the fused LayerNorm + token-wise (TWQ) INT8 quantization
// (paper Sec. 2.1 TWQ paragraph; Sec. 2.2.2 last line of the quantized attention flow;
// Sec. 2.2.3 last line of the quantized MLP flow).
//
// HBM-bound: every input element is read once and every output element written once.
// One wavefront owns one row and keeps it in registers (NCH chunks of EPL elements per
// lane, each chunk one 128-bit load per lane, consecutive lanes consecutive addresses);
// the three row reductions (sum, sum of squared deviations, absmax) are 64-lane shuffles.
// Statistics are fp32, mean first and variance about the mean.  The codes come from an
// IEEE division by the row scale followed by round-half-even, exactly the primitive.
#include "hero_common.h"

namespace {

struct LnArgs {
    const void* x; const float* x_row_scale;
    const void* r; const float* r_col_scale;
    const float* gamma; const float* beta;
    float eps; int64_t M; int D;
    int8_t* y_q; float* y_scale; void* y_hp;
    int x_dt, r_dt, hp_dt;       // r_dt / hp_dt = -1 when absent
};

__device__ __forceinline__ float byte_to_f32(int w, int i) { return (float)(int8_t)(w >> (8 * i)); }

template <bool X_I8, int NCH>
__global__ __launch_bounds__(256) void ln_quant_kernel(LnArgs a) {
    constexpr int EPL = X_I8 ? 16 : 8;
    constexpr int CH = EPL * HERO_WAVE;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;                          // whole wave leaves together
    const int D = a.D;
    float v[NCH][EPL];

    // ---- load the row (sum of the addends), fp32 -------------------------------------
    const float xs = X_I8 ? a.x_row_scale[row] : 1.0f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j0 = c * CH + lane * EPL;
        const bool act = j0 < D;
        if (!act) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) v[c][e] = 0.0f;
            continue;
        }
        const int64_t off = row * (int64_t)D + j0;
        if constexpr (X_I8) {
            v4i w = *reinterpret_cast<const v4i*>((const int8_t*)a.x + off);
#pragma unroll
            for (int e = 0; e < 16; ++e) v[c][e] = byte_to_f32(w[e >> 2], e & 3) * xs;
        } else {
            v4i w = *reinterpret_cast<const v4i*>((const uint16_t*)a.x + off);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t h = ((uint32_t)w[e >> 1] >> (16 * (e & 1))) & 0xffffu;
                v[c][e] = a.x_dt == HERO_BF16 ? bf16_bits_to_f32(h) : f16_bits_to_f32(h);
            }
        }
        if (a.r_dt == HERO_I8) {
            int w[4] = {0, 0, 0, 0};
            if constexpr (EPL == 16) {
                v4i t = *reinterpret_cast<const v4i*>((const int8_t*)a.r + off);
                w[0] = t[0]; w[1] = t[1]; w[2] = t[2]; w[3] = t[3];
            } else {
                v2i t = *reinterpret_cast<const v2i*>((const int8_t*)a.r + off);
                w[0] = t[0]; w[1] = t[1];
            }
#pragma unroll
            for (int e4 = 0; e4 < EPL / 4; ++e4) {
                v4f rc = *reinterpret_cast<const v4f*>(a.r_col_scale + j0 + 4 * e4);
#pragma unroll
                for (int t = 0; t < 4; ++t) v[c][4 * e4 + t] = fmaf(byte_to_f32(w[e4], t), rc[t], v[c][4 * e4 + t]);
            }
        } else if (a.r_dt >= 0) {
#pragma unroll
            for (int e8 = 0; e8 < EPL / 8; ++e8) {
                v4i w = *reinterpret_cast<const v4i*>((const uint16_t*)a.r + off + 8 * e8);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    uint32_t h = ((uint32_t)w[e >> 1] >> (16 * (e & 1))) & 0xffffu;
                    v[c][8 * e8 + e] += a.r_dt == HERO_BF16 ? bf16_bits_to_f32(h) : f16_bits_to_f32(h);
                }
            }
        }
    }

    // ---- LayerNorm: mean, then variance about the mean (fp32) --------------------------
    if (a.gamma) {
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < EPL; ++e) s += v[c][e];
        const float mean = wave_sum(s) / (float)D;
        float q = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bool act = c * CH + lane * EPL < D;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float dlt = v[c][e] - mean;
                v[c][e] = dlt;
                q = act ? fmaf(dlt, dlt, q) : q;
            }
        }
        const float var = wave_sum(q) / (float)D;
        const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j0 = c * CH + lane * EPL;
            if (j0 < D) {
#pragma unroll
                for (int e4 = 0; e4 < EPL / 4; ++e4) {
                    v4f g = *reinterpret_cast<const v4f*>(a.gamma + j0 + 4 * e4);
                    v4f b = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (a.beta) b = *reinterpret_cast<const v4f*>(a.beta + j0 + 4 * e4);
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[c][4 * e4 + t] = fmaf(v[c][4 * e4 + t] * rstd, g[t], b[t]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) v[c][e] = 0.0f;
            }
        }
    }

    // ---- token-wise scale and codes -------------------------------------------------------
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(v[c][e]));
    amax = wave_max(amax);
    const float sc = amax == 0.0f ? 1.0f : __fdiv_rn(amax, 127.0f);
    if (lane == 0) a.y_scale[row] = sc;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j0 = c * CH + lane * EPL;
        if (j0 >= D) continue;
        const int64_t off = row * (int64_t)D + j0;
        uint32_t pk[EPL / 4];
#pragma unroll
        for (int e4 = 0; e4 < EPL / 4; ++e4)
            pk[e4] = pack4_i8(quant_code_div(v[c][4 * e4 + 0], sc), quant_code_div(v[c][4 * e4 + 1], sc),
                              quant_code_div(v[c][4 * e4 + 2], sc), quant_code_div(v[c][4 * e4 + 3], sc));
        if constexpr (EPL == 16) {
            v4i o = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3]};
            *reinterpret_cast<v4i*>(a.y_q + off) = o;
        } else {
            v2i o = {(int)pk[0], (int)pk[1]};
            *reinterpret_cast<v2i*>(a.y_q + off) = o;
        }
        if (a.hp_dt >= 0) {
#pragma unroll
            for (int e8 = 0; e8 < EPL / 8; ++e8) {
                v4i o;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    float f0 = v[c][8 * e8 + 2 * p], f1 = v[c][8 * e8 + 2 * p + 1];
                    uint32_t h0 = a.hp_dt == HERO_BF16 ? f32_to_bf16_bits(f0) : f32_to_f16_bits(f0);
                    uint32_t h1 = a.hp_dt == HERO_BF16 ? f32_to_bf16_bits(f1) : f32_to_f16_bits(f1);
                    o[p] = (int)(h0 | (h1 << 16));
                }
                *reinterpret_cast<v4i*>((uint16_t*)a.y_hp + off + 8 * e8) = o;
            }
        }
    }
}

template <bool X_I8>
hero_status launch(const LnArgs& a, hipStream_t st) {
    constexpr int CH = (X_I8 ? 16 : 8) * HERO_WAVE;
    const int nch = (a.D + CH - 1) / CH;
    dim3 grid((unsigned)((a.M + 3) / 4)), block(256);
    if (nch <= 1) hipLaunchKernelGGL((ln_quant_kernel<X_I8, 1>), grid, block, 0, st, a);
    else if (nch <= 2) hipLaunchKernelGGL((ln_quant_kernel<X_I8, 2>), grid, block, 0, st, a);
    else if (nch <= 4) hipLaunchKernelGGL((ln_quant_kernel<X_I8, 4>), grid, block, 0, st, a);
    else if (nch <= 8) hipLaunchKernelGGL((ln_quant_kernel<X_I8, 8>), grid, block, 0, st, a);
    else return HERO_ERR_UNSUPPORTED;
    return hero_launch_status();
}

}  // namespace

extern "C" hero_status hero_ln_quant(const void* x, hero_dtype x_dt, const float* x_row_scale,
                                     const void* r, hero_dtype r_dt, const float* r_col_scale,
                                     const float* gamma, const float* beta, float eps,
                                     int64_t M, int64_t D,
                                     int8_t* y_q, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream) {
    if (M < 0 || D <= 0) return HERO_ERR_SHAPE;
    if (D % 16 != 0) return HERO_ERR_UNSUPPORTED;
    if (M == 0) return HERO_OK;
    if (!x || !y_q || !y_scale) return HERO_ERR_NULL;
    const bool x_i8 = x_dt == HERO_I8;
    if (!x_i8 && x_dt != HERO_BF16 && x_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (x_i8 && !x_row_scale) return HERO_ERR_NULL;
    if (r) {
        if (r_dt != HERO_I8 && r_dt != HERO_BF16 && r_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
        if (r_dt == HERO_I8 && !r_col_scale) return HERO_ERR_NULL;
    }
    if (!gamma && beta) return HERO_ERR_NULL;
    if (y_hp && y_hp_dt != HERO_BF16 && y_hp_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (D > (x_i8 ? 8192 : 4096)) return HERO_ERR_UNSUPPORTED;      // row must fit the register file
    if (!hero_aligned16(x) || !hero_aligned16(r) || !hero_aligned16(y_q) || !hero_aligned16(y_hp) ||
        !hero_aligned16(gamma) || !hero_aligned16(beta) || !hero_aligned16(r_col_scale))
        return HERO_ERR_ALIGN;
    if ((M + 3) / 4 > 0x7fffffffLL) return HERO_ERR_SHAPE;
    LnArgs a;
    a.x = x; a.x_row_scale = x_row_scale; a.r = r; a.r_col_scale = r_col_scale;
    a.gamma = gamma; a.beta = beta; a.eps = eps; a.M = M; a.D = (int)D;
    a.y_q = y_q; a.y_scale = y_scale; a.y_hp = y_hp;
    a.x_dt = (int)x_dt; a.r_dt = r ? (int)r_dt : -1; a.hp_dt = y_hp ? (int)y_hp_dt : -1;
    hipStream_t st = (hipStream_t)stream;
    return x_i8 ? launch<true>(a, st) : launch<false>(a, st);
}
