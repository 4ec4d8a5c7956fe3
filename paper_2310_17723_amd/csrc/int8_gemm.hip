// hero_int8_gemm: GeMM^quant, INT8 x INT8 -> INT32 on the gfx950 matrix cores with the
// dequantization / static-scale / bias / GELU / residual / requantization epilogue fused
// behind the accumulators (paper Sec. 2.1 GEMM convention and column-wise weight scales;
// Sec. 2.2.2 fused dequantization and the bare Round after folding; Sec. 2.2.3 GELU^quant).
//
// Both operands are K-contiguous ([M][K] activations, [N][K] weights), so each MFMA
// operand fragment is one 128-bit LDS read.  The block tile is staged through LDS in
// BK = 64 byte slabs (row stride padded to 80 bytes: conflict-free for 128-bit reads),
// double buffered, with the next slab's global loads in flight during the MFMAs.
//
// MFMA: v_mfma_i32_32x32x32_i8.  The weight fragment is passed as the first operand and
// the activation fragment as the second, so the accumulator of lane l holds, for ONE
// output row m = l % 32, the columns n = 8g + 4(l/32) + t  (register 4g + t): four
// consecutive columns per register group, which makes the epilogue's stores 4 columns
// wide and the per-row scale a single register.
#include "hero_common.h"

namespace {

constexpr int BK = 64;          // bytes of K per LDS slab
constexpr int LDS_LD = BK + 16; // padded LDS row stride in bytes

struct GemmArgs {
    const int8_t* A; int64_t lda; const float* a_row_scale;
    const int8_t* Bt; int64_t ldb; const float* b_col_scale;
    const float* bias; const void* residual; int64_t ldr;
    const float* out_col_scale;
    void* C; int64_t ldc;
    int M, N, K;
};

// One output value through the epilogue.  EPI / CDT are compile-time.
template <int EPI, int CDT>
__device__ __forceinline__ float epilogue_value(int acc, float rs, bool has_rs, float cs, float bs) {
    float t = (float)acc;
    if (has_rs) t = t * rs;
    float y = fmaf(t, cs, bs);
    if (EPI == HERO_EPI_DEQUANT_GELU || EPI == HERO_EPI_GELU_REQUANT) y = gelu_erf(y);
    return y;
}

template <int BM, int BN, int WM, int WN, int EPI, int CDT, int RDT>
__global__ __launch_bounds__(WM * WN * 64) void int8_gemm_kernel(GemmArgs g) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;      // 32x32 MFMA tiles per wave
    constexpr int A_UNITS = BM * (BK / 16) / NT, B_UNITS = BN * (BK / 16) / NT;
    static_assert(BM * (BK / 16) % NT == 0 && BN * (BK / 16) % NT == 0, "tile/threads mismatch");
    __shared__ __attribute__((aligned(16))) int8_t sA[2][BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) int8_t sB[2][BN * LDS_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int KT = g.K / BK;

    // global -> register staging: unit u of this thread is row (idx/4), 16-byte chunk (idx%4)
    v4i ra[A_UNITS], rb[B_UNITS];
    auto load_slab = [&](int kt) {
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u) {
            int idx = tid + u * NT, row = idx >> 2, ch = idx & 3;
            int m = min(m0 + row, g.M - 1);                                   // clamp: ragged M
            ra[u] = *reinterpret_cast<const v4i*>(g.A + (int64_t)m * g.lda + (int64_t)kt * BK + ch * 16);
        }
#pragma unroll
        for (int u = 0; u < B_UNITS; ++u) {
            int idx = tid + u * NT, row = idx >> 2, ch = idx & 3;
            int n = min(n0 + row, g.N - 1);
            rb[u] = *reinterpret_cast<const v4i*>(g.Bt + (int64_t)n * g.ldb + (int64_t)kt * BK + ch * 16);
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u) {
            int idx = tid + u * NT, row = idx >> 2, ch = idx & 3;
            *reinterpret_cast<v4i*>(&sA[buf][row * LDS_LD + ch * 16]) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < B_UNITS; ++u) {
            int idx = tid + u * NT, row = idx >> 2, ch = idx & 3;
            *reinterpret_cast<v4i*>(&sB[buf][row * LDS_LD + ch * 16]) = rb[u];
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    load_slab(0);
    store_slab(0);
    __syncthreads();
    const int frag_off = (lane & 31) * LDS_LD + (lane >> 5) * 16;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_slab(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4i fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const v4i*>(&sA[buf][(wm * TM * 32 + i * 32) * LDS_LD + frag_off + ks * 32]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const v4i*>(&sB[buf][(wn * TN * 32 + j * 32) * LDS_LD + frag_off + ks * 32]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_slab(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------
    const bool has_rs = g.a_row_scale != nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * TM * 32 + i * 32 + (lane & 31);
        if (m >= g.M) continue;
        const float rs = (EPI != HERO_EPI_RAW_I32 && has_rs) ? g.a_row_scale[m] : 1.0f;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int n = n0 + wn * TN * 32 + j * 32 + gq * 8 + (lane >> 5) * 4;
                if (n >= g.N) continue;
                const bool full = n + 3 < g.N;
                const int64_t co = (int64_t)m * g.ldc + n;
                if (EPI == HERO_EPI_RAW_I32) {
                    int* cp = (int*)g.C + co;
                    if (full) {
                        v4i o = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
                        *reinterpret_cast<v4i*>(cp) = o;
                    } else {
                        for (int t = 0; t < 4; ++t) if (n + t < g.N) cp[t] = acc[i][j][4 * gq + t];
                    }
                    continue;
                }
                float y[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int nn = min(n + t, g.N - 1);
                    const float cs = g.b_col_scale[nn];
                    const float bs = g.bias ? g.bias[nn] : 0.0f;
                    y[t] = epilogue_value<EPI, CDT>(acc[i][j][4 * gq + t], rs, has_rs, cs, bs);
                }
                if (EPI == HERO_EPI_REQUANT || EPI == HERO_EPI_GELU_REQUANT) {
                    int q[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (EPI == HERO_EPI_GELU_REQUANT) q[t] = quant_code_div(y[t], g.out_col_scale[min(n + t, g.N - 1)]);
                        else q[t] = round_sat_i8(y[t]);
                    }
                    int8_t* cp = (int8_t*)g.C + co;
                    if (full) *reinterpret_cast<uint32_t*>(cp) = pack4_i8(q[0], q[1], q[2], q[3]);
                    else for (int t = 0; t < 4; ++t) if (n + t < g.N) cp[t] = (int8_t)q[t];
                } else {    // DEQUANT / DEQUANT_GELU -> 16-bit float
                    if (RDT >= 0) {
                        const uint16_t* rp = (const uint16_t*)g.residual + (int64_t)m * g.ldr + n;
#pragma unroll
                        for (int t = 0; t < 4; ++t) if (n + t < g.N) y[t] = y[t] + hp_to_f32<RDT>(rp[t]);
                    }
                    uint16_t* cp = (uint16_t*)g.C + co;
                    uint32_t h[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) h[t] = f32_to_hp<CDT>(y[t]);
                    if (full) {
                        v2i o = {(int)(h[0] | (h[1] << 16)), (int)(h[2] | (h[3] << 16))};
                        *reinterpret_cast<v2i*>(cp) = o;
                    } else {
                        for (int t = 0; t < 4; ++t) if (n + t < g.N) cp[t] = (uint16_t)h[t];
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int EPI, int CDT, int RDT>
hero_status launch_tile(const GemmArgs& g, hipStream_t st) {
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM), block(WM * WN * 64);
    hipLaunchKernelGGL((int8_gemm_kernel<BM, BN, WM, WN, EPI, CDT, RDT>), grid, block, 0, st, g);
    return hero_launch_status();
}

template <int EPI, int CDT, int RDT>
hero_status launch_epi(const GemmArgs& g, hipStream_t st) {
    return launch_tile<128, 128, 2, 2, EPI, CDT, RDT>(g, st);
}

}  // namespace

extern "C" hero_status hero_int8_gemm(const int8_t* A, int64_t lda, const float* a_row_scale,
                                      const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                      const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                      hero_epilogue epi, const float* out_col_scale,
                                      void* C, hero_dtype c_dt, int64_t ldc,
                                      int64_t M, int64_t N, int64_t K, void* stream) {
    if (M < 0 || N < 0 || K <= 0) return HERO_ERR_SHAPE;
    if (M > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x7fffffffLL) return HERO_ERR_SHAPE;
    if (K % BK != 0) return HERO_ERR_UNSUPPORTED;
    if (lda < K || ldb < K || ldc < N) return HERO_ERR_SHAPE;
    if (M == 0 || N == 0) return HERO_OK;
    if (!A || !Bt || !C) return HERO_ERR_NULL;
    if (epi != HERO_EPI_RAW_I32 && !b_col_scale) return HERO_ERR_NULL;
    if (epi == HERO_EPI_GELU_REQUANT && !out_col_scale) return HERO_ERR_NULL;
    const bool c16 = c_dt == HERO_F16 || c_dt == HERO_BF16;
    switch (epi) {
    case HERO_EPI_RAW_I32: if (c_dt != HERO_I32) return HERO_ERR_UNSUPPORTED; break;
    case HERO_EPI_DEQUANT: case HERO_EPI_DEQUANT_GELU: if (!c16) return HERO_ERR_UNSUPPORTED; break;
    case HERO_EPI_REQUANT: case HERO_EPI_GELU_REQUANT: if (c_dt != HERO_I8) return HERO_ERR_UNSUPPORTED; break;
    default: return HERO_ERR_UNSUPPORTED;
    }
    if (residual) {
        if (epi != HERO_EPI_DEQUANT) return HERO_ERR_UNSUPPORTED;
        if (res_dt != HERO_F16 && res_dt != HERO_BF16) return HERO_ERR_UNSUPPORTED;
        if (ldr < N) return HERO_ERR_SHAPE;
        if (ldr % 4 != 0 || !hero_aligned16(residual)) return HERO_ERR_ALIGN;
    }
    if (lda % 16 != 0 || ldb % 16 != 0 || ldc % 4 != 0) return HERO_ERR_ALIGN;
    if (!hero_aligned16(A) || !hero_aligned16(Bt) || !hero_aligned16(C)) return HERO_ERR_ALIGN;
    if ((M + 127) / 128 > 65535) return HERO_ERR_UNSUPPORTED;

    GemmArgs g;
    g.A = A; g.lda = lda; g.a_row_scale = a_row_scale; g.Bt = Bt; g.ldb = ldb; g.b_col_scale = b_col_scale;
    g.bias = bias; g.residual = residual; g.ldr = ldr; g.out_col_scale = out_col_scale;
    g.C = C; g.ldc = ldc; g.M = (int)M; g.N = (int)N; g.K = (int)K;
    hipStream_t st = (hipStream_t)stream;
    switch (epi) {
    case HERO_EPI_RAW_I32: return launch_epi<HERO_EPI_RAW_I32, HERO_I32, -1>(g, st);
    case HERO_EPI_REQUANT: return launch_epi<HERO_EPI_REQUANT, HERO_I8, -1>(g, st);
    case HERO_EPI_GELU_REQUANT: return launch_epi<HERO_EPI_GELU_REQUANT, HERO_I8, -1>(g, st);
    case HERO_EPI_DEQUANT_GELU:
        return c_dt == HERO_BF16 ? launch_epi<HERO_EPI_DEQUANT_GELU, HERO_BF16, -1>(g, st)
                                 : launch_epi<HERO_EPI_DEQUANT_GELU, HERO_F16, -1>(g, st);
    case HERO_EPI_DEQUANT:
        if (!residual)
            return c_dt == HERO_BF16 ? launch_epi<HERO_EPI_DEQUANT, HERO_BF16, -1>(g, st)
                                     : launch_epi<HERO_EPI_DEQUANT, HERO_F16, -1>(g, st);
        if (c_dt == HERO_BF16 && res_dt == HERO_BF16) return launch_epi<HERO_EPI_DEQUANT, HERO_BF16, HERO_BF16>(g, st);
        if (c_dt == HERO_F16 && res_dt == HERO_F16) return launch_epi<HERO_EPI_DEQUANT, HERO_F16, HERO_F16>(g, st);
        return HERO_ERR_UNSUPPORTED;
    default: return HERO_ERR_UNSUPPORTED;
    }
}
