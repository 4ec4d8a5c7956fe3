// 16-bit side of a switched module (paper Sec. 2.3, Table 1: a module marked with a cross runs
// in FP16 / BF16): hero_hp_gemm and hero_hp_attn (and their BF16-only names hero_bf16_gemm / hero_bf16_attn).
// bf16 or fp16 operands, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16 / _f16), results in
// the operands' type.  These kernels make the mixed modes functional; they follow the same operand layouts as
// the INT8 kernels (both operands K-contiguous, weight fragment first so a lane owns one output row); large
// GEMMs go to the persistent kernels of int8_gemm.hip.
#include "hero_common.h"

namespace {

typedef __bf16 v8b __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// one 32x32x16 matrix instruction on 8 + 8 16-bit values per lane; DT = HERO_BF16 or HERO_F16
template <int DT>
__device__ __forceinline__ v16f mfma_hp(v4i a, v4i b, v16f c) {
    if constexpr (DT == HERO_BF16) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8b, a), __builtin_bit_cast(v8b, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------
// GEMM: C = act(A Wt^T + bias) (+ residual).  128x128 tile, 4 waves of 64x64, slabs of 32
// bf16 (64 bytes) of K staged through registers into double-buffered, padded LDS.
// ------------------------------------------------------------------------------------------
constexpr int GBK = 64;             // bytes of K per slab (32 bf16)
constexpr int GLD = GBK + 16;

struct BGemmArgs {
    const uint16_t* A; int64_t lda; const uint16_t* Wt; int64_t ldb;
    const float* bias; const uint16_t* residual; int64_t ldr; int gelu;
    uint16_t* C; int64_t ldc; int M, N, K;
};

template <int DT>
__global__ __launch_bounds__(256) void bf16_gemm_kernel(BGemmArgs g) {
    constexpr int BM = 128, BN = 128, TM = 2, TN = 2, NT = 256, CPR = GBK / 16;
    constexpr int UNITS = BM * CPR / NT;
    __shared__ __attribute__((aligned(16))) int8_t sA[2][BM * GLD];
    __shared__ __attribute__((aligned(16))) int8_t sB[2][BN * GLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int KT = g.K * 2 / GBK, last = KT - 1;
    const int8_t* pa[UNITS];
    const int8_t* pb[UNITS];
    int lo[UNITS];
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
        int idx = tid + u * NT, row = idx / CPR, ch = idx % CPR;
        pa[u] = (const int8_t*)(g.A + (int64_t)min(m0 + row, g.M - 1) * g.lda) + ch * 16;
        pb[u] = (const int8_t*)(g.Wt + (int64_t)min(n0 + row, g.N - 1) * g.ldb) + ch * 16;
        lo[u] = row * GLD + ch * 16;
    }
    v4i ra[UNITS], rb[UNITS];
    auto load = [&](int kt) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            ra[u] = *reinterpret_cast<const v4i*>(pa[u] + (int64_t)kt * GBK);
            rb[u] = *reinterpret_cast<const v4i*>(pb[u] + (int64_t)kt * GBK);
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            *reinterpret_cast<v4i*>(&sA[buf][lo[u]]) = ra[u];
            *reinterpret_cast<v4i*>(&sB[buf][lo[u]]) = rb[u];
        }
    };
    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    load(0);
    store(0);
    load(min(1, last));
    __syncthreads();
    const int fo = (lane & 31) * GLD + (lane >> 5) * 16;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
#pragma unroll
        for (int ks = 0; ks < GBK / 32; ++ks) {
            v4i fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i*>(&sA[buf][(wm * 64 + i * 32) * GLD + fo + ks * 32]);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i*>(&sB[buf][(wn * 64 + j * 32) * GLD + fo + ks * 32]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = mfma_hp<DT>(fb[j], fa[i], acc[i][j]);
        }
        store(buf ^ 1);                       // slab kt + 1 (a redundant copy of the last slab at the end)
        load(min(kt + 2, last));
        __syncthreads();
    }
    // epilogue: lane owns row m, 4-column groups
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * 64 + i * 32 + (lane & 31);
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int n = n0 + wn * 64 + j * 32 + gq * 8 + (lane >> 5) * 4;
                if (n >= g.N) continue;
                uint32_t h[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int nn = min(n + t, g.N - 1);
                    float y = acc[i][j][4 * gq + t] + (g.bias ? g.bias[nn] : 0.0f);
                    if (g.gelu) y = gelu_erf(y);
                    if (g.residual && n + t < g.N) y += hp_to_f32<DT>(g.residual[(int64_t)m * g.ldr + n + t]);
                    h[t] = f32_to_hp<DT>(y);
                }
                uint16_t* cp = g.C + (int64_t)m * g.ldc + n;
                if (n + 3 < g.N) {
                    v2i o = {(int)(h[0] | (h[1] << 16)), (int)(h[2] | (h[3] << 16))};
                    *reinterpret_cast<v2i*>(cp) = o;
                } else {
                    for (int t = 0; t < 4; ++t) if (n + t < g.N) cp[t] = (uint16_t)h[t];
                }
            }
    }
}

// ------------------------------------------------------------------------------------------
// Attention core softmax(q k^T * scale) v, single pass with an online softmax (nothing is
// quantized here, so the running rescale is legitimate).  Scores are computed transposed
// (S^T = K Q^T): lane l owns query l % 32, so the running max / sum and the rescale of the
// output accumulators are per-lane scalars.
// ------------------------------------------------------------------------------------------
constexpr int ABQ = 128, ABKV = 64;

struct BAttnArgs {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;
    int64_t qs[4], ks[4], vs[4];
    int B, H, Sq, Skv; float scale; int mask; const int32_t* kv_len;
    uint16_t* out; int64_t ldo;
};

template <int DH, int DT>
__global__ __launch_bounds__(256) void bf16_attn_kernel(BAttnArgs a) {
    constexpr int KLD = DH * 2 + 16;       // sK row stride, bytes
    constexpr int VLD = ABKV * 2 + 16;     // sVt row stride, bytes (64 keys of bf16)
    constexpr int DS = DH / 16;            // 16-wide MFMA k-steps over the head dimension
    constexpr int CT = DH / 32;            // 32-channel output tiles
    __shared__ __attribute__((aligned(16))) int8_t sK[ABKV * KLD];
    __shared__ __attribute__((aligned(16))) int8_t sVt[DH * VLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hh = lane >> 5, ql = lane & 31;
    // Workgroups go round-robin to the 8 XCDs: all query blocks of one (batch, head) are sent to the same XCD, back to
    // back, so its K / V stream hits that XCD's L2 after the first block; their order inside the head rotates with a
    // hash of the head's number (the blocks of a causal or padded head differ in length, and the hardware places
    // workgroups on the compute units in launch order: a fixed order hands a unit the same kind of block every time).
    const int nqb = (a.Sq + ABQ - 1) / ABQ;
    const int slot = blockIdx.x / 8, bh = (slot / nqb) * 8 + (int)(blockIdx.x % 8);
    if (bh >= a.B * a.H) return;
    const uint32_t rot = ((uint32_t)(slot / nqb) * 2654435761u) >> 20;
    const int b = bh / a.H, h = bh % a.H, q0 = (int)((slot % nqb + rot) % (uint32_t)nqb) * ABQ;
    const int len = a.kv_len ? min(max(a.kv_len[b], 0), a.Skv) : a.Skv;
    const int shift = len - a.Sq;
    const int qi = q0 + wave * 32 + ql;
    int nvis = len;
    if (a.mask == HERO_MASK_CAUSAL) nvis = min(len, qi + shift + 1);
    nvis = max(nvis, 0);
    int kmax = len;
    if (a.mask == HERO_MASK_CAUSAL) kmax = min(len, min(q0 + ABQ, a.Sq) + shift);
    // PADDING mask in self-attention: the positions >= len are padding as queries too; they see no key (output 0)
    if (a.mask == HERO_MASK_PADDING && a.Sq == a.Skv) {
        if (qi >= len) nvis = 0;
        if (q0 >= len) kmax = 0;
    }
    const int ntiles = (max(kmax, 0) + ABKV - 1) / ABKV;

    v4i qf[DS];
    {
        const uint16_t* qp = a.q + (int64_t)b * a.qs[0] + (int64_t)min(qi, a.Sq - 1) * a.qs[1] + (int64_t)h * a.qs[2];
#pragma unroll
        for (int d = 0; d < DS; ++d) qf[d] = *reinterpret_cast<const v4i*>(qp + d * 16 + hh * 8);
    }
    const uint16_t* kbase = a.k + (int64_t)b * a.ks[0] + (int64_t)h * a.ks[2];
    const uint16_t* vbase = a.v + (int64_t)b * a.vs[0] + (int64_t)h * a.vs[2];
    const float c2 = a.scale * 1.44269504088896340736f;
    float m2 = -INFINITY, l = 0.0f;
    v16f o[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[c][r] = 0.0f;

    // K / V tiles: global -> registers (the next tile's loads are in flight during the current tile's math) -> LDS.
    // A thread's unit is one 16-byte chunk (8 channels) of TWO neighbouring key rows 2r, 2r + 1: V is stored transposed
    // and the two keys sit side by side there, so a channel's pair of values goes out as one 32-bit store.
    constexpr int CPRW = DH / 8;                           // 16-byte chunks per K/V row
    constexpr int PAIRS = (ABKV / 2) * CPRW / 256;         // units per thread and tile
    v4i rk[PAIRS][2], rv[PAIRS][2];
    auto fetch = [&](int tile) {
#pragma unroll
        for (int u = 0; u < PAIRS; ++u) {
            const int idx = tid + u * 256, rp = idx / CPRW, ch = idx % CPRW;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int key = min(tile * ABKV + 2 * rp + j, a.Skv - 1);
                rk[u][j] = *reinterpret_cast<const v4i*>(kbase + (int64_t)key * a.ks[1] + ch * 8);
                rv[u][j] = *reinterpret_cast<const v4i*>(vbase + (int64_t)key * a.vs[1] + ch * 8);
            }
        }
    };
    if (ntiles > 0) fetch(0);
    for (int tile = 0; tile < ntiles; ++tile) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PAIRS; ++u) {
            const int idx = tid + u * 256, rp = idx / CPRW, ch = idx % CPRW, row = 2 * rp;
            *reinterpret_cast<v4i*>(&sK[row * KLD + ch * 16]) = rk[u][0];
            *reinterpret_cast<v4i*>(&sK[(row + 1) * KLD + ch * 16]) = rk[u][1];
            // key row 32kb + 8g + 4h' + t of the tile -> position 32kb + 16(g>>1) + 8h' + 4(g&1) + t:
            // within each 16-key MFMA step, half h' holds its 8 keys (g&1, t) contiguously; rows 2r and 2r + 1
            // differ in the lowest bit of t only
            const int r32 = row & 31, g4 = r32 >> 3, hp = (r32 >> 2) & 1, t = r32 & 3;
            const int pos = (row & 32) + (g4 >> 1) * 16 + hp * 8 + (g4 & 1) * 4 + t;
#pragma unroll
            for (int j = 0; j < 4; ++j) {                   // channels 2j, 2j + 1 of both keys
                const uint32_t w0 = (uint32_t)rv[u][0][j], w1 = (uint32_t)rv[u][1][j];
                *reinterpret_cast<uint32_t*>(&sVt[(ch * 8 + 2 * j) * VLD + pos * 2]) = __builtin_amdgcn_perm(w1, w0, 0x05040100u);
                *reinterpret_cast<uint32_t*>(&sVt[(ch * 8 + 2 * j + 1) * VLD + pos * 2]) = __builtin_amdgcn_perm(w1, w0, 0x07060302u);
            }
        }
        __syncthreads();
        if (tile + 1 < ntiles) fetch(tile + 1);
#pragma unroll
        for (int s = 0; s < ABKV / 32; ++s) {
            v16f acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int d = 0; d < DS; ++d) {
                v4i kf = *reinterpret_cast<const v4i*>(&sK[(s * 32 + ql) * KLD + d * 32 + hh * 16]);
                acc = mfma_hp<DT>(kf, qf[d], acc);
            }
            float tmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = tile * ABKV + s * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
                acc[r] = key < nvis ? acc[r] * c2 : -INFINITY;
                tmax = fmaxf(tmax, acc[r]);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            uint32_t pb[8];
            if (tmax > -INFINITY) {
                const float mn = fmaxf(m2, tmax);
                const float resc = __builtin_amdgcn_exp2f(m2 - mn);
                float sum = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float e0 = __builtin_amdgcn_exp2f(acc[r] - mn), e1 = __builtin_amdgcn_exp2f(acc[r + 1] - mn);
                    const uint32_t pk = pack2_hp<DT>(e0, e1);
                    sum += hp_to_f32<DT>(pk & 0xffffu) + hp_to_f32<DT>(pk >> 16);           // the sum of what PV really multiplies
                    pb[r >> 1] = pk;
                }
                l = fmaf(l, resc, sum);
                // the accumulators are rescaled only in steps where some query of the wave raises its maximum
                // (otherwise every factor is exactly 1)
                if (__builtin_amdgcn_ballot_w64(mn != m2) != 0) {
#pragma unroll
                    for (int c = 0; c < CT; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[c][r] *= resc;
                }
                m2 = mn;
            } else {
#pragma unroll
                for (int r = 0; r < 8; ++r) pb[r] = 0;
            }
            // registers 0..7 (g = 0,1) feed the first 16-key MFMA step, 8..15 (g = 2,3) the second
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                v4i pf = {(int)pb[4 * st], (int)pb[4 * st + 1], (int)pb[4 * st + 2], (int)pb[4 * st + 3]};
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    v4i vf = *reinterpret_cast<const v4i*>(&sVt[(c * 32 + ql) * VLD + (s * 32 + st * 16 + hh * 8) * 2]);
                    o[c] = mfma_hp<DT>(vf, pf, o[c]);
                }
            }
        }
    }
    l += __shfl_xor(l, 32);
    if (qi >= a.Sq) return;
    const float inv_l = l > 0.0f ? 1.0f / l : 0.0f;
    const int64_t orow = ((int64_t)b * a.Sq + qi) * a.ldo + (int64_t)h * DH;
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int e0 = c * 32 + g * 8 + hh * 4;
            v2i w = {(int)pack2_hp<DT>(o[c][4 * g] * inv_l, o[c][4 * g + 1] * inv_l),
                     (int)pack2_hp<DT>(o[c][4 * g + 2] * inv_l, o[c][4 * g + 3] * inv_l)};
            *reinterpret_cast<v2i*>(a.out + orow + e0) = w;
        }
}

__global__ void zero_bf16_kernel(uint16_t* out, int64_t rows, int64_t cols, int64_t ld) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * cols) out[(i / cols) * ld + i % cols] = 0;
}

}  // namespace

static hero_status run_hp_gemm(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                               const float* bias, const void* residual, int64_t ldr, int gelu,
                               void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, void* stream, int tile) {
    if (dt != HERO_BF16 && dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K <= 0 || M > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x3fffffffLL) return HERO_ERR_SHAPE;
    if (K % 32 != 0) return HERO_ERR_UNSUPPORTED;
    if (lda < K || ldb < K || ldc < N || (residual && ldr < N)) return HERO_ERR_SHAPE;
    if (M == 0 || N == 0) return HERO_OK;
    if (!A || !Wt || !C) return HERO_ERR_NULL;
    if (lda % 8 || ldb % 8 || ldc % 4 || !hero_aligned16(A) || !hero_aligned16(Wt) || !hero_aligned16(C)) return HERO_ERR_ALIGN;
    if (!residual || (ldr % 8 == 0 && hero_aligned16(residual))) {        // large problems: the persistent kernels
        const hero_status big = hero_hp_gemm_large(A, lda, Wt, ldb, bias, residual, ldr, gelu, C, ldc, M, N, K, dt, (hipStream_t)stream, tile);
        if (big != HERO_ERR_UNSUPPORTED) return big;
    }
    if ((M + 127) / 128 > 65535) return HERO_ERR_UNSUPPORTED;
    BGemmArgs g;
    g.A = (const uint16_t*)A; g.lda = lda; g.Wt = (const uint16_t*)Wt; g.ldb = ldb; g.bias = bias;
    g.residual = (const uint16_t*)residual; g.ldr = ldr; g.gelu = gelu; g.C = (uint16_t*)C; g.ldc = ldc;
    g.M = (int)M; g.N = (int)N; g.K = (int)K;
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    if (dt == HERO_BF16) hipLaunchKernelGGL(bf16_gemm_kernel<HERO_BF16>, grid, dim3(256), 0, (hipStream_t)stream, g);
    else hipLaunchKernelGGL(bf16_gemm_kernel<HERO_F16>, grid, dim3(256), 0, (hipStream_t)stream, g);
    return hero_launch_status();
}

extern "C" hero_status hero_hp_gemm(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                                    const float* bias, const void* residual, int64_t ldr, int gelu,
                                    void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, void* stream) {
    return run_hp_gemm(A, lda, Wt, ldb, bias, residual, ldr, gelu, C, ldc, M, N, K, dt, stream, -1);
}

extern "C" hero_status hero_bf16_gemm(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                                      const float* bias, const void* residual, int64_t ldr, int gelu,
                                      void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    return run_hp_gemm(A, lda, Wt, ldb, bias, residual, ldr, gelu, C, ldc, M, N, K, HERO_BF16, stream, -1);
}

// Test and tuning hook (include/hero_debug.h): tile 7 / 8 = the persistent 256x256 / 128x128 kernel, 0 = the plain one.
extern "C" hero_status hero_hp_gemm_tile(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                                         const float* bias, const void* residual, int64_t ldr, int gelu,
                                         void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, void* stream, int tile) {
    if (tile != 0 && tile != 7 && tile != 8) return HERO_ERR_UNSUPPORTED;
    return run_hp_gemm(A, lda, Wt, ldb, bias, residual, ldr, gelu, C, ldc, M, N, K, dt, stream, tile);
}

extern "C" hero_status hero_bf16_attn(const void* q, const int64_t q_strides[4],
                                      const void* k, const int64_t k_strides[4],
                                      const void* v, const int64_t v_strides[4],
                                      int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                                      hero_mask mask, const int32_t* kv_len, void* out, int64_t ldo, void* stream) {
    return hero_hp_attn(q, q_strides, k, k_strides, v, v_strides, B, H, Sq, Skv, Dh, scale, mask, kv_len, out, ldo, HERO_BF16, stream);
}

extern "C" hero_status hero_hp_attn(const void* q, const int64_t q_strides[4],
                                    const void* k, const int64_t k_strides[4],
                                    const void* v, const int64_t v_strides[4],
                                    int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                                    hero_mask mask, const int32_t* kv_len, void* out, int64_t ldo, hero_dtype dt, void* stream) {
    if (dt != HERO_BF16 && dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (B < 0 || H < 0 || Sq < 0 || Skv < 0) return HERO_ERR_SHAPE;
    if (Dh != 64 && Dh != 128) return HERO_ERR_UNSUPPORTED;
    if (mask != HERO_MASK_NONE && mask != HERO_MASK_PADDING && mask != HERO_MASK_CAUSAL) return HERO_ERR_UNSUPPORTED;
    if (B == 0 || H == 0 || Sq == 0) return HERO_OK;
    if (!out || !q_strides || !k_strides || !v_strides) return HERO_ERR_NULL;
    if (Skv > 0 && (!q || !k || !v)) return HERO_ERR_NULL;
    if (mask == HERO_MASK_PADDING && !kv_len) return HERO_ERR_NULL;
    if (ldo < H * Dh) return HERO_ERR_SHAPE;
    if (B > 65535 || H > 65535 || Sq > 0x7fffffffLL || Skv > 0x7fffffffLL) return HERO_ERR_SHAPE;
    const int64_t* ss[3] = {q_strides, k_strides, v_strides};
    for (int t = 0; t < 3; ++t) {
        if (ss[t][3] != 1) return HERO_ERR_UNSUPPORTED;
        if (ss[t][0] % 8 || ss[t][1] % 8 || ss[t][2] % 8) return HERO_ERR_ALIGN;
    }
    if (ldo % 4 || !hero_aligned16(out) || !hero_aligned16(q) || !hero_aligned16(k) || !hero_aligned16(v)) return HERO_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (Skv == 0) {
        const int64_t n = B * Sq * H * Dh;
        hipLaunchKernelGGL(zero_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint16_t*)out, B * Sq, H * Dh, ldo);
        return hero_launch_status();
    }
    BAttnArgs a;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    for (int t = 0; t < 4; ++t) { a.qs[t] = q_strides[t]; a.ks[t] = k_strides[t]; a.vs[t] = v_strides[t]; }
    a.B = (int)B; a.H = (int)H; a.Sq = (int)Sq; a.Skv = (int)Skv; a.scale = scale; a.mask = (int)mask; a.kv_len = kv_len;
    a.out = (uint16_t*)out; a.ldo = ldo;
    const int64_t nblocks = ((B * H + 7) / 8) * 8 * ((Sq + ABQ - 1) / ABQ);   // whole rounds of 8 heads, one per XCD
    if (nblocks > 0x7fffffffLL) return HERO_ERR_SHAPE;
    dim3 grid((unsigned)nblocks);
    if (dt == HERO_BF16) {
        if (Dh == 64) hipLaunchKernelGGL((bf16_attn_kernel<64, HERO_BF16>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((bf16_attn_kernel<128, HERO_BF16>), grid, dim3(256), 0, st, a);
    } else {
        if (Dh == 64) hipLaunchKernelGGL((bf16_attn_kernel<64, HERO_F16>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((bf16_attn_kernel<128, HERO_F16>), grid, dim3(256), 0, st, a);
    }
    return hero_launch_status();
}
