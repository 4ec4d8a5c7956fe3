// hero_int8_gemm: GeMM^quant, INT8 x INT8 -> INT32 on the gfx950 matrix cores with the
// dequantization / static-scale / bias / GELU / residual / requantization epilogue fused
// behind the accumulators (paper Sec. 2.1 GEMM convention and column-wise weight scales;
// Sec. 2.2.2 fused dequantization and the bare Round after folding; Sec. 2.2.3 GELU^quant).
//
// Both operands are K-contiguous ([M][K] activations, [N][K] weights), so every MFMA
// operand fragment is one 128-bit LDS read.  MFMA: v_mfma_i32_32x32x32_i8 with the WEIGHT
// fragment as first operand and the activation fragment as second, so the accumulator of
// lane l holds, for ONE output row m = l % 32, the columns n = 8g + 4(l/32) + t (register
// 4g + t): the per-row scale is one register and a lane owns 4 consecutive columns.
//
// Three main loops share one epilogue:
//   * int8_gemm_persistent_kernel (large problems): 256x256 block tile, 8 waves of 128x64,
//     slabs of 64 bytes of K copied global -> LDS directly (global_load_lds_dwordx4) through
//     a ring of 4 stages; one workgroup per CU walks its tiles and the ring runs through the
//     tile boundaries.  A second form, 128x128 with 4 waves of 64x64 and two workgroups per CU,
//     serves the sizes at which the large tile would leave CUs idle; per tile area it needs
//     twice the L2 -> LDS traffic and is 10-15 % slower once every CU has work.
//   * int8_gemm_dma_kernel: the same tile, one tile per workgroup (short K, huge strides).
//   * int8_gemm_kernel (small or skinny problems): 128x128 / 64x64 tile staged through registers.
// The epilogue works in registers: a lane-half exchange (v_permlane32_swap) gives every lane a
// contiguous piece of one output row, written with 128-bit stores.
#include "hero_common.h"
#include <atomic>
#include <cstdlib>
#include <type_traits>

namespace {

constexpr int KMULT = 64;       // K must be a multiple of this
constexpr int BK = 64;          // bytes of K per LDS slab
constexpr int LDS_LD = BK + 16; // padded slab row stride of the register-staged kernel
constexpr int GROUP_M = 8;      // tile order: 8 row panels x 8 column panels run together on one XCD
constexpr int NUM_XCD = 8;

struct GemmArgs {
    const int8_t* A; int64_t lda; const float* a_row_scale;
    const int8_t* Bt; int64_t ldb; const float* b_col_scale;
    const float* bias; const void* residual; int64_t ldr;
    const float* out_col_scale;
    void* C; int64_t ldc;
    int M, N, K;
    int ntm, ntn, per_xcd;      // tile grid and tiles per XCD
    // split-K (skinny M): blockIdx.y picks a range of kslabs slabs and writes raw int32 partial sums
    // to its own [M][ldc] plane of C (plane stride M * ldc elements); a second kernel adds the planes
    int ksplit, kslabs;
    // optional (persistent kernels only): memory the NEXT kernel of the caller's chain will read (a layer's next weight
    // matrix).  Every tile requests pf_lpt of its pf_lines 128-byte lines once, at the start of its epilogue.
    const int8_t* pf = nullptr; int pf_lines = 0, pf_lpt = 0;
};

// Operand types of the main loops.  ADT = HERO_I8: INT8 operands, int32 accumulators.  ADT = HERO_BF16: bf16
// operands (the BF16 side of a switched module, Sec. 2.3 / Table 1), fp32 accumulators, no scales; K, lda and ldb
// are then in BYTES, and a 64-byte slab holds two v_mfma_f32_32x32x16_bf16 steps exactly as it holds two INT8
// steps.  ADT = HERO_F8E4M3: the FP8 variant (Sec. 2.1), fp32 accumulators, the INT8 epilogue; a 16-byte
// fragment feeds two v_mfma_f32_32x32x16_fp8_fp8 (its low and its high 8 bytes: any grouping of K is a valid
// contraction as long as both operands use the same one).
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8hf __attribute__((ext_vector_type(8)));
template <int ADT, typename ACC>
__device__ __forceinline__ ACC mfma_step(v4i a, v4i b, ACC c) {
    if constexpr (ADT == HERO_I8) return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    else if constexpr (ADT == HERO_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    else if constexpr (ADT == HERO_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8hf, a), __builtin_bit_cast(v8hf, b), c, 0, 0, 0);
    else {
        const long a0 = (long)(((uint64_t)(uint32_t)a[1] << 32) | (uint32_t)a[0]), a1 = (long)(((uint64_t)(uint32_t)a[3] << 32) | (uint32_t)a[2]);
        const long b0 = (long)(((uint64_t)(uint32_t)b[1] << 32) | (uint32_t)b[0]), b1 = (long)(((uint64_t)(uint32_t)b[3] << 32) | (uint32_t)b[2]);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a0, b0, c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a1, b1, c, 0, 0, 0);
    }
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) { f(std::integral_constant<int, I>{}); static_for<N, I + 1>(f); }
}
template <int ADT> struct AccOf { using type = typename std::conditional<ADT == HERO_I8, v16i, v16f>::type; };

template <int CDT> struct ElemSize { static constexpr int v = CDT == HERO_I32 ? 4 : ((CDT == HERO_I8 || CDT == HERO_F8E4M3) ? 1 : 2); };

// XCD-aware tile order: workgroups go round-robin to the 8 XCDs, so XCD x takes the
// contiguous range [x * per_xcd, (x+1) * per_xcd) of a grouped order in which 64
// consecutive tiles form an 8 x 8 square of panels (operands shared through that XCD's L2).
template <int BM, int BN>
__device__ __forceinline__ void tile_from_seq(const GemmArgs& g, int seq, int& m0, int& n0) {
    const int grp = seq / (GROUP_M * g.ntn), rem = seq % (GROUP_M * g.ntn);
    const int gsize = min(g.ntm - grp * GROUP_M, GROUP_M);
    m0 = (grp * GROUP_M + rem % gsize) * BM;
    n0 = (rem / gsize) * BN;
}
template <int BM, int BN>
__device__ __forceinline__ bool tile_origin(const GemmArgs& g, int& m0, int& n0) {
    const int seq = (blockIdx.x % NUM_XCD) * g.per_xcd + blockIdx.x / NUM_XCD;
    if (seq >= g.ntm * g.ntn) return false;
    tile_from_seq<BM, BN>(g, seq, m0, n0);
    return true;
}

// Per-column epilogue vectors of the tile -> LDS ([3][BN] floats: column scale, bias,
// output scale), issued before the main loop so their latency hides behind it.
template <int BN, int NT, int EPI>
__device__ __forceinline__ void stage_col_vectors(const GemmArgs& g, float* sv, int n0, int tid) {
    if (EPI == HERO_EPI_RAW_I32) return;
    for (int c = tid; c < BN; c += NT) {
        const int n = min(n0 + c, g.N - 1);
        sv[c] = g.b_col_scale[n];
        sv[BN + c] = g.bias ? g.bias[n] : 0.0f;
        if (EPI == HERO_EPI_GELU_REQUANT) sv[2 * BN + c] = __fdiv_rn(1.0f, g.out_col_scale[n]);   // 1 / S_a[j]
    }
}

// ---- direct epilogue ---------------------------------------------------------------------------
// No LDS: after the fp32 epilogue a lane holds, for ONE output row, 4-column groups q (columns
// 8q + 4hh .. + 3 of the wave's 32*TN columns).  v_permlane32_swap exchanges the groups q >= NQ/2
// of lanes 0..31 with the groups q < NQ/2 of lanes 32..63, after which lane l < 32 owns the
// row's first 16*TN columns and lane l + 32 the other 16*TN, contiguous in registers: every lane
// writes one contiguous piece of its row (32 B of INT8 codes, 64 B of 16-bit values for TN = 2)
// with 128-bit stores, and the residual of the fused add is read in the same layout.
__device__ __forceinline__ void swap32(uint32_t a, uint32_t b, uint32_t& lo, uint32_t& hi) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);   // r[0] = {a.low, b.low}, r[1] = {a.high, b.high}
    lo = r[0]; hi = r[1];
}
// ND dwords of one row, first column col (ES bytes per element), bounds-checked against N unless `full`
template <int ES, int ND>
__device__ __forceinline__ void store_piece(int8_t* cp, const uint32_t (&d)[ND], int col, int N, bool full, bool al16) {
    constexpr int EPD = 4 / ES;                                     // elements per dword
    if (full) {
        if (al16) {
#pragma unroll
            for (int k = 0; k < ND / 4; ++k) {
                v4i o = {(int)d[4 * k], (int)d[4 * k + 1], (int)d[4 * k + 2], (int)d[4 * k + 3]};
                *reinterpret_cast<v4i*>(cp + 16 * k) = o;
            }
        } else {
#pragma unroll
            for (int k = 0; k < ND; ++k) *reinterpret_cast<uint32_t*>(cp + 4 * k) = d[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            const int c = col + k * EPD;
            if (c + EPD <= N) *reinterpret_cast<uint32_t*>(cp + 4 * k) = d[k];
            else if (ES < 4) {
#pragma unroll
                for (int b = 0; b < EPD; ++b)
                    if (c + b < N) {
                        if (ES == 1) cp[4 * k + b] = (int8_t)(d[k] >> (8 * b));
                        else *reinterpret_cast<uint16_t*>(cp + 4 * k + 2 * b) = (uint16_t)(d[k] >> (16 * b));
                    }
            }
        }
    }
}

// ACC is v16i (INT8 operands) or v16f (bf16 operands: UNIT, no scales, y = acc + bias).
template <int BM, int BN, int WM, int WN, int EPI, int CDT, int RDT, bool OS_RAW = false, bool UNIT = false, typename ACC = v16i>
__device__ __forceinline__ void epilogue_direct(const GemmArgs& g, ACC (&acc)[BM / WM / 32][BN / WN / 32],
                                                const float* sv, const float (&rsr)[BM / WM / 32],
                                                int m0, int n0, int tid) {
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NQ = TN * 4, H = NQ / 2;
    constexpr bool FUSE_RES = RDT >= 0;
    constexpr int ES = ElemSize<CDT>::v;
    const int lane = tid & 63, wave = tid >> 6, wm = wave / WN, wn = wave % WN;
    const int hh = lane >> 5, ml = lane & 31;
    const bool has_rs = g.a_row_scale != nullptr;
    const int colw = n0 + wn * TN * 32;                            // first column of this wave
    const int col0 = colw + hh * H * 8;                            // first column this lane stores (after the swap)
    const bool al16 = (g.ldc * ES) % 16 == 0;
    const bool full = col0 + H * 8 <= g.N;

    // per-column vectors of this lane's 4-column groups, from LDS into registers once
    v4f cs[NQ], bs[NQ];
    if (EPI != HERO_EPI_RAW_I32) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int nl = wn * TN * 32 + q * 8 + hh * 4;
            if (!UNIT) cs[q] = *reinterpret_cast<const v4f*>(sv + nl);
            bs[q] = *reinterpret_cast<const v4f*>(sv + BN + nl);
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * TM * 32 + i * 32 + ml;
        const bool rowok = row < g.M;
        const float rs = rsr[i];
        if constexpr (EPI == HERO_EPI_RAW_I32) {                  // 16 bytes per group: stored as they are
            if (rowok) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int j = q >> 2, gq = q & 3, col = colw + q * 8 + hh * 4;
                    const uint32_t d[4] = {(uint32_t)acc[i][j][4 * gq], (uint32_t)acc[i][j][4 * gq + 1],
                                           (uint32_t)acc[i][j][4 * gq + 2], (uint32_t)acc[i][j][4 * gq + 3]};
                    if (col < g.N) store_piece<4, 4>((int8_t*)g.C + ((int64_t)row * g.ldc + col) * 4, d, col, g.N, col + 4 <= g.N, al16);
                }
            }
        } else {
            float y[NQ][4];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int j = q >> 2, gq = q & 3;
                v4f os;                                           // 1 / S_a of the group, re-read per pass (registers)
                if (EPI == HERO_EPI_GELU_REQUANT) {
                    int nl = wn * TN * 32 + q * 8 + hh * 4;
                    asm volatile("" : "+v"(nl));                  // opaque: one load per pass, not one long-lived copy
                    os = *reinterpret_cast<const v4f*>(sv + 2 * BN + nl);
                    if (OS_RAW)                                   // the vector holds S_a itself: hardware reciprocal (1 ulp; +-1 LSB class)
#pragma unroll
                        for (int t = 0; t < 4; ++t) os[t] = __builtin_amdgcn_rcpf(os[t]);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    float v = (float)acc[i][j][4 * gq + t];
                    if (UNIT) v = v + bs[q][t];
                    else {
                        if (has_rs) v = v * rs;
                        v = fmaf(v, cs[q][t], bs[q][t]);
                    }
                    if (EPI == HERO_EPI_DEQUANT_GELU || EPI == HERO_EPI_GELU_REQUANT) v = gelu_erf(v);
                    // GELU^quant is in the +-1 LSB class (fp32 GELU vs the definition's fp64), so the
                    // division by S_a[j] is a multiplication by its reciprocal
                    if (EPI == HERO_EPI_GELU_REQUANT) v = v * os[t];
                    y[q][t] = v;
                }
            }
            if constexpr (ES == 1) {
                uint32_t w[NQ], d[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q)
                    w[q] = CDT == HERO_F8E4M3 ? fp8x4_sat(y[q][0], y[q][1], y[q][2], y[q][3]) : quant4_sat(y[q][0], y[q][1], y[q][2], y[q][3]);
#pragma unroll
                for (int q = 0; q < H; ++q) swap32(w[q], w[q + H], d[2 * q], d[2 * q + 1]);
                if (rowok && col0 < g.N) store_piece<1, NQ>((int8_t*)g.C + (int64_t)row * g.ldc + col0, d, col0, g.N, full, al16);
            } else if constexpr (!FUSE_RES) {
                uint32_t d[2 * NQ];
#pragma unroll
                for (int q = 0; q < H; ++q) {
                    const uint32_t a0 = pack2_hp<CDT>(y[q][0], y[q][1]), a1 = pack2_hp<CDT>(y[q][2], y[q][3]);
                    const uint32_t b0 = pack2_hp<CDT>(y[q + H][0], y[q + H][1]), b1 = pack2_hp<CDT>(y[q + H][2], y[q + H][3]);
                    swap32(a0, b0, d[4 * q], d[4 * q + 2]);
                    swap32(a1, b1, d[4 * q + 1], d[4 * q + 3]);
                }
                if (rowok && col0 < g.N) store_piece<2, 2 * NQ>((int8_t*)g.C + ((int64_t)row * g.ldc + col0) * 2, d, col0, g.N, full, al16);
            } else {
                // fused residual: the fp32 values change lanes, the residual is read in the stored layout
                uint32_t z[H][8], d[2 * NQ];
#pragma unroll
                for (int q = 0; q < H; ++q)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        swap32(__float_as_uint(y[q][t]), __float_as_uint(y[q + H][t]), z[q][t], z[q][4 + t]);
                if (rowok && col0 < g.N) {
                    const uint16_t* rp = (const uint16_t*)g.residual + (int64_t)row * g.ldr + col0;
                    const bool rl16 = (g.ldr * 2) % 16 == 0;
#pragma unroll
                    for (int q = 0; q < H; ++q) {
                        uint32_t r[4];
                        if (full && rl16) {
                            v4i rv = *reinterpret_cast<const v4i*>(rp + 8 * q);
                            r[0] = rv[0]; r[1] = rv[1]; r[2] = rv[2]; r[3] = rv[3];
                        } else {
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const int c = col0 + 8 * q + 2 * k;
                                const uint32_t e0 = c < g.N ? rp[8 * q + 2 * k] : 0, e1 = c + 1 < g.N ? rp[8 * q + 2 * k + 1] : 0;
                                r[k] = e0 | (e1 << 16);
                            }
                        }
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            d[4 * q + k] = pack2_hp<CDT>(__uint_as_float(z[q][2 * k]) + hp_to_f32<RDT>(r[k] & 0xffffu),
                                                         __uint_as_float(z[q][2 * k + 1]) + hp_to_f32<RDT>(r[k] >> 16));
                        }
                    }
                    store_piece<2, 2 * NQ>((int8_t*)g.C + ((int64_t)row * g.ldc + col0) * 2, d, col0, g.N, full, al16);
                }
            }
        }
    }
}

// =====================================================================================
// Register-staged main loop (small / ragged problems).  BK-byte slabs, double-buffered in
// LDS with an 80-byte padded row stride, PD slabs in flight in registers.
// =====================================================================================
// KG > 1: KG groups of WM x WN waves share the tile and split K among themselves (every group has its own
// slab buffers and runs the same number of iterations, so the barriers stay workgroup-wide); the groups'
// accumulators are added through LDS before the epilogue.  For small problems with a long K: the number of
// workgroups is fixed by M and N, more waves per workgroup shorten the K loop.
template <int BM, int BN, int WM, int WN, int PD, int MINW, int EPI, int CDT, int RDT, bool SPLITK = false, int KG = 1, int ADT = HERO_I8>
__global__ __launch_bounds__(WM * WN * 64 * KG, MINW) void int8_gemm_kernel(GemmArgs g) {
    using ACC = typename AccOf<ADT>::type;
    static_assert(ADT == HERO_I8 || !SPLITK, "split K over workgroups: integer partial sums only");
    constexpr int NT = WM * WN * 64;                          // threads of one K group
    constexpr int CPR = BK / 16;                              // 16-byte chunks per slab row
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;      // 32x32 MFMA tiles per wave
    constexpr int A_UNITS = BM * CPR / NT, B_UNITS = BN * CPR / NT;
    static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads mismatch");
    static_assert(PD % 2 == 0, "prefetch distance must be even (LDS buffer parity is compile-time)");
    constexpr int POOL = 2 * (BM + BN) * LDS_LD;
    static_assert(KG == 1 || (!SPLITK && BM * BN * 4 <= POOL), "K groups: one tile of accumulators must fit a group's slab buffers");
    __shared__ __attribute__((aligned(16))) int8_t smem[KG * POOL + 3 * BN * 4];
    const int kg = KG == 1 ? 0 : (int)threadIdx.x / NT;       // K group of this wave
    int8_t* const sA0 = smem + kg * POOL;                     // [2][BM * LDS_LD]
    int8_t* const sB0 = sA0 + 2 * BM * LDS_LD;                // [2][BN * LDS_LD]
    float* const sv = reinterpret_cast<float*>(smem + KG * POOL);

    const int tid = KG == 1 ? (int)threadIdx.x : (int)threadIdx.x % NT, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int m0, n0;
    if (!tile_origin<BM, BN>(g, m0, n0)) return;
    // this group's slabs: all of K, the blockIdx.y-th range of kslabs slabs (never empty), or the kg-th
    // of KG equal ranges (the launch requires K / BK to be a multiple of KG)
    const int kt0 = SPLITK ? (int)blockIdx.y * g.kslabs : kg * (g.K / BK / KG);
    const int KT = SPLITK ? min(g.kslabs, g.K / BK - kt0) : g.K / BK / KG;

    stage_col_vectors<BN, NT * KG, EPI>(g, sv, n0, (int)threadIdx.x);
    float rsr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
        rsr[i] = (EPI != HERO_EPI_RAW_I32 && g.a_row_scale) ? g.a_row_scale[min(m0 + wm * TM * 32 + i * 32 + (lane & 31), g.M - 1)] : 1.0f;

    // global -> register -> LDS staging.  Unit u of this thread is slab row idx / CPR,
    // 16-byte chunk idx % CPR.  PD slabs are in flight in registers ahead of the one in LDS.
    const int8_t* pa[A_UNITS];
    const int8_t* pb[B_UNITS];
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
        int idx = tid + u * NT, row = idx / CPR, ch = idx % CPR;
        pa[u] = g.A + (int64_t)min(m0 + row, g.M - 1) * g.lda + ch * 16 + (int64_t)kt0 * BK;   // clamp: ragged M
    }
#pragma unroll
    for (int u = 0; u < B_UNITS; ++u) {
        int idx = tid + u * NT, row = idx / CPR, ch = idx % CPR;
        pb[u] = g.Bt + (int64_t)min(n0 + row, g.N - 1) * g.ldb + ch * 16 + (int64_t)kt0 * BK;
    }
    const int lds_unit0 = (tid / CPR) * LDS_LD + (tid % CPR) * 16;                // + u * (NT / CPR) * LDS_LD
    v4i ra[PD][A_UNITS], rb[PD][B_UNITS];
    auto load_slab = [&](int kt, int p) {
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u) ra[p][u] = *reinterpret_cast<const v4i*>(pa[u] + (int64_t)kt * BK);
#pragma unroll
        for (int u = 0; u < B_UNITS; ++u) rb[p][u] = *reinterpret_cast<const v4i*>(pb[u] + (int64_t)kt * BK);
    };
    auto store_slab = [&](int buf, int p) {
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u)
            *reinterpret_cast<v4i*>(sA0 + buf * BM * LDS_LD + lds_unit0 + u * (NT / CPR) * LDS_LD) = ra[p][u];
#pragma unroll
        for (int u = 0; u < B_UNITS; ++u)
            *reinterpret_cast<v4i*>(sB0 + buf * BN * LDS_LD + lds_unit0 + u * (NT / CPR) * LDS_LD) = rb[p][u];
    };

    ACC acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Every load is unconditional (slab indices are clamped to the last slab, whose
    // redundant copies are never read): with no branch between a load and its use the
    // compiler can wait for exactly the oldest register set and leave the younger ones
    // in flight.
    const int last = KT - 1;
    load_slab(0, 0);
    store_slab(0, 0);
#pragma unroll
    for (int p = 0; p < PD; ++p) load_slab(min(1 + p, last), p);  // slab s waits in register set (s-1) % PD
    __syncthreads();
    const int frag_a = (wm * TM * 32 + (lane & 31)) * LDS_LD + (lane >> 5) * 16;
    const int frag_b = (wn * TN * 32 + (lane & 31)) * LDS_LD + (lane >> 5) * 16;
    // One slab.  The body is written in the issue order wanted and pinned with scheduling
    // barriers: every MFMA is followed by at most one LDS read, one LDS write or one global
    // load.  A wave issues in order, and a burst of vector-memory instructions stalls it in
    // front of its next MFMA while the address unit drains; spread out, the memory
    // instructions issue in the shadow of the 32-cycle MFMAs.
    constexpr int NM = TM * TN, NFR = TM + TN, NW = A_UNITS + B_UNITS;
    auto iteration = [&](int kt, int buf, auto U) {
        constexpr int u = decltype(U)::value;
        const int8_t* sa = sA0 + buf * BM * LDS_LD + frag_a;
        const int8_t* sb = sB0 + buf * BN * LDS_LD + frag_b;
        int8_t* wa = sA0 + (buf ^ 1) * BM * LDS_LD + lds_unit0;
        int8_t* wb = sB0 + (buf ^ 1) * BN * LDS_LD + lds_unit0;
        const int64_t koff = (int64_t)min(kt + 1 + PD, last) * BK;
        v4i f0[NFR], f1[NFR];                                     // fragments of k-step 0 / 1: B tiles first, then A tiles
#pragma unroll
        for (int t = 0; t < NFR; ++t)
            f0[t] = *reinterpret_cast<const v4i*>((t < TN ? sb + t * 32 * LDS_LD : sa + (t - TN) * 32 * LDS_LD));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NM; ++n) {                             // k-step 0; memory instructions dealt round-robin
            const int jj = n / TM, ii = n % TM;
            acc[ii][jj] = mfma_step<ADT>(f0[jj], f0[TN + ii], acc[ii][jj]);
#pragma unroll
            for (int t = n; t < NFR; t += NM)
                f1[t] = *reinterpret_cast<const v4i*>((t < TN ? sb + t * 32 * LDS_LD : sa + (t - TN) * 32 * LDS_LD) + 32);
#pragma unroll
            for (int t = n; t < NW; t += NM) {                     // slab kt + 1 from register set u into LDS
                if (t < A_UNITS) *reinterpret_cast<v4i*>(wa + t * (NT / CPR) * LDS_LD) = ra[u][t];
                else *reinterpret_cast<v4i*>(wb + (t - A_UNITS) * (NT / CPR) * LDS_LD) = rb[u][t - A_UNITS];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int n = 0; n < NM; ++n) {                             // k-step 1
            const int jj = n / TM, ii = n % TM;
            acc[ii][jj] = mfma_step<ADT>(f1[jj], f1[TN + ii], acc[ii][jj]);
#pragma unroll
            for (int t = n; t < NW; t += NM) {                     // slab kt + 1 + PD into the freed register set
                if (t < A_UNITS) ra[u][t] = *reinterpret_cast<const v4i*>(pa[t] + koff);
                else rb[u][t - A_UNITS] = *reinterpret_cast<const v4i*>(pb[t - A_UNITS] + koff);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };
    // PD iterations per trip, one per register set (the set index and the LDS buffer parity are compile-time);
    // the tail runs the first KT % PD of them
    int kt = 0;
    auto trip = [&](auto FULL) {
        static_for<PD>([&](auto U) {
            constexpr int u = decltype(U)::value;
            if (decltype(FULL)::value || kt + u < KT) iteration(kt + u, u & 1, U);
        });
    };
    for (; kt + PD <= KT; kt += PD) trip(std::true_type{});
    if (kt < KT) trip(std::false_type{});
    if constexpr (KG > 1) {
        // groups 1 .. KG-1 hand their accumulators to group 0 (register-major, lane-minor: no bank conflicts);
        // the loop's last barrier has released every group's slab buffers.  Integer sums are exact in any order;
        // the fp32 sums of the FP8 variant are added in the fixed order group 0, 1, .., KG-1.
        using V4 = typename std::conditional<ADT == HERO_I8, v4i, v4f>::type;
        constexpr int NV = TM * TN * 4;
        V4* const mine = reinterpret_cast<V4*>(smem + kg * POOL) + (wave * NV) * 64 + lane;
        if (kg > 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int ij = v >> 2, c = (v & 3) * 4;
                mine[v * 64] = V4{acc[ij / TN][ij % TN][c], acc[ij / TN][ij % TN][c + 1], acc[ij / TN][ij % TN][c + 2], acc[ij / TN][ij % TN][c + 3]};
            }
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int k = 1; k < KG; ++k) {
            const V4* other = reinterpret_cast<const V4*>(smem + k * POOL) + (wave * NV) * 64 + lane;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int ij = v >> 2, c = (v & 3) * 4;
                const V4 o = other[v * 64];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[ij / TN][ij % TN][c + e] += o[e];
            }
        }
    }
    if constexpr (SPLITK && ADT == HERO_I8) {
        static_assert(EPI == HERO_EPI_RAW_I32, "split-K writes raw partial sums");
        GemmArgs gp = g;
        gp.C = (int32_t*)g.C + (int64_t)blockIdx.y * g.M * g.ldc;
        epilogue_direct<BM, BN, WM, WN, EPI, CDT, RDT>(gp, acc, sv, rsr, m0, n0, tid);
        return;
    }
    epilogue_direct<BM, BN, WM, WN, EPI, CDT, RDT, false, false>(g, acc, sv, rsr, m0, n0, tid);
}

// =====================================================================================
// Direct-to-LDS main loop (large problems).  A wave-level global_load_lds_dwordx4 writes
// 1 KB of consecutive LDS, so slab rows are 64 bytes, unpadded, and the four 16-byte chunks
// of row r are stored at position c ^ ((r >> 2) & 3): the 128-bit fragment reads of 16
// consecutive rows then fall into 16 different 16-byte bank groups.
// =====================================================================================
// s_waitcnt immediate that waits only for vmcnt <= n (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// One direct global->LDS load: 64 lanes x 16 bytes land at LDS address lds_base + lane * 16
// (lds_base is wave-uniform and travels in M0).  Written as inline assembly on purpose: the
// compiler then does not track these loads and does not force vmcnt(0) in front of every LDS
// read; the kernel waits for exactly the slab it is about to read (vmcnt counts them in order).
__device__ __forceinline__ void dma16(const int8_t* gp, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gp), "s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)((const __attribute__((address_space(3))) void*)p);
}

template <int BM, int BN, int WM, int WN, int NS, int MINW, int EPI, int CDT, int RDT>
__global__ __launch_bounds__(WM * WN * 64, MINW) void int8_gemm_dma_kernel(GemmArgs g) {
    constexpr int NT = WM * WN * 64, NWAVE = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    constexpr int A_UNITS = A_BYTES / 16 / NT, B_UNITS = B_BYTES / 16 / NT, NW = A_UNITS + B_UNITS;
    constexpr int NM = TM * TN, NFR = TM + TN;
    static_assert(NS >= 3, "ring needs at least three stages");
    static_assert(NW <= NM && NFR <= NM, "interleave plan needs one slot per memory instruction");
    constexpr int POOL = NS * STAGE;
    __shared__ __attribute__((aligned(1024))) int8_t smem[POOL + 3 * BN * 4];
    float* const sv = reinterpret_cast<float*>(smem + POOL);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int m0, n0;
    if (!tile_origin<BM, BN>(g, m0, n0)) return;
    const int KT = g.K / BK, last = KT - 1;

    stage_col_vectors<BN, NT, EPI>(g, sv, n0, tid);
    float rsr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
        rsr[i] = (EPI != HERO_EPI_RAW_I32 && g.a_row_scale) ? g.a_row_scale[min(m0 + wm * TM * 32 + i * 32 + (lane & 31), g.M - 1)] : 1.0f;

    // loader: unit u of wave w fills LDS granules [(u * NWAVE + w) * 64, +64) of the A (or B)
    // part of a stage; lane l owns granule q = that + l  ->  row q / 4, stored chunk q % 4,
    // which holds global chunk (q % 4) ^ ((row >> 2) & 3).
    const int8_t* pa[A_UNITS];
    const int8_t* pb[B_UNITS];
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
        const int q = (u * NWAVE + wave) * 64 + lane, row = q >> 2, c = (q & 3) ^ ((row >> 2) & 3);
        pa[u] = g.A + (int64_t)min(m0 + row, g.M - 1) * g.lda + c * 16;
    }
#pragma unroll
    for (int u = 0; u < B_UNITS; ++u) {
        const int q = (u * NWAVE + wave) * 64 + lane, row = q >> 2, c = (q & 3) ^ ((row >> 2) & 3);
        pb[u] = g.Bt + (int64_t)min(n0 + row, g.N - 1) * g.ldb + c * 16;
    }
    const uint32_t wbase = __builtin_amdgcn_readfirstlane(lds_offset(smem) + wave * 1024);   // + stage * STAGE + unit offset
    auto issue = [&](int n, int kt, int stage) {        // the n-th direct load of slab kt
        const int64_t koff = (int64_t)min(kt, last) * BK;
        if (n < A_UNITS) dma16(pa[n] + koff, wbase + stage * STAGE + n * NWAVE * 1024);
        else dma16(pb[n - A_UNITS] + koff, wbase + stage * STAGE + A_BYTES + (n - A_UNITS) * NWAVE * 1024);
    };
    // fragment offsets inside a stage (row rr, k-step ks, half hh): rr*64 + ((2ks+hh) ^ ((rr>>2)&3))*16
    const int hh = lane >> 5, ml = lane & 31;
    int fo[2][NFR];
#pragma unroll
    for (int t = 0; t < NFR; ++t) {
        const int rr = (t < TN ? wn * TN * 32 + t * 32 : wm * TM * 32 + (t - TN) * 32) + ml;
        const int base = (t < TN ? A_BYTES : 0) + rr * 64;
        fo[0][t] = base + (((0 + hh) ^ ((rr >> 2) & 3)) << 4);
        fo[1][t] = base + (((2 + hh) ^ ((rr >> 2) & 3)) << 4);
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // prologue: slabs 0 .. NS-2 in flight, slab 0 landed, its k-step-0 fragments in registers
#pragma unroll
    for (int s0 = 0; s0 < NS - 1; ++s0)
#pragma unroll
        for (int n = 0; n < NW; ++n) issue(n, s0, s0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * NW));
    __syncthreads();
    v4i f0[NFR], f1[NFR];
#pragma unroll
    for (int t = 0; t < NFR; ++t) f0[t] = *reinterpret_cast<const v4i*>(smem + fo[0][t]);

    // One slab per iteration; the barrier sits in the MIDDLE: k-step 0 runs on fragments read
    // during the previous slab, the barrier then makes slab kt+1 visible, and k-step 1 runs
    // while the first fragments of slab kt+1 and the direct loads of slab kt+NS-1 are issued,
    // one memory instruction per MFMA.
    int stage = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int8_t* st = smem + stage * STAGE;
        const int nstage = stage + 1 == NS ? 0 : stage + 1;      // slab kt + 1
        const int pstage = stage == 0 ? NS - 1 : stage - 1;      // slab kt - 1 == slab kt + NS - 1
        const int8_t* stn = smem + nstage * STAGE;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NM; ++n) {                             // k-step 0
            const int jj = n / TM, ii = n % TM;
            acc[ii][jj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f0[jj], f0[TN + ii], acc[ii][jj], 0, 0, 0);
            if (n < NFR) f1[n] = *reinterpret_cast<const v4i*>(st + fo[1][n]);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 3) * NW));     // slab kt + 1 has landed (mine)
        __syncthreads();                                           // ... and everybody's
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NM; ++n) {                             // k-step 1
            const int jj = n / TM, ii = n % TM;
            acc[ii][jj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f1[jj], f1[TN + ii], acc[ii][jj], 0, 0, 0);
            if (n < NFR) f0[n] = *reinterpret_cast<const v4i*>(stn + fo[0][n]);
            if (n < NW) issue(n, kt + NS - 1, pstage);
            __builtin_amdgcn_sched_barrier(0);
        }
        stage = nstage;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                      // the redundant tail loads
    __syncthreads();
    epilogue_direct<BM, BN, WM, WN, EPI, CDT, RDT>(g, acc, sv, rsr, m0, n0, tid);
}

// =====================================================================================
// Persistent variant of the direct-to-LDS kernel (large problems): one
// workgroup per CU walks a strided list of tiles, and the slab ring runs straight through
// the tile boundaries, so the first slabs of the next tile (and its per-column / per-row
// epilogue vectors, fetched by the same direct loads into a double-buffered LDS area) are
// already resident when the epilogue of the current tile ends.  Slab addresses are a wave-uniform tile base in SGPRs
// plus a per-lane 32-bit offset, so advancing along K is scalar arithmetic.
// =====================================================================================
__device__ __forceinline__ void dma16s(uint32_t voff, const int8_t* sbase, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ void dma4s(uint32_t voff, const float* sbase, uint32_t lds_base) {   // lane l -> lds_base + 4 l
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory", "m0");
}

template <int BM, int BN, int WM, int WN, int NS, int EPI, int CDT, int RDT, int ADT = HERO_I8>
__global__ __launch_bounds__(WM * WN * 64, 2) void int8_gemm_persistent_kernel(GemmArgs g) {
    using ACC = typename AccOf<ADT>::type;
    constexpr bool UNIT = ADT == HERO_BF16 || ADT == HERO_F16;      // 16-bit operands: no scales, y = acc + bias
    constexpr bool WIDE = ADT == HERO_F8E4M3;
    constexpr int NT = WM * WN * 64, NWAVE = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    constexpr int A_UNITS = A_BYTES / 16 / NT, B_UNITS = B_BYTES / 16 / NT, NW = A_UNITS + B_UNITS;
    constexpr int NM = TM * TN, NFR = TM + TN;
    static_assert(NS == 4 && NW <= NM && NFR <= 2 * NM && NFR % 2 == 0, "ring / interleave plan");
    constexpr int RING = NS * STAGE;
    constexpr int SVF = 4 * BN;                                  // floats per vector set: column scale, bias, S_a, row scale
    static_assert(BM == BN, "the row-scale vector shares the column vectors' length");
    constexpr int PF_OFF = RING + 2 * SVF * 4;                   // 256 bytes per wave where the prefetch requests land (never read)
    static_assert(PF_OFF + NWAVE * 256 <= 160 * 1024, "LDS budget");
    __shared__ __attribute__((aligned(1024))) int8_t smem[PF_OFF + NWAVE * 256];
    float* const sv0 = reinterpret_cast<float*>(smem + RING);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int seq_end = min((xcd + 1) * g.per_xcd, g.ntm * g.ntn);
    int seq = xcd * g.per_xcd + slot;                            // this workgroup's tiles: seq, seq + nslot, ...
    if (seq >= seq_end) return;
    const int KT = g.K / BK;
    const bool has_rs = g.a_row_scale != nullptr, has_bias = g.bias != nullptr;
    if (!has_bias)                                               // the bias vectors are read by the epilogue either way
        for (int c = tid; c < 2 * BN; c += NT) sv0[(c / BN) * SVF + BN + c % BN] = 0.0f;

    // loader: unit u of wave w fills LDS granules [(u * NWAVE + w) * 64, +64) of the A (or B) part of
    // a stage; lane l owns row u * 128 + lrow, stored chunk l % 4 = global chunk (l % 4) ^ ((row >> 2) & 3).
    const int lrow = wave * 16 + (lane >> 2);
    const uint32_t lc = (uint32_t)(((lane & 3) ^ ((lrow >> 2) & 3)) * 16);
    const uint32_t wbase = __builtin_amdgcn_readfirstlane(lds_offset(smem) + wave * 1024);
    const uint32_t svbase = __builtin_amdgcn_readfirstlane(lds_offset(sv0));

    // ---- issue stream: the tile / slab the next direct loads belong to (runs NS-1 slabs ahead)
    int iseq = seq, ikt = 0, ipar = 0;
    const int8_t* ia; const int8_t* ib;                          // wave-uniform: tile base + slab offset
    uint32_t oa[A_UNITS], ob[B_UNITS];
    int m0i = 0, n0i = 0;                                        // origin of the issue stream's tile
    auto set_issue_tile = [&](int s) {
        tile_from_seq<BM, BN>(g, s, m0i, n0i);
        ia = g.A + (int64_t)m0i * g.lda;
        ib = g.Bt + (int64_t)n0i * g.ldb;
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u) oa[u] = (uint32_t)min(lrow + u * (NWAVE * 16), g.M - 1 - m0i) * (uint32_t)g.lda + lc;
#pragma unroll
        for (int u = 0; u < B_UNITS; ++u) ob[u] = (uint32_t)min(lrow + u * (NWAVE * 16), g.N - 1 - n0i) * (uint32_t)g.ldb + lc;
    };
    // The epilogue vectors of the issue stream's tile go out together with its FIRST pair, not when the stream
    // moves on to the tile: their buffer (parity of the tile) is still being read by the epilogue of the tile
    // two back until every wave has started the tile in between.
    auto issue_tile_vectors = [&](int par) {
        // wave w fetches 64 entries (chunk w % CH) of vectors w / CH and 2 + w / CH
        constexpr int CH = BN / 64;
        static_assert(NWAVE == 2 * CH, "two vectors per wave");
        const int wu = __builtin_amdgcn_readfirstlane(wave);
        const int ch = (wu % CH) * 64, which = wu / CH;
        const uint32_t dst = svbase + par * SVF * 4 + ch * 4;
        const uint32_t cn = (uint32_t)min(ch + lane, g.N - 1 - n0i) * 4u, cm = (uint32_t)min(ch + lane, g.M - 1 - m0i) * 4u;
        if (EPI == HERO_EPI_RAW_I32) return;
        if (which == 0) {
            if (!UNIT) dma4s(cn, g.b_col_scale + n0i, dst);
            if (EPI == HERO_EPI_GELU_REQUANT) dma4s(cn, g.out_col_scale + n0i, dst + 2 * BN * 4);
        } else {
            if (has_bias) dma4s(cn, g.bias + n0i, dst + BN * 4);
            if (has_rs) dma4s(cm, g.a_row_scale + m0i, dst + 3 * BN * 4);
        }
    };
    // The issue stream moves in PAIRS of slabs (128 bytes of every row = one cache line): the j-th direct load
    // of a pair is unit j / 2 of slab j % 2, so the two 64-byte halves of a line are requested back to back and
    // the second one is served by the line the first one brought in.  A CU pulls 48 B/clk from the L2 that way,
    // against 30 B/clk when the halves are requested one slab apart (measured; a 256 x 256 tile needs 32).
    auto issue_pair = [&](int j, int stage0) {                   // stage0: the (even) stage of the pair's first slab
        if (j == 0 && ikt == 0) issue_tile_vectors(ipar);
        const int u = j >> 1;
        const uint32_t lds = wbase + (stage0 + (j & 1)) * STAGE;
        // (the second slab through its own scalar base: an instruction offset would move the LDS side too)
        if (u < A_UNITS) dma16s(oa[u], ia + (j & 1) * BK, lds + u * NWAVE * 1024);
        else dma16s(ob[u - A_UNITS], ib + (j & 1) * BK, lds + A_BYTES + (u - A_UNITS) * NWAVE * 1024);
    };
    auto advance = [&]() {                                       // next pair; past the last tile the last pair repeats (never read)
        ikt += 2;
        if (ikt < KT) { ia += 2 * BK; ib += 2 * BK; return; }
        if (iseq + nslot < seq_end) {
            iseq += nslot; ikt = 0; ipar ^= 1;
            set_issue_tile(iseq);
        } else {
            ikt = KT - 2;
        }
    };

    // fragment offsets inside a stage (row rr, k-step ks, half hh): rr*64 + ((2ks+hh) ^ ((rr>>2)&3))*16
    const int hh = lane >> 5, ml = lane & 31;
    int fo[2][NFR];
#pragma unroll
    for (int t = 0; t < NFR; ++t) {
        const int rr = (t < TN ? wn * TN * 32 + t * 32 : wm * TM * 32 + (t - TN) * 32) + ml;
        const int base = (t < TN ? A_BYTES : 0) + rr * 64;
        fo[0][t] = base + (((0 + hh) ^ ((rr >> 2) & 3)) << 4);
        fo[1][t] = base + (((2 + hh) ^ ((rr >> 2) & 3)) << 4);
    }

    // prologue: vectors of the first tile, both pairs of the ring in flight, slab 0 landed
    set_issue_tile(seq);
#pragma unroll
    for (int p0 = 0; p0 < 2; ++p0) {
#pragma unroll
        for (int j = 0; j < 2 * NW; ++j) issue_pair(j, 2 * p0);
        advance();
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * NW + 1));
    __syncthreads();

    int stage = 0, par = 0;
    for (;;) {
        int m0, n0;
        tile_from_seq<BM, BN>(g, seq, m0, n0);
        ACC acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        v4i f0[NFR], f1[NFR];
#pragma unroll
        for (int t = 0; t < NFR; ++t) f0[t] = *reinterpret_cast<const v4i*>(smem + stage * STAGE + fo[0][t]);
        if (WIDE)
#pragma unroll
            for (int t = 0; t < NFR; ++t) f1[t] = *reinterpret_cast<const v4i*>(smem + stage * STAGE + fo[1][t]);

        // One slab per iteration with the barrier in the middle (see int8_gemm_dma_kernel).  KT is even and the
        // ring holds two pairs: after the barrier of an ODD iteration i every wave has read the last fragment
        // of the pair (i-1, i), whose two stages then take the pair (i+3, i+4) of the stream, which may
        // already belong to the next tile.  In program order the loads of a pair alternate between its slabs,
        // so "slab i+1 has landed" is vmcnt(1) in an odd iteration (only the last load of slab i+2 may be
        // out) and vmcnt(2 NW) in an even one (the younger pair may be out).
        auto iteration = [&](auto ODD) {
            constexpr bool odd = decltype(ODD)::value;
            const int8_t* st = smem + stage * STAGE;
            const int nstage = stage + 1 == NS ? 0 : stage + 1;
            const int pstage = stage == 0 ? NS - 1 : stage - 1;
            const int8_t* stn = smem + nstage * STAGE;
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (WIDE) {
                // FP8: one 32x32x64 matrix instruction per accumulator and slab (both k halves of a fragment
                // side by side: any K grouping shared by the two operands is the same contraction).  A
                // fragment is reloaded from the next slab right after its last use; the barrier that
                // publishes that slab sits after the first TM instructions.
#pragma unroll
                for (int n = 0; n < NM; ++n) {
                    const int jj = n / TM, ii = n % TM;
                    acc[ii][jj] = mfma_wide_f8(f0[jj], f1[jj], f0[TN + ii], f1[TN + ii], acc[ii][jj]);
                    if (n == TM - 1) {
                        __builtin_amdgcn_s_waitcnt(vmcnt_imm(odd ? 1 : 2 * NW));
                        __syncthreads();
                    }
                    if (n >= TM - 1) {
#pragma unroll
                        for (int t = 0; t < NFR; ++t) {
                            const int last = t < TN ? t * TM + TM - 1 : (TN - 1) * TM + (t - TN);
                            if ((last < TM - 1 ? TM - 1 : last) == n) {
                                f0[t] = *reinterpret_cast<const v4i*>(stn + fo[0][t]);
                                f1[t] = *reinterpret_cast<const v4i*>(stn + fo[1][t]);
                            }
                        }
                        if (odd) {                                     // PPS units of the new pair per instruction slot
                            constexpr int SLOTS = NM - TM + 1, PPS = (NW + SLOTS - 1) / SLOTS;
#pragma unroll
                            for (int u = (n - (TM - 1)) * PPS; u < (n - (TM - 1) + 1) * PPS; ++u)
                                if (u < NW) { issue_pair(2 * u, pstage); issue_pair(2 * u + 1, pstage); }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int n = 0; n < NM; ++n) {                         // k-step 0
                    const int jj = n / TM, ii = n % TM;
                    acc[ii][jj] = mfma_step<ADT>(f0[jj], f0[TN + ii], acc[ii][jj]);
                    if (n < NFR / 2) {                                 // early: the reads must be back before the barrier
                        f1[2 * n] = *reinterpret_cast<const v4i*>(st + fo[1][2 * n]);
                        f1[2 * n + 1] = *reinterpret_cast<const v4i*>(st + fo[1][2 * n + 1]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(odd ? 1 : 2 * NW));   // the next slab has landed (mine)
                __syncthreads();                                       // ... and everybody's
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = 0; n < NM; ++n) {                         // k-step 1
                    const int jj = n / TM, ii = n % TM;
                    acc[ii][jj] = mfma_step<ADT>(f1[jj], f1[TN + ii], acc[ii][jj]);
                    if (n < NFR / 2) {
                        f0[2 * n] = *reinterpret_cast<const v4i*>(stn + fo[0][2 * n]);
                        f0[2 * n + 1] = *reinterpret_cast<const v4i*>(stn + fo[0][2 * n + 1]);
                    }
                    if (odd && n < NW) { issue_pair(2 * n, pstage); issue_pair(2 * n + 1, pstage); }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (odd) advance();
            stage = nstage;
        };
        for (int kt = 0; kt < KT; kt += 2) {
            iteration(std::false_type{});
            iteration(std::true_type{});
        }
        // Prefetch for the caller's next kernel: this tile's share of the lines, one dword of each, through the same
        // direct loads into a scratch corner of the LDS (no register is written, so nothing has to wait for them; the
        // waits of the next main loop only count loads issued after these, and the epilogue in between is far
        // longer than a miss).  What the request brings is the line: into this XCD's L2 and, on its way, into the
        // memory-side cache, where the next kernel's first tiles would otherwise all miss at once.
        if (g.pf_lines > 0) {
            const int w0 = __builtin_amdgcn_readfirstlane(wave) * 64;
            if (w0 < g.pf_lpt) {
                const uint32_t line = (uint32_t)min(seq * g.pf_lpt + w0 + lane, g.pf_lines - 1);
                dma4s(line * 128u, reinterpret_cast<const float*>(g.pf),
                      __builtin_amdgcn_readfirstlane(lds_offset(smem + PF_OFF)) + (uint32_t)w0 * 4u);
            }
        }
        // epilogue of this tile; the ring keeps filling with the next tile's slabs meanwhile
        const float* sv = sv0 + par * SVF;
        float rsr[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) rsr[i] = (EPI != HERO_EPI_RAW_I32 && has_rs) ? sv[3 * BN + wm * TM * 32 + i * 32 + ml] : 1.0f;
        epilogue_direct<BM, BN, WM, WN, EPI, CDT, RDT, true, UNIT>(g, acc, sv, rsr, m0, n0, tid);
        seq += nslot;
        par ^= 1;
        if (seq >= seq_end) break;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                      // the redundant tail loads
}

// =====================================================================================
// Persistent kernel with the epilogue INSIDE the next tile's main loop (large problems, K >= 1024).
// The vector ALU issues while the matrix pipe of the same SIMD is busy (measured: a wave that puts 4 fp32
// instructions behind each of its v_mfma_i32_32x32x32_i8 runs 15 % longer than the matrix instructions alone,
// not the 34 % the two take one after the other), but only if both kinds of work are there at the same
// time.  Here a wave keeps TWO sets of accumulators: while the matrix instructions of tile t+1 fill one, the
// dequantization / GELU / requantization / stores of tile t drain the other, a fixed handful of vector
// instructions behind every matrix instruction (the epilogue of a tile is cut into 128 such steps, the first
// 16 slabs of the next tile).  A 256 x 256 tile would need 2 x 128 accumulator registers per lane, which the
// register file does not have beside everything else, so the tile is 256 x 128: 8 waves of 64 x 64 (4
// accumulators, 2 x 64 registers).  The smaller tile needs 1.5 x the L2 -> LDS bytes per multiply-add; in exchange
// a stage is 24 KB and the ring holds SIX slabs (three pairs), i.e. five slabs of lookahead instead of three.
// The last tile of a workgroup has no successor: its epilogue runs after the loop, unhidden.
// Measured (16384 x 4096 x 1024): the epilogue does disappear -- GELU^quant costs 7 us over the plain requantization
// where it costs 25 us behind the 256 x 256 tile -- but the main loop of the smaller tile is slower by about as much
// (92 us against 76 us: 1.33 x the LDS fragment reads per matrix instruction and 1.5 x the direct-load bytes on a
// load stream that is latency-bound), so the two kernels end within 2 % of each other (99 / 101 us with
// GELU^quant) when both are timed alone with operands that stay in the memory-side cache.  Inside a layer the
// weights come from HBM, and there the deeper ring decides: this kernel is the tile choice's pick for a GELU epilogue
// with K < 2048 (the numbers are beside the rule in launch_epi); the test entry point reaches it as tile code 9.
// =====================================================================================
// wait for vmcnt <= N and for every LDS access of this wave, then the workgroup barrier.  Inline assembly: the
// kernel below has global stores inside its main loop, and a __syncthreads() there would make the compiler
// wait for ALL outstanding vector-memory operations, the direct loads of the next slabs included.  The memory
// clobber keeps the compiler from moving LDS accesses across the barrier.
template <int N>
__device__ __forceinline__ void wait_vm_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(N) : "memory");
}

template <int EPI, int CDT>
__global__ __launch_bounds__(512, 2) void int8_gemm_ovl_kernel(GemmArgs g) {
    constexpr int BM = 256, BN = 128, WN = 2, NS = 6, NWAVE = 8, NT = 512;
    constexpr int TM = 2, TN = 2, NM = TM * TN, NFR = TM + TN;
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    constexpr int A_UNITS = A_BYTES / 16 / NT, B_UNITS = B_BYTES / 16 / NT, NW = A_UNITS + B_UNITS;
    static_assert(A_UNITS == 2 && B_UNITS == 1 && NW <= NM && NFR == NM, "interleave plan");
    constexpr int RING = NS * STAGE;
    // per-tile epilogue vectors in LDS: column scale, bias, S_a (BN each), row scale (BM); three sets, because
    // the set of tile t is read during tile t+1 while the issue stream already fetches the one of tile t+2
    constexpr int SV_CS = 0, SV_BIAS = BN, SV_OS = 2 * BN, SV_RS = 3 * BN, SVF = 3 * BN + BM, NSV = 3;
    constexpr int ES = ElemSize<CDT>::v;
    constexpr bool GELU = EPI == HERO_EPI_DEQUANT_GELU || EPI == HERO_EPI_GELU_REQUANT;
    constexpr int SPREAD = 16;                                   // slabs of the next tile the epilogue is spread over
    constexpr int NSTEP = 16, NPIECE = 8;                        // 8 pieces of 8 outputs per lane, 16 steps each
    static_assert(NPIECE * NSTEP == SPREAD * 2 * NM, "one epilogue step behind every matrix instruction");
    constexpr int PF_OFF = RING + NSV * SVF * 4;                 // 256 bytes per wave where the prefetch requests land (never read)
    static_assert(PF_OFF + NWAVE * 256 <= 160 * 1024, "LDS budget");
    __shared__ __attribute__((aligned(1024))) int8_t smem[PF_OFF + NWAVE * 256];
    float* const sv0 = reinterpret_cast<float*>(smem + RING);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int hh = lane >> 5, ml = lane & 31;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int seq_end = min((xcd + 1) * g.per_xcd, g.ntm * g.ntn);
    int seq = xcd * g.per_xcd + slot;                            // this workgroup's tiles: seq, seq + nslot, ...
    if (seq >= seq_end) return;
    const int KT = g.K / BK;                                     // even, >= SPREAD (the launch checks)
    const bool has_rs = g.a_row_scale != nullptr, has_bias = g.bias != nullptr;
    // absent vectors: the epilogue multiplies by 1 and adds 0 (both exact)
    if (!has_bias) for (int c = tid; c < NSV * BN; c += NT) sv0[(c / BN) * SVF + SV_BIAS + c % BN] = 0.0f;
    if (!has_rs) for (int c = tid; c < NSV * BM; c += NT) sv0[(c / BM) * SVF + SV_RS + c % BM] = 1.0f;

    // loader: unit u of wave w fills LDS granules [(u * NWAVE + w) * 64, +64) of the A (or B) part of a stage;
    // lane l owns row u * 128 + lrow, stored chunk l % 4 = global chunk (l % 4) ^ ((row >> 2) & 3)
    const int lrow = wave * 16 + (lane >> 2);
    const uint32_t lc = (uint32_t)(((lane & 3) ^ ((lrow >> 2) & 3)) * 16);
    const uint32_t wbase = __builtin_amdgcn_readfirstlane(lds_offset(smem) + wave * 1024);
    const uint32_t svbase = __builtin_amdgcn_readfirstlane(lds_offset(sv0));

    // ---- issue stream: the tile / slab the next direct loads belong to (runs NS - 1 slabs ahead)
    int iseq = seq, ikt = 0, ibuf = 0;
    const int8_t* ia; const int8_t* ib;                          // wave-uniform: tile base + slab offset
    uint32_t oa[A_UNITS], ob;
    int m0i = 0, n0i = 0;
    auto set_issue_tile = [&](int s) {
        tile_from_seq<BM, BN>(g, s, m0i, n0i);
        ia = g.A + (int64_t)m0i * g.lda;
        ib = g.Bt + (int64_t)n0i * g.ldb;
#pragma unroll
        for (int u = 0; u < A_UNITS; ++u) oa[u] = (uint32_t)min(lrow + u * (NWAVE * 16), g.M - 1 - m0i) * (uint32_t)g.lda + lc;
        ob = (uint32_t)min(lrow, g.N - 1 - n0i) * (uint32_t)g.ldb + lc;
    };
    // The vectors of a tile are 10 chunks of 64 floats: 0-1 column scale, 2-3 bias, 4-5 S_a, 6-9 row scale.  Wave w
    // fetches chunk w, waves 0 and 1 also chunks 8 and 9; what a wave fetches is fixed for the whole kernel, so
    // it is worked out here once (source, clamp, destination) and the issue is one predicated load per chunk.
    const int wu = __builtin_amdgcn_readfirstlane(wave);
    const int vwhich = wu < 6 ? wu >> 1 : 3;                     // 0 column scale, 1 bias, 2 S_a, 3 row scale
    const int vch = wu < 6 ? (wu & 1) * 64 : (wu - 6) * 64;
    const float* const vsrc = vwhich == 0 ? g.b_col_scale : vwhich == 1 ? g.bias : vwhich == 2 ? g.out_col_scale : g.a_row_scale;
    const bool von = EPI != HERO_EPI_RAW_I32 && (vwhich == 0 || (vwhich == 1 && has_bias) ||
                                                 (vwhich == 2 && EPI == HERO_EPI_GELU_REQUANT) || (vwhich == 3 && has_rs));
    const uint32_t vdst = svbase + (uint32_t)(vwhich * BN + vch) * 4;
    const bool von2 = EPI != HERO_EPI_RAW_I32 && wu < 2 && has_rs;   // chunks 8, 9: rows 128 .. 255 of the row scale
    const uint32_t vdst2 = svbase + (uint32_t)(SV_RS + 128 + wu * 64) * 4;
    auto issue_tile_vectors = [&](int buf) {                     // when the stream enters a tile: older than all its slabs
        const uint32_t bo = (uint32_t)buf * (SVF * 4);
        if (von) {
            const int lim = vwhich == 3 ? g.M - 1 - m0i : g.N - 1 - n0i, org = vwhich == 3 ? m0i : n0i;
            dma4s((uint32_t)min(vch + lane, lim) * 4u, vsrc + org, vdst + bo);
        }
        if (von2) dma4s((uint32_t)min(128 + wu * 64 + lane, g.M - 1 - m0i) * 4u, g.a_row_scale + m0i, vdst2 + bo);
        // the prefetch hint (see the persistent kernel): this tile's share of the lines the caller's next kernel reads.
        // Like the vectors the requests are older than every slab of the tile, and five slabs pass before a wait
        // asks for them.
        if (g.pf_lines > 0 && wu * 64 < g.pf_lpt)
            dma4s((uint32_t)min(iseq * g.pf_lpt + wu * 64 + lane, g.pf_lines - 1) * 128u, reinterpret_cast<const float*>(g.pf),
                  __builtin_amdgcn_readfirstlane(lds_offset(smem + PF_OFF)) + (uint32_t)wu * 256u);
    };
    // The stream moves in PAIRS of slabs (128 bytes of every row = one cache line): load j of a pair is unit
    // j / 2 of slab j % 2, so the two 64-byte halves of a line are requested back to back.
    auto issue_pair = [&](int j, int stage0) {                   // stage0: the (even) stage of the pair's first slab
        const int u = j >> 1;
        const uint32_t lds = wbase + (stage0 + (j & 1)) * STAGE;
        if (u < A_UNITS) dma16s(oa[u], ia + (j & 1) * BK, lds + u * NWAVE * 1024);
        else dma16s(ob, ib + (j & 1) * BK, lds + A_BYTES);
    };
    // next pair; past the last tile the last pair repeats (never read).  The vectors of a tile go out the moment
    // the stream enters it: their set (tile count mod 3) was last read by the epilogue of the tile three back,
    // which ended before the current tile began.
    auto advance = [&]() {
        ikt += 2;
        if (ikt < KT) { ia += 2 * BK; ib += 2 * BK; return; }
        if (iseq + nslot < seq_end) {
            iseq += nslot; ikt = 0; ibuf = ibuf == NSV - 1 ? 0 : ibuf + 1;
            set_issue_tile(iseq);
            issue_tile_vectors(ibuf);
        } else {
            ikt = KT - 2;
        }
    };

    // fragment offsets inside a stage (row rr, k-step ks, half hh): rr*64 + ((2ks+hh) ^ ((rr>>2)&3))*16
    int fo[2][NFR];
#pragma unroll
    for (int t = 0; t < NFR; ++t) {
        const int rr = (t < TN ? wn * TN * 32 + t * 32 : wm * TM * 32 + (t - TN) * 32) + ml;
        const int base = (t < TN ? A_BYTES : 0) + rr * 64;
        fo[0][t] = base + (((0 + hh) ^ ((rr >> 2) & 3)) << 4);
        fo[1][t] = base + (((2 + hh) ^ ((rr >> 2) & 3)) << 4);
    }

    // prologue: the first tile's vectors and the three pairs of the ring in flight, slab 0 landed
    set_issue_tile(seq);
    issue_tile_vectors(0);
#pragma unroll
    for (int p0 = 0; p0 < NS / 2; ++p0) {
#pragma unroll
        for (int j = 0; j < 2 * NW; ++j) issue_pair(j, 2 * p0);
        advance();
    }
    wait_vm_barrier<(NS / 2 - 1) * 2 * NW + 1>();                 // only the last load of slab 1 and the two younger pairs may be out

    v16i acc[TM][TN], prev[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0; prev[i][j][r] = 0; }
    v4i f0[NFR], f1[NFR];
#pragma unroll
    for (int t = 0; t < NFR; ++t) f0[t] = *reinterpret_cast<const v4i*>(smem + fo[0][t]);

    // ---- the tile whose epilogue is being drained: none yet (row origin M switches every store off)
    int m0p = g.M, n0p = 0;
    float* svp = sv0 + (NSV - 1) * SVF;
    const bool al8 = g.ldc % 8 == 0;                             // rows of C start on 8-element boundaries
    bool interior = false;                                       // the draining tile lies inside C and its rows are aligned: plain wide stores
    // state of the piece in flight (8 outputs of one row per lane)
    float ey[8], ez[8], ep[8];
    v4f ecs[2], ebs[2], eos[2];
    float ers = 1.0f;
    // Step s of the epilogue of the previous tile.  Piece pc = s / 16 covers, for output row
    // wm*64 + i*32 + ml (i = pc / 4), the 4-column groups q = pc % 4 of both accumulators of that row:
    // columns wn*64 + 8q + 4hh + t and + 32.  After the lane-half exchange a lane owns 8 contiguous columns.
    auto epi_step = [&](auto S) {
        constexpr int s = decltype(S)::value, pc = s / NSTEP, st = s % NSTEP, i = pc / 4, qq = pc % 4;
        const int rowl = wm * 64 + i * 32 + ml, c0 = wn * 64 + 8 * qq + 4 * hh;
        if constexpr (s == 0 && EPI == HERO_EPI_GELU_REQUANT) {
            // S_a -> 1 / S_a once per tile (IEEE division), published by the barrier in the middle of this slab;
            // the first read is in step 10 of piece 0, well behind it
            if (tid < BN) svp[SV_OS + tid] = __fdiv_rn(1.0f, svp[SV_OS + tid]);
        }
        if constexpr (EPI == HERO_EPI_RAW_I32) {
            if constexpr (st == 1) {
                const int row = m0p + rowl;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int col = n0p + c0 + 32 * j;
                    const uint32_t d[4] = {(uint32_t)prev[i][j][4 * qq], (uint32_t)prev[i][j][4 * qq + 1],
                                           (uint32_t)prev[i][j][4 * qq + 2], (uint32_t)prev[i][j][4 * qq + 3]};
                    int8_t* cp = (int8_t*)g.C + ((int64_t)row * g.ldc + col) * 4;
                    if (interior) *reinterpret_cast<v4i*>(cp) = v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
                    else if (row < g.M && col < g.N) store_piece<4, 4>(cp, d, col, g.N, col + 4 <= g.N, true);
                }
            }
        } else {
            if constexpr (st == 0) {
                ecs[0] = *reinterpret_cast<const v4f*>(svp + SV_CS + c0);
                ecs[1] = *reinterpret_cast<const v4f*>(svp + SV_CS + c0 + 32);
                ebs[0] = *reinterpret_cast<const v4f*>(svp + SV_BIAS + c0);
                ebs[1] = *reinterpret_cast<const v4f*>(svp + SV_BIAS + c0 + 32);
                ers = svp[SV_RS + rowl];
            } else if constexpr (st == 1) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = (float)prev[i][e >> 2][4 * qq + (e & 3)];
            } else if constexpr (st == 2) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = ey[e] * ers;
            } else if constexpr (st == 3) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = fmaf(ey[e], ecs[e >> 2][e & 3], ebs[e >> 2][e & 3]);
            } else if constexpr (GELU && st == 4) {               // erf-form GELU as in gelu_erf(), cut into steps
#pragma unroll
                for (int e = 0; e < 8; ++e) { ez[e] = fminf(fabsf(ey[e]), 6.0f); ep[e] = fmaf(3.309558087e-05f, ez[e], -7.692443905e-04f); }
            } else if constexpr (GELU && st == 5) {
#pragma unroll
                for (int e = 0; e < 8; ++e) { ep[e] = fmaf(ep[e], ez[e], 8.080800064e-03f); ep[e] = fmaf(ep[e], ez[e], -5.341223627e-02f); }
            } else if constexpr (GELU && st == 6) {
#pragma unroll
                for (int e = 0; e < 8; ++e) { ep[e] = fmaf(ep[e], ez[e], -4.587708712e-01f); ep[e] = fmaf(ep[e], ez[e], -1.151201725e+00f); }
            } else if constexpr (GELU && st == 7) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ep[e] = fmaf(ep[e], ez[e], -9.999930859e-01f);
            } else if constexpr (GELU && st == 8) {
#pragma unroll
                for (int e = 0; e < 4; ++e) ep[e] = __builtin_amdgcn_exp2f(ep[e]);
            } else if constexpr (GELU && st == 9) {
#pragma unroll
                for (int e = 4; e < 8; ++e) ep[e] = __builtin_amdgcn_exp2f(ep[e]);
            } else if constexpr (GELU && st == 10) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ez[e] = fmaxf(ey[e], 0.0f);
                if constexpr (EPI == HERO_EPI_GELU_REQUANT) {
                    eos[0] = *reinterpret_cast<const v4f*>(svp + SV_OS + c0);
                    eos[1] = *reinterpret_cast<const v4f*>(svp + SV_OS + c0 + 32);
                }
            } else if constexpr (GELU && st == 11) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = fmaf(-fabsf(ey[e]), ep[e], ez[e]);
            } else if constexpr (EPI == HERO_EPI_GELU_REQUANT && st == 12) {
                // GELU^quant is in the +-1 LSB class (fp32 GELU against the definition's fp64): the division by
                // S_a[j] is a multiplication by the correctly rounded reciprocal
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = ey[e] * eos[e >> 2][e & 3];
            } else if constexpr (ES == 1 && st == 13) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = __builtin_amdgcn_fmed3f(ey[e], -127.0f, 127.0f);
            } else if constexpr (ES == 1 && st == 14) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ey[e] = ey[e] + 12582912.0f;   // rne_low_byte(): the low byte of the sum is the code
            } else if constexpr (st == 15) {
                const int row = m0p + rowl, col = n0p + wn * 64 + hh * 32 + 8 * qq;   // first of this lane's 8 columns
                const bool ok = row < g.M && col < g.N, full = col + 8 <= g.N;   // (only looked at on the edge tiles)
                if constexpr (ES == 1) {
                    const uint32_t w0 = pack_low_bytes(__float_as_uint(ey[0]), __float_as_uint(ey[1]), __float_as_uint(ey[2]), __float_as_uint(ey[3]));
                    const uint32_t w1 = pack_low_bytes(__float_as_uint(ey[4]), __float_as_uint(ey[5]), __float_as_uint(ey[6]), __float_as_uint(ey[7]));
                    uint32_t d[2];
                    swap32(w0, w1, d[0], d[1]);
                    int8_t* cp = (int8_t*)g.C + (int64_t)row * g.ldc + col;
                    if (interior) *reinterpret_cast<v2i*>(cp) = v2i{(int)d[0], (int)d[1]};
                    else if (ok) store_piece<1, 2>(cp, d, col, g.N, full, false);
                } else {
                    uint32_t d[4];
                    swap32(pack2_hp<CDT>(ey[0], ey[1]), pack2_hp<CDT>(ey[4], ey[5]), d[0], d[2]);
                    swap32(pack2_hp<CDT>(ey[2], ey[3]), pack2_hp<CDT>(ey[6], ey[7]), d[1], d[3]);
                    int8_t* cp = (int8_t*)g.C + ((int64_t)row * g.ldc + col) * 2;
                    if (interior) *reinterpret_cast<v4i*>(cp) = v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
                    else if (ok) store_piece<2, 4>(cp, d, col, g.N, full, false);
                }
            }
        }
    };

    int stage = 0, buf = 0;
    // One slab: the barrier sits in the middle (k-step 0 runs on fragments read during the previous slab, the
    // barrier makes slab kt+1 visible, k-step 1 runs while its first fragments and, in odd slabs, the direct loads
    // of the pair five slabs ahead are issued).  In program order the loads of a pair alternate between its two
    // slabs, so "slab kt+1 has landed" is: at most the pair's last load and the two younger pairs outstanding in an
    // odd slab, the two younger pairs in an even one.  The stores of the epilogue steps count in vmcnt as well; they
    // can only make the wait longer, never shorter than needed (loads return in order among themselves).
    auto iteration = [&](auto ODD, auto SLOT0, auto FIRST) {
        constexpr bool odd = decltype(ODD)::value, first = decltype(FIRST)::value;
        constexpr int s0 = decltype(SLOT0)::value;                   // first epilogue step of this slab; < 0: none
        const int8_t* st = smem + stage * STAGE;
        const int nstage = stage + 1 == NS ? 0 : stage + 1;
        const int pstage = stage == 0 ? NS - 1 : stage - 1;
        const int8_t* stn = smem + nstage * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        static_for<NM>([&](auto N_) {                                // k-step 0
            constexpr int n = decltype(N_)::value, jj = n / TM, ii = n % TM;
            if constexpr (first) {
                const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                acc[ii][jj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f0[jj], f0[TN + ii], zero, 0, 0, 0);
            } else {
                acc[ii][jj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f0[jj], f0[TN + ii], acc[ii][jj], 0, 0, 0);
            }
            if constexpr (n < NFR / 2) {                             // early: the reads must be back before the barrier
                f1[2 * n] = *reinterpret_cast<const v4i*>(st + fo[1][2 * n]);
                f1[2 * n + 1] = *reinterpret_cast<const v4i*>(st + fo[1][2 * n + 1]);
            }
            if constexpr (s0 >= 0) epi_step(std::integral_constant<int, (s0 >= 0 ? s0 + n : 0)>{});
            __builtin_amdgcn_sched_barrier(0);
        });
        wait_vm_barrier<odd ? 2 * NW + 1 : 4 * NW>();
        __builtin_amdgcn_sched_barrier(0);
        static_for<NM>([&](auto N_) {                                // k-step 1
            constexpr int n = decltype(N_)::value, jj = n / TM, ii = n % TM;
            acc[ii][jj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f1[jj], f1[TN + ii], acc[ii][jj], 0, 0, 0);
            if constexpr (n < NFR / 2) {
                f0[2 * n] = *reinterpret_cast<const v4i*>(stn + fo[0][2 * n]);
                f0[2 * n + 1] = *reinterpret_cast<const v4i*>(stn + fo[0][2 * n + 1]);
            }
            if constexpr (odd && n < NW) { issue_pair(2 * n, pstage); issue_pair(2 * n + 1, pstage); }
            if constexpr (s0 >= 0) epi_step(std::integral_constant<int, (s0 >= 0 ? s0 + NM + n : 0)>{});
            __builtin_amdgcn_sched_barrier(0);
        });
        if (odd) advance();
        stage = nstage;
    };

    for (;;) {
        // the first SPREAD slabs carry the epilogue of the previous tile, one step behind every matrix instruction
        static_for<SPREAD>([&](auto I_) {
            constexpr int it = decltype(I_)::value;
            iteration(std::integral_constant<bool, (it & 1) != 0>{}, std::integral_constant<int, it * 2 * NM>{},
                      std::integral_constant<bool, it == 0>{});
        });
        for (int kt = SPREAD; kt < KT; kt += 2) {
            iteration(std::false_type{}, std::integral_constant<int, -1>{}, std::false_type{});
            iteration(std::true_type{}, std::integral_constant<int, -1>{}, std::false_type{});
        }
        // hand the finished accumulators to the epilogue that runs inside the next tile
        tile_from_seq<BM, BN>(g, seq, m0p, n0p);
        interior = __builtin_amdgcn_readfirstlane((int)(al8 && m0p + BM <= g.M && n0p + BN <= g.N)) != 0;
        svp = sv0 + buf * SVF;
        buf = buf == NSV - 1 ? 0 : buf + 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) prev[i][j] = acc[i][j];
        seq += nslot;
        if (seq >= seq_end) break;
    }
    // the last tile's epilogue, unhidden
    static_for<NPIECE * NSTEP>([&](auto S) {
        epi_step(S);
        if constexpr (decltype(S)::value == 3 && EPI == HERO_EPI_GELU_REQUANT) wait_vm_barrier<63>();   // publishes 1 / S_a
    });
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                      // the redundant tail loads
}

// Split-K for skinny M with a long K (M <= 128, K >= 8192, at most 128 tiles: the weights are streamed once and
// too few tiles exist to do that from every CU).  Pass 1: the register-staged kernel with a second grid dimension over K ranges writes raw int32
// partial sums, one [M][ldp] plane per range, into the caller's scratch.  Pass 2 (splitk_reduce_kernel) adds
// the planes and runs the epilogue.  Integer sums commute and the epilogue arithmetic is the same, in the
// same order, as in the one-pass kernels, so the results are identical; the kernel boundary is the only
// synchronisation (device-wide fences inside one kernel measured 4x slower than no split at all).
struct SplitK { int BM, BN, ksplit, kslabs; int64_t ldp; size_t bytes; };
inline SplitK splitk_plan(int64_t M, int64_t N, int64_t K) {
    SplitK p = {0, 0, 1, 0, 0, 0};
    if (M <= 0 || N <= 0 || M > 128 || K % BK != 0) return p;
    p.BM = p.BN = M <= 64 ? 64 : 128;
    const int64_t tiles = ((M + p.BM - 1) / p.BM) * ((N + p.BN - 1) / p.BN), kt = K / BK;
    // Measured: two launches pay only for a long K over few tiles (64 x 4096 x 16384: 20 us against 31 in one pass);
    // with K = 4096 the one-pass kernels (four K groups per workgroup up to 128 tiles, plain 64 x 64 tiles beyond)
    // are 20-35 % faster than the split (64 x 12288 x 4096: 15.4 against 20.1 us), and small weights are
    // launch-bound anyway.
    if (tiles > 128 || kt < 128 || N * K < (4 << 20)) return p;
    int64_t want = (512 + tiles - 1) / tiles;                         // about two workgroups per CU
    if (want > 16) want = 16;
    int64_t kslabs = (kt + want - 1) / want;
    if (kslabs < 4) kslabs = 4;
    p.kslabs = (int)kslabs;
    p.ksplit = (int)((kt + kslabs - 1) / kslabs);                     // every range non-empty
    if (p.ksplit <= 1) { p.ksplit = 1; return p; }
    p.ldp = (N + 3) & ~(int64_t)3;
    p.bytes = (size_t)p.ksplit * M * p.ldp * 4;
    return p;
}

// Pass 2 of split-K: one thread per 4 consecutive columns of a row.
template <int EPI, int CDT, int RDT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g, const int32_t* part, int64_t ldp) {
    constexpr int ES = ElemSize<CDT>::v;
    const int nq = (g.N + 3) / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)g.M * nq) return;
    const int m = (int)(idx / nq), n = (int)(idx % nq) * 4;
    v4i a = {0, 0, 0, 0};
    for (int ks = 0; ks < g.ksplit; ++ks)
        a += *reinterpret_cast<const v4i*>(part + ((int64_t)ks * g.M + m) * ldp + n);
    const int nv = min(4, g.N - n);                                    // valid columns
    uint32_t e[4];                                                     // outputs as element bit patterns
    if constexpr (EPI == HERO_EPI_RAW_I32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) e[t] = (uint32_t)a[t];
    } else {
        const float rs = g.a_row_scale ? g.a_row_scale[m] : 1.0f;
        float y[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int nn = min(n + t, g.N - 1);
            float v = (float)a[t];
            if (g.a_row_scale) v = v * rs;
            v = fmaf(v, g.b_col_scale[nn], g.bias ? g.bias[nn] : 0.0f);
            if (EPI == HERO_EPI_DEQUANT_GELU || EPI == HERO_EPI_GELU_REQUANT) v = gelu_erf(v);
            if (EPI == HERO_EPI_GELU_REQUANT) v = v * __fdiv_rn(1.0f, g.out_col_scale[nn]);
            if (RDT >= 0 && t < nv) v += hp_to_f32<RDT>(((const uint16_t*)g.residual)[(int64_t)m * g.ldr + n + t]);
            y[t] = v;
        }
        if constexpr (ES == 1) {
            const uint32_t w = quant4_sat(y[0], y[1], y[2], y[3]);
#pragma unroll
            for (int t = 0; t < 4; ++t) e[t] = (w >> (8 * t)) & 0xffu;
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) e[t] = f32_to_hp<CDT>(y[t]);
        }
    }
    int8_t* cp = (int8_t*)g.C + ((int64_t)m * g.ldc + n) * ES;
    if (nv == 4) {
        if constexpr (ES == 1) *reinterpret_cast<uint32_t*>(cp) = e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24);
        else if constexpr (ES == 2) *reinterpret_cast<v2i*>(cp) = v2i{(int)(e[0] | (e[1] << 16)), (int)(e[2] | (e[3] << 16))};
        else *reinterpret_cast<v4i*>(cp) = v4i{(int)e[0], (int)e[1], (int)e[2], (int)e[3]};
    } else {
        for (int t = 0; t < nv; ++t) {
            if (ES == 1) cp[t] = (int8_t)e[t];
            else if (ES == 2) reinterpret_cast<uint16_t*>(cp)[t] = (uint16_t)e[t];
            else reinterpret_cast<uint32_t*>(cp)[t] = e[t];
        }
    }
}

template <int EPI, int CDT, int RDT>
hero_status launch_splitk(const GemmArgs& g, const SplitK& p, void* ws, hipStream_t st) {
    GemmArgs g1 = g;                                                   // pass 1: raw partial planes in the scratch
    g1.a_row_scale = nullptr; g1.b_col_scale = nullptr; g1.bias = nullptr; g1.residual = nullptr; g1.out_col_scale = nullptr;
    g1.C = ws; g1.ldc = p.ldp;
    g1.ntm = (g.M + p.BM - 1) / p.BM;
    g1.ntn = (g.N + p.BN - 1) / p.BN;
    const int64_t tiles = (int64_t)g1.ntm * g1.ntn;
    g1.per_xcd = (int)((tiles + NUM_XCD - 1) / NUM_XCD);
    g1.ksplit = p.ksplit; g1.kslabs = p.kslabs;
    const dim3 grid((unsigned)(g1.per_xcd * NUM_XCD), (unsigned)p.ksplit);
    // (measured on 64 x 4096 x 16384 with cold weights: 8 slabs in flight are 3 % slower than 4; 26 us with the
    // reduction pass, 2.6 TB/s)
    if (p.BM == 64) hipLaunchKernelGGL((int8_gemm_kernel<64, 64, 2, 2, 4, 2, HERO_EPI_RAW_I32, HERO_I32, -1, true>), grid, dim3(256), 0, st, g1);
    else hipLaunchKernelGGL((int8_gemm_kernel<128, 128, 2, 2, 2, 2, HERO_EPI_RAW_I32, HERO_I32, -1, true>), grid, dim3(256), 0, st, g1);
    hero_status s1 = hero_launch_status();
    if (s1 != HERO_OK) return s1;
    GemmArgs g2 = g;                                                   // pass 2: sum of the planes + epilogue
    g2.ksplit = p.ksplit; g2.kslabs = p.kslabs;
    const int64_t threads = (int64_t)g.M * ((g.N + 3) / 4);
    hipLaunchKernelGGL((splitk_reduce_kernel<EPI, CDT, RDT>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                       g2, (const int32_t*)ws, p.ldp);
    return hero_launch_status();
}

template <typename K>
hero_status launch_grid(GemmArgs g, int BM, int BN, int threads, K kernel, hipStream_t st) {
    g.ntm = (g.M + BM - 1) / BM;
    g.ntn = (g.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)g.ntm * g.ntn;
    g.per_xcd = (int)((tiles + NUM_XCD - 1) / NUM_XCD);
    if ((int64_t)g.per_xcd * NUM_XCD > 0x7fffffffLL) return HERO_ERR_SHAPE;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(g.per_xcd * NUM_XCD)), dim3(threads), 0, st, g);
    return hero_launch_status();
}

// Tile choice (all measured on MI355X): the persistent 256x256 direct-to-LDS kernel, one workgroup per CU, once
// the grid has enough tiles (160) to keep most of the 256 CUs busy; the persistent 128x128 form of the same kernel,
// two workgroups per CU, below that (with 96-128 tiles of 256x256 half of the CUs would idle: 10-30 % faster there)
// and where the last round of 256x256 tiles would be so empty that the small tile fills the chip better
// (small_tile_fills_better below; per full round the small tile is 10-15 % slower, it needs twice the L2 -> LDS
// traffic); 64x64 register-staged tiles, or smaller ones, while
// fewer than 192 tiles of 128x128 exist (small problems are latency-bound: more, shorter workgroups).  The
// persistent kernels need K >= 256, K % 128 == 0 and 32-bit per-lane offsets; otherwise the one-tile-per-workgroup
// 256x256 kernel or the register-staged 128x128 one take their place.
// The test hook hero_int8_gemm_tile forces a form: 0 = 128x128 register-staged, 1 = 256x256 one tile per workgroup,
// 2 = 64x64 (and its skinny relatives), 7 = 256x256 persistent, 8 = 128x128 persistent.
// the prefetch hint's share per tile: at most one request per lane
inline void share_prefetch(GemmArgs& g, int64_t tiles, int lanes) {
    if (g.pf_lines <= 0) return;
    const int64_t lpt = (g.pf_lines + tiles - 1) / tiles;
    g.pf_lpt = (int)(lpt < lanes ? lpt : lanes);
}
// Only regions of at most 8 MB are requested: a BERT-large weight matrix (1-4 MB) waits in the memory-side cache until
// its kernel starts and saves it 5-7 us of simultaneous first misses; GPT's 16-64 MB matrices are pushed out again by
// the activations written in between (FC1 alone writes 268 MB), and requesting them cost 0.3 % of the layer.
inline void set_prefetch(GemmArgs& g, const void* prefetch, size_t prefetch_bytes) {
    if (prefetch && prefetch_bytes >= 128 && prefetch_bytes <= ((size_t)8 << 20) && ((uintptr_t)prefetch & 3) == 0) {
        g.pf = (const int8_t*)prefetch;
        g.pf_lines = (int)(prefetch_bytes / 128);                // whole lines inside the region
    }
}

template <int BM, int BN, int WM, int WN, int EPI, int CDT, int RDT>
hero_status launch_persistent(const GemmArgs& g, int wg_per_cu, hipStream_t st) {
    GemmArgs gp = g;
    gp.ntm = (g.M + BM - 1) / BM; gp.ntn = (g.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)gp.ntm * gp.ntn;
    if (tiles > 0x7fffff00LL) return HERO_ERR_SHAPE;
    gp.per_xcd = (int)((tiles + NUM_XCD - 1) / NUM_XCD);
    share_prefetch(gp, tiles, WM * WN * 64);
    const int cap = 32 * wg_per_cu;                                   // 32 CUs per XCD
    const int nslot = gp.per_xcd < cap ? gp.per_xcd : cap;
    hipLaunchKernelGGL((int8_gemm_persistent_kernel<BM, BN, WM, WN, 4, EPI, CDT, RDT>), dim3((unsigned)(nslot * NUM_XCD)), dim3(WM * WN * 64), 0, st, gp);
    return hero_launch_status();
}

// The persistent kernel with the epilogue inside the next tile's main loop (256 x 128 tiles).
template <int EPI, int CDT>
hero_status launch_ovl(const GemmArgs& g, hipStream_t st) {
    GemmArgs gp = g;
    gp.ntm = (g.M + 255) / 256; gp.ntn = (g.N + 127) / 128;
    const int64_t tiles = (int64_t)gp.ntm * gp.ntn;
    if (tiles > 0x7fffff00LL) return HERO_ERR_SHAPE;
    gp.per_xcd = (int)((tiles + NUM_XCD - 1) / NUM_XCD);
    const int nslot = gp.per_xcd < 32 ? gp.per_xcd : 32;              // one workgroup per CU (152 KB of LDS), 32 CUs per XCD
    share_prefetch(gp, tiles, 512);
    hipLaunchKernelGGL((int8_gemm_ovl_kernel<EPI, CDT>), dim3((unsigned)(nslot * NUM_XCD)), dim3(512), 0, st, gp);
    return hero_launch_status();
}

// tile: -1 = chosen from the problem size (the product path); 0 = 128x128 register-staged, 1 = 256x256 one tile per
// workgroup, 2 = 64x64, 7 = 256x256 persistent, 8 = 128x128 persistent, 9 = 256x128 persistent with the overlapped
// epilogue (forced by the test entry point hero_int8_gemm_tile only; a forced kernel that cannot run the shape falls
// back to its one-tile-per-workgroup relative).
// 256 x 256 tiles, one workgroup per CU, or 128 x 128 tiles, two per CU?  Per full round the small tile is 10-15 % slower
// (twice the L2 -> LDS traffic), but the large one wastes what its last round leaves empty: 384 tiles on 256 CUs are
// one and a half rounds (8192 x 3072 x 1024, 16-bit output: 47.3 us against 42.0 with the small tile), 512 tiles are
// two full ones (8192 x 4096 x 1024: 40.7 against 43.6).  Compare the filled fractions, the small tile's scaled by 0.87.
inline bool small_tile_fills_better(int64_t t256, int64_t t128) {
    const double e256 = (double)t256 / (double)(((t256 + 255) / 256) * 256);
    const double e128 = 0.87 * (double)t128 / (double)(((t128 + 511) / 512) * 512);
    return e128 > e256;
}

template <int EPI, int CDT, int RDT>
hero_status launch_epi(const GemmArgs& g, void* ws, size_t ws_bytes, hipStream_t st, int tile) {
    int cfg = tile;
    if (cfg < 0 && ws) {                                               // skinny M with a workspace: split K
        const SplitK p = splitk_plan(g.M, g.N, g.K);
        if (p.ksplit > 1 && ws_bytes >= p.bytes) return launch_splitk<EPI, CDT, RDT>(g, p, ws, st);
    }
    // persistent kernels: K long enough that the slab ring never runs more than one tile ahead, whole pairs of
    // slabs, 32-bit per-lane offsets (256 rows of lda / ldb bytes)
    const bool pers_ok = g.K >= 4 * BK && g.K % (2 * BK) == 0 && g.lda < (1 << 24) && g.ldb < (1 << 24);
    // the overlapped-epilogue kernel: its epilogue is spread over the first 16 slabs of the next tile; no fused residual
    const bool ovl_ok = pers_ok && g.K >= 16 * BK && RDT < 0;
    if (cfg < 0) {
        const int64_t t256 = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256), t128 = (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
        if (t256 >= 160) cfg = !pers_ok ? 1 : (small_tile_fills_better(t256, t128) ? 8 : 7);
        else if (g.M <= 64 || t128 < 192) cfg = 2;
        else cfg = pers_ok ? 8 : 0;
    } else if (cfg == 9 && !ovl_ok) {
        cfg = pers_ok ? 7 : 1;
    } else if ((cfg == 7 || cfg == 8) && !pers_ok) {
        cfg = cfg == 7 ? 1 : 0;
    }
    // A GELU epilogue behind a short K goes to the overlapped-epilogue kernel: timed alone with resident operands it
    // is 3 % behind the 256 x 256 tile (95 against 92.5 us at 16384 x 4096 x 1024), but in a layer the weights come
    // from HBM and its six slabs of lookahead lose 4 us to that where the other loses 13 (rotating operands: 99.5
    // against 105.2 us; the 24-layer BERT-large stack 7.95 -> 7.75 ms).  From K = 4096 on its slower main loop
    // costs more than the hidden epilogue saves (GPT prefill, FC1 16384 x 16384 x 4096: +11 %).
    // Forcing each of the layer's other GEMMs (QKV, attention-output, FC2) to this kernel or to the 128 x 128 tiles
    // inside the stack made every one of them slower (7.46 -> 7.50-7.67 ms per 24 layers).
    constexpr bool GELU_EPI = EPI == HERO_EPI_GELU_REQUANT || EPI == HERO_EPI_DEQUANT_GELU;
    if (GELU_EPI && tile < 0 && cfg == 7 && ovl_ok && g.K < 2048) cfg = 9;
    if constexpr (RDT < 0) { if (cfg == 9) return launch_ovl<EPI, CDT>(g, st); }
    if (cfg == 7) return launch_persistent<256, 256, 2, 4, EPI, CDT, RDT>(g, 1, st);
    if (cfg == 8) return launch_persistent<128, 128, 2, 2, EPI, CDT, RDT>(g, 2, st);
    if (cfg == 1) return launch_grid(g, 256, 256, 512, int8_gemm_dma_kernel<256, 256, 2, 4, 4, 2, EPI, CDT, RDT>, st);
    if (cfg == 2) {                             // small or skinny problems: 64x64 tiles
        // few tiles and a long K: 4 groups of waves per workgroup split K (K / 64 must divide evenly);
        // measured: 8-10 % at 128 tiles or fewer, a loss with more tiles or with 2 groups
        const int64_t t64 = (int64_t)((g.M + 63) / 64) * ((g.N + 63) / 64);
        const int kt = g.K / BK;
        // One row of tiles (M <= 64: a decode step) streams the weight matrix once and is bound by how many of its
        // bytes are in flight.  Measured inside a layer, i.e. with weights that are NOT in the Infinity Cache (timed
        // alone and back to back the same kernels look 30 % faster than they are): up to 128 tiles, 64 x 32 tiles
        // with 8 slabs in flight in registers (64 x 4096 x 4096: 13.1 us against 16.6 for the four-K-group form);
        // beyond, two K groups per workgroup with 4 slabs each (64 x 12288 x 4096: 17.5 against 23.3 us for the
        // plain 64 x 64 tile; 64 x 16384 x 4096: 18.8-21.0 against 26.5-27.0; 8 or 16 slabs in flight, four K
        // groups or 64 x 32 tiles are all slower there).  More bytes in flight do not help beyond that: a form of
        // this kernel with two producer waves that kept seven 16 KB stages (112 KB per workgroup) on their way
        // straight into an LDS ring was correct and no faster (64 x 16384 x 4096: 23.4 us; with 64 workgroups, 64 x
        // 4096 x 16384: 51 us = 21 GB/s per compute unit).  A compute unit pulls about 21-23 GB/s from HBM whatever
        // it has outstanding (the decode attention reaches 5.9 TB/s with all 256 of them streaming), so what counts
        // is that every unit streams its 1/256 of the weights: 64-column tiles do that for N = 16384 and leave a
        // quarter of the chip idle for N = 12288.  Narrower strips do not fix that either: every workgroup also reads
        // all of the M x K activations (from the L2, but through the same per-unit path), so 16-column strips (tried
        // with 32-wide tiles whose upper half repeats the last owned column) move four times the activation bytes per
        // weight byte: 64 x 4096 x 4096 11.8 us (13.0 with 32 columns), 64 x 12288 x 4096 29-38 us (17.5),
        // 64 x 4096 x 16384 without a split 35-40 us (28 with the split and its reduction pass).
        if (g.M <= 64 && kt >= 32) {
            if (t64 <= 128) return launch_grid(g, 64, 32, 128, int8_gemm_kernel<64, 32, 2, 1, 8, 2, EPI, CDT, RDT>, st);
            if (kt % 2 == 0) return launch_grid(g, 64, 64, 512, int8_gemm_kernel<64, 64, 2, 2, 4, 1, EPI, CDT, RDT, false, 2>, st);
        }
        // Small problems (a BERT-base layer: 128 tokens) are bound by how many compute units stream the weights at
        // all, so the tiles shrink with the problem.  Measured as the layer runs them (weights in the caches): up to 32
        // tiles of 64 x 64, 32 x 32 tiles with four K groups (128 x 768 x 3072: 5.5 us against 8.4 for 64 x 64 with
        // four groups) or, with a short K, two (128 x 768 x 768: 3.9 against 4.4); up to 128 tiles, 64 x 32 tiles with
        // two K groups (128 x 2304 x 768: 4.2 against 4.6; 128 x 3072 x 768 + GELU^quant: 4.7 against 5.1;
        // 512 x 1024 x 4096: 8.6 against 10.2); beyond, plain 64 x 64 tiles (512 x 3072 x 1024: 7.2, every smaller
        // tile slower).
        if (t64 <= 32 && kt >= 32 && kt % 4 == 0)
            return launch_grid(g, 32, 32, 256, int8_gemm_kernel<32, 32, 1, 1, 4, 1, EPI, CDT, RDT, false, 4>, st);
        if (t64 <= 32 && kt % 2 == 0)
            return launch_grid(g, 32, 32, 128, int8_gemm_kernel<32, 32, 1, 1, 8, 2, EPI, CDT, RDT, false, 2>, st);
        if (t64 <= 128 && kt % 2 == 0)
            return launch_grid(g, 64, 32, 256, int8_gemm_kernel<64, 32, 2, 1, 4, 2, EPI, CDT, RDT, false, 2>, st);
        if (t64 <= 128 && kt >= 32 && kt % 4 == 0)
            return launch_grid(g, 64, 64, 1024, int8_gemm_kernel<64, 64, 2, 2, 2, 1, EPI, CDT, RDT, false, 4>, st);
        return launch_grid(g, 64, 64, 256, int8_gemm_kernel<64, 64, 2, 2, 2, 2, EPI, CDT, RDT>, st);
    }
    return launch_grid(g, 128, 128, 256, int8_gemm_kernel<128, 128, 2, 2, 2, 2, EPI, CDT, RDT>, st);
}

}  // namespace

// 16-bit operands (bf16 or fp16: the 16-bit side of a switched module) through the persistent kernels (called by
// hero_hp_gemm for large problems; HERO_ERR_UNSUPPORTED means "not this kernel's case", the caller then uses its
// own).  The tile is chosen as for INT8 operands; tile = 7 / 8 / 0 (from the test entry point hero_hp_gemm_tile)
// forces the 256x256 / 128x128 form / the caller's kernel, -1 chooses.
namespace {
template <int BM, int BN, int WM, int WN, int DT>
hero_status launch_hp_persistent(GemmArgs g, int wg_per_cu, bool gelu, hipStream_t st) {
    g.ntm = (g.M + BM - 1) / BM; g.ntn = (g.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)g.ntm * g.ntn;
    g.per_xcd = (int)((tiles + NUM_XCD - 1) / NUM_XCD);
    const int cap = 32 * wg_per_cu, nslot = g.per_xcd < cap ? g.per_xcd : cap;
    const dim3 grid((unsigned)(nslot * NUM_XCD)), block(WM * WN * 64);
    if (gelu) {
        if (g.residual) hipLaunchKernelGGL((int8_gemm_persistent_kernel<BM, BN, WM, WN, 4, HERO_EPI_DEQUANT_GELU, DT, DT, DT>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((int8_gemm_persistent_kernel<BM, BN, WM, WN, 4, HERO_EPI_DEQUANT_GELU, DT, -1, DT>), grid, block, 0, st, g);
    } else {
        if (g.residual) hipLaunchKernelGGL((int8_gemm_persistent_kernel<BM, BN, WM, WN, 4, HERO_EPI_DEQUANT, DT, DT, DT>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((int8_gemm_persistent_kernel<BM, BN, WM, WN, 4, HERO_EPI_DEQUANT, DT, -1, DT>), grid, block, 0, st, g);
    }
    return hero_launch_status();
}
}  // namespace

hero_status hero_hp_gemm_large(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                               const float* bias, const void* residual, int64_t ldr, int gelu,
                               void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, hipStream_t st, int tile) {
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256), t128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (t128 < 192 || t128 > 0x7fffff00LL || K % 64 != 0 || K * 2 < 4 * BK || lda * 2 >= (1 << 24) || ldb * 2 >= (1 << 24))
        return HERO_ERR_UNSUPPORTED;
    GemmArgs g;
    g.A = (const int8_t*)A; g.lda = lda * 2; g.a_row_scale = nullptr; g.Bt = (const int8_t*)Wt; g.ldb = ldb * 2;
    g.b_col_scale = nullptr; g.bias = bias; g.residual = residual; g.ldr = ldr; g.out_col_scale = nullptr;
    g.C = C; g.ldc = ldc; g.M = (int)M; g.N = (int)N; g.K = (int)(K * 2);
    g.ksplit = 1; g.kslabs = 0;
    const int cfg = tile >= 0 ? tile : ((t256 < 160 || small_tile_fills_better(t256, t128)) ? 8 : 7);
    if (cfg == 0) return HERO_ERR_UNSUPPORTED;
    if (dt == HERO_BF16) {
        if (cfg == 8) return launch_hp_persistent<128, 128, 2, 2, HERO_BF16>(g, 2, gelu != 0, st);
        return launch_hp_persistent<256, 256, 2, 4, HERO_BF16>(g, 1, gelu != 0, st);
    }
    if (cfg == 8) return launch_hp_persistent<128, 128, 2, 2, HERO_F16>(g, 2, gelu != 0, st);
    return launch_hp_persistent<256, 256, 2, 4, HERO_F16>(g, 1, gelu != 0, st);
}

// The FP8 variant: the same kernels with E4M3 operands (no split-K: fp32 partial sums would not commute).
template <int EPI, int CDT, int RDT>
hero_status launch_epi_fp8(GemmArgs g, hipStream_t st, int cfg) {
    const int64_t t256 = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256), t128 = (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
    const bool pers_ok = t128 <= 0x7fffff00LL && g.K >= 4 * BK && g.K % (2 * BK) == 0 && g.lda < (1 << 24) && g.ldb < (1 << 24);
    // cfg: -1 = chosen here; 0 / 7 / 8 forced by the test entry point hero_fp8_gemm_tile
    const bool small = g.M <= 64 || t128 < 192;
    if (pers_ok && (cfg == 7 || cfg == 8 || (cfg < 0 && !small))) {
        const bool tile128 = cfg == 8 || (cfg < 0 && (t256 < 160 || small_tile_fills_better(t256, t128)));
        g.ntm = tile128 ? (g.M + 127) / 128 : (g.M + 255) / 256; g.ntn = tile128 ? (g.N + 127) / 128 : (g.N + 255) / 256;
        g.per_xcd = (int)(((tile128 ? t128 : t256) + NUM_XCD - 1) / NUM_XCD);
        const int cap = tile128 ? 64 : 32, nslot = g.per_xcd < cap ? g.per_xcd : cap;
        share_prefetch(g, tile128 ? t128 : t256, tile128 ? 256 : 512);
        if (tile128) hipLaunchKernelGGL((int8_gemm_persistent_kernel<128, 128, 2, 2, 4, EPI, CDT, RDT, HERO_F8E4M3>), dim3((unsigned)(nslot * NUM_XCD)), dim3(256), 0, st, g);
        else hipLaunchKernelGGL((int8_gemm_persistent_kernel<256, 256, 2, 4, 4, EPI, CDT, RDT, HERO_F8E4M3>), dim3((unsigned)(nslot * NUM_XCD)), dim3(512), 0, st, g);
        return hero_launch_status();
    }
    if (small && cfg != 0) {
        // few tiles and a long K: four groups of waves per workgroup split K, as for INT8 operands
        const int64_t t64 = (int64_t)((g.M + 63) / 64) * ((g.N + 63) / 64);
        const int kt = g.K / BK;
        if (g.M <= 64 && kt >= 32) {                          // one row of tiles: the forms chosen for INT8 operands (cold weights)
            if (t64 <= 128 && kt < 128) return launch_grid(g, 64, 32, 128, int8_gemm_kernel<64, 32, 2, 1, 8, 2, EPI, CDT, RDT, false, 1, HERO_F8E4M3>, st);
            if (t64 > 128 && kt % 2 == 0) return launch_grid(g, 64, 64, 512, int8_gemm_kernel<64, 64, 2, 2, 4, 1, EPI, CDT, RDT, false, 2, HERO_F8E4M3>, st);
        }
        if (t64 <= 128 && kt >= 32 && kt % 4 == 0)
            return launch_grid(g, 64, 64, 1024, int8_gemm_kernel<64, 64, 2, 2, 2, 1, EPI, CDT, RDT, false, 4, HERO_F8E4M3>, st);
        return launch_grid(g, 64, 64, 256, int8_gemm_kernel<64, 64, 2, 2, 2, 2, EPI, CDT, RDT, false, 1, HERO_F8E4M3>, st);
    }
    return launch_grid(g, 128, 128, 256, int8_gemm_kernel<128, 128, 2, 2, 2, 2, EPI, CDT, RDT, false, 1, HERO_F8E4M3>, st);
}

static hero_status run_fp8_gemm(const void* A, int64_t lda, const float* a_row_scale,
                                const void* Bt, int64_t ldb, const float* b_col_scale,
                                const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                hero_epilogue epi, const float* out_col_scale,
                                void* C, hero_dtype c_dt, int64_t ldc,
                                int64_t M, int64_t N, int64_t K, void* stream, int tile,
                                const void* prefetch = nullptr, size_t prefetch_bytes = 0) {
    if (M < 0 || N < 0 || K <= 0) return HERO_ERR_SHAPE;
    if (M > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x7fffffffLL) return HERO_ERR_SHAPE;
    if (K % KMULT != 0) return HERO_ERR_UNSUPPORTED;
    if (lda < K || ldb < K || ldc < N) return HERO_ERR_SHAPE;
    if (M == 0 || N == 0) return HERO_OK;
    if (!A || !Bt || !C || !b_col_scale) return HERO_ERR_NULL;
    if (epi == HERO_EPI_GELU_REQUANT && !out_col_scale) return HERO_ERR_NULL;
    const bool c16 = c_dt == HERO_F16 || c_dt == HERO_BF16;
    switch (epi) {
    case HERO_EPI_DEQUANT: case HERO_EPI_DEQUANT_GELU: if (!c16) return HERO_ERR_UNSUPPORTED; break;
    case HERO_EPI_REQUANT: case HERO_EPI_GELU_REQUANT: if (c_dt != HERO_F8E4M3) return HERO_ERR_UNSUPPORTED; break;
    default: return HERO_ERR_UNSUPPORTED;
    }
    if (residual) {
        if (epi != HERO_EPI_DEQUANT || res_dt != c_dt) return HERO_ERR_UNSUPPORTED;
        if (ldr < N) return HERO_ERR_SHAPE;
        if (ldr % 4 != 0 || !hero_aligned16(residual)) return HERO_ERR_ALIGN;
    }
    if (lda % 16 != 0 || ldb % 16 != 0 || ldc % 4 != 0) return HERO_ERR_ALIGN;
    if (!hero_aligned16(A) || !hero_aligned16(Bt) || !hero_aligned16(C)) return HERO_ERR_ALIGN;
    GemmArgs g;
    g.A = (const int8_t*)A; g.lda = lda; g.a_row_scale = a_row_scale; g.Bt = (const int8_t*)Bt; g.ldb = ldb; g.b_col_scale = b_col_scale;
    g.bias = bias; g.residual = residual; g.ldr = ldr; g.out_col_scale = out_col_scale;
    g.C = C; g.ldc = ldc; g.M = (int)M; g.N = (int)N; g.K = (int)K;
    g.ksplit = 1; g.kslabs = 0;
    set_prefetch(g, prefetch, prefetch_bytes);
    hipStream_t st = (hipStream_t)stream;
    switch (epi) {
    case HERO_EPI_REQUANT: return launch_epi_fp8<HERO_EPI_REQUANT, HERO_F8E4M3, -1>(g, st, tile);
    case HERO_EPI_GELU_REQUANT: return launch_epi_fp8<HERO_EPI_GELU_REQUANT, HERO_F8E4M3, -1>(g, st, tile);
    case HERO_EPI_DEQUANT_GELU:
        return c_dt == HERO_BF16 ? launch_epi_fp8<HERO_EPI_DEQUANT_GELU, HERO_BF16, -1>(g, st, tile)
                                 : launch_epi_fp8<HERO_EPI_DEQUANT_GELU, HERO_F16, -1>(g, st, tile);
    default:
        if (!residual)
            return c_dt == HERO_BF16 ? launch_epi_fp8<HERO_EPI_DEQUANT, HERO_BF16, -1>(g, st, tile)
                                     : launch_epi_fp8<HERO_EPI_DEQUANT, HERO_F16, -1>(g, st, tile);
        return c_dt == HERO_BF16 ? launch_epi_fp8<HERO_EPI_DEQUANT, HERO_BF16, HERO_BF16>(g, st, tile)
                                 : launch_epi_fp8<HERO_EPI_DEQUANT, HERO_F16, HERO_F16>(g, st, tile);
    }
}

extern "C" size_t hero_int8_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    return splitk_plan(M, N, K).bytes;
}

extern "C" hero_status hero_int8_gemm(const int8_t* A, int64_t lda, const float* a_row_scale,
                                      const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                      const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                      hero_epilogue epi, const float* out_col_scale,
                                      void* C, hero_dtype c_dt, int64_t ldc,
                                      int64_t M, int64_t N, int64_t K, void* stream) {
    return hero_int8_gemm_ws(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                             C, c_dt, ldc, M, N, K, nullptr, 0, stream);
}

namespace {
// Everything that can be checked about a GeMM^quant request, before anything is launched.  *noop: nothing to do.
hero_status check_gemm_args(const int8_t* A, int64_t lda, const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                            const void* residual, hero_dtype res_dt, int64_t ldr, hero_epilogue epi,
                            const float* out_col_scale, void* C, hero_dtype c_dt, int64_t ldc,
                            int64_t M, int64_t N, int64_t K, bool* noop) {
    *noop = false;
    if (M < 0 || N < 0 || K <= 0) return HERO_ERR_SHAPE;
    if (M >= (1LL << 23) || N > 0x7fffffffLL || K > 0x7fffffffLL) return HERO_ERR_SHAPE;
    if (K % KMULT != 0) return HERO_ERR_UNSUPPORTED;
    if (lda < K || ldb < K || ldc < N) return HERO_ERR_SHAPE;
    if (M == 0 || N == 0) { *noop = true; return HERO_OK; }
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
        if (res_dt != c_dt) return HERO_ERR_UNSUPPORTED;
        if (ldr < N) return HERO_ERR_SHAPE;
        if (ldr % 4 != 0 || !hero_aligned16(residual)) return HERO_ERR_ALIGN;
    }
    if (lda % 16 != 0 || ldb % 16 != 0 || ldc % 4 != 0) return HERO_ERR_ALIGN;
    if (!hero_aligned16(A) || !hero_aligned16(Bt) || !hero_aligned16(C)) return HERO_ERR_ALIGN;
    return HERO_OK;
}
}  // namespace

static hero_status run_int8_gemm(const int8_t* A, int64_t lda, const float* a_row_scale,
                                 const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                 const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                 hero_epilogue epi, const float* out_col_scale,
                                 void* C, hero_dtype c_dt, int64_t ldc,
                                 int64_t M, int64_t N, int64_t K,
                                 void* workspace, size_t workspace_bytes, void* stream, int tile,
                                 const void* prefetch = nullptr, size_t prefetch_bytes = 0) {
    if (workspace && ((uintptr_t)workspace & 255)) return HERO_ERR_WORKSPACE;
    bool noop = false;
    const hero_status cs = check_gemm_args(A, lda, Bt, ldb, b_col_scale, residual, res_dt, ldr, epi, out_col_scale,
                                           C, c_dt, ldc, M, N, K, &noop);
    if (cs != HERO_OK || noop) return cs;

    GemmArgs g;
    g.A = A; g.lda = lda; g.a_row_scale = a_row_scale; g.Bt = Bt; g.ldb = ldb; g.b_col_scale = b_col_scale;
    g.bias = bias; g.residual = residual; g.ldr = ldr; g.out_col_scale = out_col_scale;
    g.C = C; g.ldc = ldc; g.M = (int)M; g.N = (int)N; g.K = (int)K;
    g.ksplit = 1; g.kslabs = 0;
    set_prefetch(g, prefetch, prefetch_bytes);
    hipStream_t st = (hipStream_t)stream;
    switch (epi) {
    case HERO_EPI_RAW_I32: return launch_epi<HERO_EPI_RAW_I32, HERO_I32, -1>(g, workspace, workspace_bytes, st, tile);
    case HERO_EPI_REQUANT: return launch_epi<HERO_EPI_REQUANT, HERO_I8, -1>(g, workspace, workspace_bytes, st, tile);
    case HERO_EPI_GELU_REQUANT: return launch_epi<HERO_EPI_GELU_REQUANT, HERO_I8, -1>(g, workspace, workspace_bytes, st, tile);
    case HERO_EPI_DEQUANT_GELU:
        return c_dt == HERO_BF16 ? launch_epi<HERO_EPI_DEQUANT_GELU, HERO_BF16, -1>(g, workspace, workspace_bytes, st, tile)
                                 : launch_epi<HERO_EPI_DEQUANT_GELU, HERO_F16, -1>(g, workspace, workspace_bytes, st, tile);
    case HERO_EPI_DEQUANT:
        if (!residual)
            return c_dt == HERO_BF16 ? launch_epi<HERO_EPI_DEQUANT, HERO_BF16, -1>(g, workspace, workspace_bytes, st, tile)
                                     : launch_epi<HERO_EPI_DEQUANT, HERO_F16, -1>(g, workspace, workspace_bytes, st, tile);
        if (c_dt == HERO_BF16) return launch_epi<HERO_EPI_DEQUANT, HERO_BF16, HERO_BF16>(g, workspace, workspace_bytes, st, tile);
        return launch_epi<HERO_EPI_DEQUANT, HERO_F16, HERO_F16>(g, workspace, workspace_bytes, st, tile);
    default: return HERO_ERR_UNSUPPORTED;
    }
}

// hero_int8_gemm_ws for a caller that knows what its chain reads next (hero_layer_fwd: the next module's weights):
// the large-problem kernels request that memory while they run, the others ignore the hint.  Not part of the C ABI.
hero_status hero_int8_gemm_prefetching(const int8_t* A, int64_t lda, const float* a_row_scale,
                                       const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                       const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                       hero_epilogue epi, const float* out_col_scale,
                                       void* C, hero_dtype c_dt, int64_t ldc,
                                       int64_t M, int64_t N, int64_t K,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       const void* prefetch, size_t prefetch_bytes) {
    return run_int8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                         C, c_dt, ldc, M, N, K, workspace, workspace_bytes, stream, -1, prefetch, prefetch_bytes);
}

hero_status hero_fp8_gemm_prefetching(const void* A, int64_t lda, const float* a_row_scale,
                                      const void* Bt, int64_t ldb, const float* b_col_scale,
                                      const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                      hero_epilogue epi, const float* out_col_scale,
                                      void* C, hero_dtype c_dt, int64_t ldc,
                                      int64_t M, int64_t N, int64_t K, void* stream,
                                      const void* prefetch, size_t prefetch_bytes) {
    return run_fp8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                        C, c_dt, ldc, M, N, K, stream, -1, prefetch, prefetch_bytes);
}

extern "C" hero_status hero_int8_gemm_ws(const int8_t* A, int64_t lda, const float* a_row_scale,
                                         const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                         const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                         hero_epilogue epi, const float* out_col_scale,
                                         void* C, hero_dtype c_dt, int64_t ldc,
                                         int64_t M, int64_t N, int64_t K,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    return run_int8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                         C, c_dt, ldc, M, N, K, workspace, workspace_bytes, stream, -1);
}

extern "C" hero_status hero_fp8_gemm(const void* A, int64_t lda, const float* a_row_scale,
                                     const void* Bt, int64_t ldb, const float* b_col_scale,
                                     const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                     hero_epilogue epi, const float* out_col_scale,
                                     void* C, hero_dtype c_dt, int64_t ldc,
                                     int64_t M, int64_t N, int64_t K, void* stream) {
    return run_fp8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                        C, c_dt, ldc, M, N, K, stream, -1);
}

// Test and tuning hooks (include/hero_debug.h): the same calls with the kernel choice forced.
extern "C" hero_status hero_int8_gemm_tile(const int8_t* A, int64_t lda, const float* a_row_scale,
                                           const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                           const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                           hero_epilogue epi, const float* out_col_scale,
                                           void* C, hero_dtype c_dt, int64_t ldc,
                                           int64_t M, int64_t N, int64_t K, void* stream, int tile) {
    if (tile != 0 && tile != 1 && tile != 2 && tile != 7 && tile != 8 && tile != 9) return HERO_ERR_UNSUPPORTED;
    return run_int8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                         C, c_dt, ldc, M, N, K, nullptr, 0, stream, tile);
}

extern "C" hero_status hero_fp8_gemm_tile(const void* A, int64_t lda, const float* a_row_scale,
                                          const void* Bt, int64_t ldb, const float* b_col_scale,
                                          const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                          hero_epilogue epi, const float* out_col_scale,
                                          void* C, hero_dtype c_dt, int64_t ldc,
                                          int64_t M, int64_t N, int64_t K, void* stream, int tile) {
    if (tile != 0 && tile != 7 && tile != 8) return HERO_ERR_UNSUPPORTED;
    return run_fp8_gemm(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                        C, c_dt, ldc, M, N, K, stream, tile);
}

// ---- hero_int8_gemm_static: the split-K scratch lives in the library ---------------------------------------
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid hipMalloc).  The
// array below exists once per GPU the library is loaded on, until the process ends.  Its name is a host-side
// stand-in, not a device address: the address is asked for once per device (hipGetSymbolAddress with that
// device current) and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[HERO_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES];                         // per device; racing first calls store the same value

hero_status static_scratch_ptr(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return HERO_ERR_LAUNCH;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HERO_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return HERO_OK;
}
}  // namespace

extern "C" hero_status hero_int8_gemm_static(const int8_t* A, int64_t lda, const float* a_row_scale,
                                             const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                             const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                             hero_epilogue epi, const float* out_col_scale,
                                             void* C, hero_dtype c_dt, int64_t ldc,
                                             int64_t M, int64_t N, int64_t K, void* stream) {
    bool noop = false;
    const hero_status cs = check_gemm_args(A, lda, Bt, ldb, b_col_scale, residual, res_dt, ldr, epi, out_col_scale,
                                           C, c_dt, ldc, M, N, K, &noop);
    if (cs != HERO_OK || noop) return cs;
    const size_t need = splitk_plan(M, N, K).bytes;
    if (need > (size_t)HERO_STATIC_SCRATCH_BYTES) return HERO_ERR_WORKSPACE;   // beyond the built-in scratch
    void* ws = nullptr;
    if (need) {
        const hero_status ss = static_scratch_ptr(&ws);
        if (ss != HERO_OK) return ss;
    }
    return hero_int8_gemm_ws(A, lda, a_row_scale, Bt, ldb, b_col_scale, bias, residual, res_dt, ldr, epi, out_col_scale,
                             C, c_dt, ldc, M, N, K, ws, need, stream);
}
