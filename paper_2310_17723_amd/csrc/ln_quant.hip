// hero_ln_quant: LN^quant, the fused LayerNorm + token-wise (TWQ) INT8 quantization
// (paper Sec. 2.1 TWQ paragraph; Sec. 2.2.2 last line of the quantized attention flow;
// Sec. 2.2.3 last line of the quantized MLP flow).
//
// HBM-bound: every input element is read once and every output element written once.
//   * One wavefront owns one row at a time and keeps it in registers (NCH chunks of EPL
//     elements per lane; a chunk is one 128-bit load per lane, consecutive lanes consecutive
//     addresses).  Workgroups are persistent and wide (up to 16 waves, one workgroup per CU for
//     large inputs): a wave walks rows with a grid-sized stride and has the loads of the next
//     row in flight while it works on the current one.  The fetched registers are passed
//     through an empty asm statement at the top of each row so that the compiler cannot hoist
//     their first use (and with it the wait for the loads) up to the point of issue.
//   * gamma, beta and the FWQ column scale are staged in LDS once per workgroup, not re-read
//     from the caches per row.
//   * INT8 codes are unpacked with one SDWA conversion each (sign-extending byte select).
//   * The three row reductions (sum, sum of squared deviations, absmax) run on the DPP
//     cross-lane network (quad_perm / row_mirror / row_bcast), no LDS round trips.
//   * Statistics are fp32, mean first and variance about the mean.
//   * Codes are rne(y / s) with IEEE fp32 division BY DEFINITION.  Without LayerNorm (pure
//     per-token quantization, bit-exact by contract) the kernel multiplies by 1/s and falls back
//     to the true division for the rare lanes whose product lies within 4e-5 of a rounding tie,
//     the only place where the two can disagree; rounding and the two's-complement byte come out
//     of one fp32 add of 1.5 * 2^23.  Behind a LayerNorm the fp32 statistics already differ from
//     the definition's fp64 ones by more than that, so the +-1 LSB class applies: hardware
//     reciprocal / reciprocal square root, and v_cvt_pk_u8_f32 of y/s + 128 rounds, saturates
//     and packs in one instruction (the offset is removed by an XOR of the packed dword).
#include "hero_common.h"
#include <atomic>
#include <type_traits>

namespace {

struct LnArgs {
    const void* x; const float* x_row_scale;
    const void* r; const float* r_col_scale;
    const float* gamma; const float* beta;
    float eps; int64_t M; int D;
    int8_t* y_q; float* y_scale; void* y_hp;
    int x_dt, r_dt, hp_dt;       // r_dt / hp_dt = -1 when absent
    int y_fp8;                   // token-wise E4M3 codes (scale max|y| / 448) instead of INT8 codes
    int in_fp8;                  // the 8-bit inputs (x and / or r with x_dt / r_dt = HERO_I8 here) hold E4M3 codes
    // gathered form (embedding): row i of x / r / r2 is row x_idx[i] / r_idx[i] / r2_idx[i] of a table
    // with x_rows / r_rows / r2_rows rows (indices are clamped into the table); r2 is a third addend in r_dt
    const int32_t* x_idx; const int32_t* r_idx; const void* r2; const int32_t* r2_idx;
    int x_rows, r_rows, r2_rows;
};

// sign-extended byte B of w -> fp32 in one instruction
template <int B>
__device__ __forceinline__ float sbyte_f32(int w) {
    float r;
    if constexpr (B == 0) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0" : "=v"(r) : "v"(w));
    else if constexpr (B == 1) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(r) : "v"(w));
    else if constexpr (B == 2) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(r) : "v"(w));
    else asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3" : "=v"(r) : "v"(w));
    return r;
}
// the four codes of one dword: INT8, or E4M3 (v_cvt_f32_fp8 with a byte select) when f8 (wave-uniform)
__device__ __forceinline__ void unpack4(int w, float (&o)[4], bool f8 = false) {
    if (f8) {
        o[0] = __builtin_amdgcn_cvt_f32_fp8(w, 0); o[1] = __builtin_amdgcn_cvt_f32_fp8(w, 1);
        o[2] = __builtin_amdgcn_cvt_f32_fp8(w, 2); o[3] = __builtin_amdgcn_cvt_f32_fp8(w, 3);
    } else {
        o[0] = sbyte_f32<0>(w); o[1] = sbyte_f32<1>(w); o[2] = sbyte_f32<2>(w); o[3] = sbyte_f32<3>(w);
    }
}

// ---- 64-lane reductions on the DPP network; the result is wave-uniform ---------------------------
template <bool IS_MAX>
__device__ __forceinline__ float dpp_step(float x, float y) { return IS_MAX ? fmaxf(x, y) : x + y; }
template <bool IS_MAX>
__device__ __forceinline__ float wave_reduce(float x) {
    int xi;
#define HERO_DPP(ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, 0xF, 0xF, true))
    x = dpp_step<IS_MAX>(x, HERO_DPP(0xB1));      // quad_perm [1,0,3,2]
    x = dpp_step<IS_MAX>(x, HERO_DPP(0x4E));      // quad_perm [2,3,0,1]
    x = dpp_step<IS_MAX>(x, HERO_DPP(0x141));     // row_half_mirror: 8 lanes
    x = dpp_step<IS_MAX>(x, HERO_DPP(0x140));     // row_mirror: 16 lanes (every lane holds its row's value)
#undef HERO_DPP
    // rows 1,3 take lane 15 of the row before; then rows 2,3 take lane 31: lane 63 has all four rows
    xi = __builtin_amdgcn_update_dpp(IS_MAX ? __builtin_bit_cast(int, -INFINITY) : 0, __builtin_bit_cast(int, x), 0x142, 0xA, 0xF, false);
    x = dpp_step<IS_MAX>(x, __builtin_bit_cast(float, xi));
    xi = __builtin_amdgcn_update_dpp(IS_MAX ? __builtin_bit_cast(int, -INFINITY) : 0, __builtin_bit_cast(int, x), 0x143, 0xC, 0xF, false);
    x = dpp_step<IS_MAX>(x, __builtin_bit_cast(float, xi));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

template <int DT, int EPL>
__device__ __forceinline__ void store_hp(const float (&v)[EPL], uint16_t* dst) {
#pragma unroll
    for (int e8 = 0; e8 < EPL / 8; ++e8) {
        v4i o;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            o[p] = (int)pack2_hp<DT>(v[8 * e8 + 2 * p], v[8 * e8 + 2 * p + 1]);
        *reinterpret_cast<v4i*>(dst + 8 * e8) = o;
    }
}

constexpr int ln_max_waves(int nch) { return nch <= 2 ? 16 : (nch == 4 ? 8 : 4); }   // per workgroup: the row must fit the registers

// XDT: HERO_I8 / HERO_BF16 / HERO_F16.  RDT: -1 (no second addend) / HERO_I8 / HERO_BF16 / HERO_F16.
template <int XDT, int RDT, int NCH, bool HAS_LN, bool GATHER = false>
__global__ __launch_bounds__(64 * ln_max_waves(NCH)) void ln_quant_kernel(LnArgs a) {
    static_assert(!GATHER || (XDT == HERO_I8 && (RDT == HERO_BF16 || RDT == HERO_F16) && HAS_LN), "gathered form: INT8 table + 16-bit tables");
    constexpr bool X_I8 = XDT == HERO_I8;
    constexpr int EPL = X_I8 ? 16 : 8;
    constexpr int CH = EPL * HERO_WAVE;
    constexpr bool r_i8 = RDT == HERO_I8, r_hp = RDT == HERO_BF16 || RDT == HERO_F16;
    // rows in flight ahead of the current one.  Measured at D = 1024 (one 16-wave workgroup per CU): two rows ahead
    // (25 more registers) and gamma / beta / S_o held in registers instead of LDS (no staging, no barrier before the
    // first row; 35 more registers) are both 5-12 % SLOWER at 16384 rows and equal at 65536: the kernel runs at the
    // rate of a plain copy of the same size once it streams, what is left is the ramp of a 15 us launch.
    constexpr int PF = 1;
    extern __shared__ __attribute__((aligned(16))) float sp[];   // [3][Dp]: gamma, beta, r_col_scale
    const int D = a.D, Dp = NCH * CH;
    const int tid = threadIdx.x, lane = tid & 63, nwb = blockDim.x >> 6;
    const int64_t tw = (int64_t)gridDim.x * nwb;              // waves in the grid = row stride of a wave
    int64_t row = (int64_t)blockIdx.x * nwb + (tid >> 6);

    // raw data of the rows in flight
    v4i rx[PF][NCH], rr0[PF][NCH], rr1[PF][NCH], rs0[GATHER ? NCH : 1], rs1[GATHER ? NCH : 1];
    float xsr[PF];
    // gathered form: the table rows of the NEXT fetch, looked up one row earlier than the data they address
    int gx = 0, gr = 0, g2 = 0;
    const bool has_r2 = GATHER && a.r2 != nullptr;
    auto lookup = [&](int64_t rw) {
        if (!GATHER || rw >= a.M) return;
        gx = min(max(a.x_idx[rw], 0), a.x_rows - 1);
        gr = min(max(a.r_idx[rw], 0), a.r_rows - 1);
        if (has_r2) g2 = min(max(a.r2_idx[rw], 0), a.r2_rows - 1);
    };
    auto fetch = [&](int64_t rw, auto P) {
        constexpr int p = decltype(P)::value;
        if (rw >= a.M) return;                                // wave-uniform
        const int64_t xrow = GATHER ? gx : rw, rrow = GATHER ? gr : rw;
        xsr[p] = X_I8 ? a.x_row_scale[xrow] : 1.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j0 = c * CH + lane * EPL;
            if (j0 < D) {
                const int64_t off = xrow * (int64_t)D + j0, roff = rrow * (int64_t)D + j0;
                rx[p][c] = X_I8 ? *reinterpret_cast<const v4i*>((const int8_t*)a.x + off)
                                : *reinterpret_cast<const v4i*>((const uint16_t*)a.x + off);
                if constexpr (r_i8) {
                    if constexpr (EPL == 16) rr0[p][c] = *reinterpret_cast<const v4i*>((const int8_t*)a.r + roff);
                    else { v2i t = *reinterpret_cast<const v2i*>((const int8_t*)a.r + roff); rr0[p][c][0] = t[0]; rr0[p][c][1] = t[1]; }
                } else if constexpr (r_hp) {
                    rr0[p][c] = *reinterpret_cast<const v4i*>((const uint16_t*)a.r + roff);
                    if constexpr (EPL == 16) rr1[p][c] = *reinterpret_cast<const v4i*>((const uint16_t*)a.r + roff + 8);
                }
                if constexpr (GATHER) {
                    if (has_r2) {
                        const int64_t off2 = (int64_t)g2 * D + j0;
                        rs0[c] = *reinterpret_cast<const v4i*>((const uint16_t*)a.r2 + off2);
                        rs1[c] = *reinterpret_cast<const v4i*>((const uint16_t*)a.r2 + off2 + 8);
                    }
                }
            }
        }
    };
    lookup(row);
    fetch(row, std::integral_constant<int, 0>{});             // in flight while the parameters are staged
    if constexpr (PF > 1) fetch(row + tw, std::integral_constant<int, PF - 1>{});
    lookup(row + PF * tw);

    // parameters -> LDS, 8 columns per thread and round with all their loads issued before the first LDS
    // store (one memory latency per round, not one per column: this is the whole cost of a small launch)
    for (int j0 = tid; j0 < Dp; j0 += 8 * blockDim.x) {
        float pg[8], pb[8], pr[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int j = j0 + k * blockDim.x;
            const bool in = j < D;
            pg[k] = (HAS_LN && in) ? a.gamma[j] : 0.0f;
            pb[k] = (HAS_LN && a.beta && in) ? a.beta[j] : 0.0f;
            pr[k] = (r_i8 && in) ? a.r_col_scale[j] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int j = j0 + k * blockDim.x;
            if (j < Dp) {
                // column j = chunk c, lane l, element 4*e4 + t  ->  [c][e4][l][t]: a wave's 128-bit read of one
                // (c, e4) then covers 64 consecutive 16-byte slots (no bank conflicts)
                const int w = j % CH, pos = (((j / CH) * (EPL / 4) + (w % EPL) / 4) * 64 + w / EPL) * 4 + (w % 4);
                sp[pos] = pg[k]; sp[Dp + pos] = pb[k]; sp[2 * Dp + pos] = pr[k];
            }
        }
    }
    __syncthreads();
    if (row >= a.M) return;
    const bool in_f8 = !GATHER && a.in_fp8 != 0;
    const float inv_d = 1.0f / (float)D;

    auto process = [&](int64_t row, auto P) {
        constexpr int p = decltype(P)::value;
        // first use of the fetched registers: nothing that reads them may move above this point
        asm volatile("" : "+v"(xsr[p]));
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            asm volatile("" : "+v"(rx[p][c]));
            if constexpr (r_i8 || r_hp) asm volatile("" : "+v"(rr0[p][c]));
            if constexpr (r_hp && EPL == 16) asm volatile("" : "+v"(rr1[p][c]));
            if constexpr (GATHER) { asm volatile("" : "+v"(rs0[c])); asm volatile("" : "+v"(rs1[c])); }
        }
        float v[NCH][EPL];
        const float xs = xsr[p];
        // ---- unpack the fetched row into fp32 (sum of the addends) ---------------------------
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j0 = c * CH + lane * EPL;
            if (j0 < D) {
                if constexpr (X_I8) {
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        float f[4];
                        unpack4(rx[p][c][e4], f, in_f8);
#pragma unroll
                        for (int t = 0; t < 4; ++t) v[c][4 * e4 + t] = f[t] * xs;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        uint32_t h = ((uint32_t)rx[p][c][e >> 1] >> (16 * (e & 1))) & 0xffffu;
                        v[c][e] = hp_to_f32<XDT>(h);
                    }
                }
                if constexpr (r_i8) {
#pragma unroll
                    for (int e4 = 0; e4 < EPL / 4; ++e4) {
                        float f[4];
                        unpack4(rr0[p][c][e4], f, in_f8);
                        const v4f rc = *reinterpret_cast<const v4f*>(sp + 2 * Dp + ((c * (EPL / 4) + e4) * 64 + lane) * 4);
#pragma unroll
                        for (int t = 0; t < 4; ++t) v[c][4 * e4 + t] = fmaf(f[t], rc[t], v[c][4 * e4 + t]);
                    }
                } else if constexpr (r_hp) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) {
                        const int w = e < 8 ? rr0[p][c][(e & 7) >> 1] : rr1[p][c][(e & 7) >> 1];
                        uint32_t h = ((uint32_t)w >> (16 * (e & 1))) & 0xffffu;
                        v[c][e] += hp_to_f32<RDT>(h);
                    }
                    if constexpr (GATHER) {
                        if (has_r2) {
#pragma unroll
                            for (int e = 0; e < EPL; ++e) {
                                const int w = e < 8 ? rs0[c][(e & 7) >> 1] : rs1[c][(e & 7) >> 1];
                                uint32_t h = ((uint32_t)w >> (16 * (e & 1))) & 0xffffu;
                                v[c][e] += hp_to_f32<RDT>(h);
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) v[c][e] = 0.0f;
            }
        }
        // ---- the loads of the row PF strides ahead go out now, into the register set just unpacked
        fetch(row + PF * tw, P);
        lookup(row + 2 * PF * tw);

        // ---- LayerNorm: mean, then variance about the mean (fp32) --------------------------
        if constexpr (HAS_LN) {
            float s = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int e = 0; e < EPL; ++e) s += v[c][e];
            const float mean = wave_reduce<false>(s) * inv_d;
            float q = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                // a lane whose chunk lies in the padding (columns >= D; it holds zeros) stays out of the sum of
                // squared deviations: it subtracts 0 instead of the mean
                const float mean_c = c * CH + lane * EPL < D ? mean : 0.0f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    const float dlt = v[c][e] - mean_c;
                    v[c][e] = dlt;
                    q = fmaf(dlt, dlt, q);
                }
            }
            const float var = wave_reduce<false>(q) * inv_d;
            const float rstd = __builtin_amdgcn_rsqf(var + a.eps);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                // (padded columns have gamma = beta = 0)
#pragma unroll
                for (int e4 = 0; e4 < EPL / 4; ++e4) {
                    const v4f g = *reinterpret_cast<const v4f*>(sp + ((c * (EPL / 4) + e4) * 64 + lane) * 4);
                    const v4f b = *reinterpret_cast<const v4f*>(sp + Dp + ((c * (EPL / 4) + e4) * 64 + lane) * 4);
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[c][4 * e4 + t] = fmaf(v[c][4 * e4 + t] * rstd, g[t], b[t]);
                }
            }
        }

        // ---- token-wise scale and codes -------------------------------------------------------
        float amax = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(v[c][e]));
        amax = wave_reduce<true>(amax);
        const float sc = amax == 0.0f ? 1.0f : __fdiv_rn(amax, a.y_fp8 ? 448.0f : 127.0f);
        const float inv_sc = HAS_LN ? __builtin_amdgcn_rcpf(sc) : __fdiv_rn(1.0f, sc);
        if (lane == 0) a.y_scale[row] = sc;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j0 = c * CH + lane * EPL;
            if (j0 >= D) continue;
            const int64_t off = row * (int64_t)D + j0;
            uint32_t pk[EPL / 4];
            if (a.y_fp8) {
                // FP8 output (the variant of Sec. 2.1's 8-bit format): E4M3 of the true quotient, round to
                // nearest even; |y / s| <= 448 (1 + 2^-23) is clamped to the format's range
#pragma unroll
                for (int e4 = 0; e4 < EPL / 4; ++e4)
                    pk[e4] = fp8x4_sat(__fdiv_rn(v[c][4 * e4], sc), __fdiv_rn(v[c][4 * e4 + 1], sc),
                                       __fdiv_rn(v[c][4 * e4 + 2], sc), __fdiv_rn(v[c][4 * e4 + 3], sc));
            } else if constexpr (HAS_LN) {
                // |v * inv_sc| <= 127 (1 + 2^-22): v * inv_sc + 128 rounds into 1 .. 255
#pragma unroll
                for (int e4 = 0; e4 < EPL / 4; ++e4) {
                    uint32_t w = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        w = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(v[c][4 * e4 + t], inv_sc, 128.0f), t, w);
                    pk[e4] = w ^ 0x80808080u;
                }
            } else {
                // |v * inv_sc| <= 127 (absmax row scale), so no clamp is needed before the rounding add
                float t[EPL];
                bool near_tie = false;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    t[e] = v[c][e] * inv_sc;
                    near_tie |= fabsf(t[e] - __builtin_rintf(t[e])) > 0.49996f;
                }
                if (near_tie) {                              // rare: redo this lane's chunk with the true division
#pragma unroll
                    for (int e = 0; e < EPL; ++e) t[e] = __fdiv_rn(v[c][e], sc);
                }
#pragma unroll
                for (int e4 = 0; e4 < EPL / 4; ++e4)
                    pk[e4] = pack_low_bytes(rne_low_byte(t[4 * e4]), rne_low_byte(t[4 * e4 + 1]),
                                            rne_low_byte(t[4 * e4 + 2]), rne_low_byte(t[4 * e4 + 3]));
            }
            if constexpr (EPL == 16) {
                v4i o = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3]};
                *reinterpret_cast<v4i*>(a.y_q + off) = o;
            } else {
                v2i o = {(int)pk[0], (int)pk[1]};
                *reinterpret_cast<v2i*>(a.y_q + off) = o;
            }
            if (a.hp_dt == HERO_BF16) store_hp<HERO_BF16, EPL>(v[c], (uint16_t*)a.y_hp + off);
            else if (a.hp_dt == HERO_F16) store_hp<HERO_F16, EPL>(v[c], (uint16_t*)a.y_hp + off);
        }
    };
    // register sets rotate with the row: unrolled by PF so the set index is a compile-time constant
    for (;;) {
        process(row, std::integral_constant<int, 0>{});
        row += tw;
        if (row >= a.M) break;
        if constexpr (PF > 1) {
            process(row, std::integral_constant<int, PF - 1>{});
            row += tw;
            if (row >= a.M) break;
        }
    }
}

template <int XDT, int RDT, int NCH, bool GATHER = false>
hero_status launch_nch(const LnArgs& a, hipStream_t st) {
    constexpr int CH = (XDT == HERO_I8 ? 16 : 8) * HERO_WAVE;
    const size_t lds = (size_t)3 * NCH * CH * sizeof(float);
    const bool has_ln = a.gamma != nullptr;
    const void* fn = GATHER ? (const void*)ln_quant_kernel<XDT, RDT, NCH, true, GATHER>
                   : has_ln ? (const void*)ln_quant_kernel<XDT, RDT, NCH, true> : (const void*)ln_quant_kernel<XDT, RDT, NCH, false>;
    if (lds > 65536) {                                    // more than 64 KB of dynamic LDS needs the opt-in: once per device
        static std::atomic<bool> raised[3][64];
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return HERO_ERR_LAUNCH;
        std::atomic<bool>& done = raised[GATHER ? 2 : (has_ln ? 1 : 0)][dev];
        if (!done.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return HERO_ERR_LAUNCH;
            done.store(true, std::memory_order_release);
        }
    }
    // persistent workgroups: wide ones (one per CU) once every CU has several rows per wave, else
    // 4-wave workgroups, never more than the rows need.  Measured at D = 1024, 16384 and 65536 rows: more waves
    // per CU than these 16 (2 x 16, 2 x 12, 2-4 x 8, 4-8 x 4 per CU, which the 72 registers of the kernel allow)
    // are all equal or 2-10 % slower; rows in flight are not what bounds the kernel.
    constexpr int MAXW = ln_max_waves(NCH);
    const int wpb = a.M >= 256 * MAXW ? MAXW : 4;
    int64_t blocks = (a.M + wpb - 1) / wpb;
    const int64_t cap = 256 * (MAXW / wpb);
    if (blocks > cap) blocks = cap;
    if constexpr (GATHER) hipLaunchKernelGGL((ln_quant_kernel<XDT, RDT, NCH, true, true>), dim3((unsigned)blocks), dim3(64 * wpb), lds, st, a);
    else if (has_ln) hipLaunchKernelGGL((ln_quant_kernel<XDT, RDT, NCH, true>), dim3((unsigned)blocks), dim3(64 * wpb), lds, st, a);
    else hipLaunchKernelGGL((ln_quant_kernel<XDT, RDT, NCH, false>), dim3((unsigned)blocks), dim3(64 * wpb), lds, st, a);
    return hero_launch_status();
}

template <int XDT, int RDT>
hero_status launch_r(const LnArgs& a, hipStream_t st) {
    constexpr int CH = (XDT == HERO_I8 ? 16 : 8) * HERO_WAVE;
    const int nch = (a.D + CH - 1) / CH;
    if (nch <= 1) return launch_nch<XDT, RDT, 1>(a, st);
    if (nch <= 2) return launch_nch<XDT, RDT, 2>(a, st);
    if (nch <= 4) return launch_nch<XDT, RDT, 4>(a, st);
    if (nch <= 8) return launch_nch<XDT, RDT, 8>(a, st);
    return HERO_ERR_UNSUPPORTED;
}

template <int RDT>
hero_status launch_gather(const LnArgs& a, hipStream_t st) {
    const int nch = (a.D + 16 * HERO_WAVE - 1) / (16 * HERO_WAVE);
    if (nch <= 1) return launch_nch<HERO_I8, RDT, 1, true>(a, st);
    if (nch <= 2) return launch_nch<HERO_I8, RDT, 2, true>(a, st);
    if (nch <= 4) return launch_nch<HERO_I8, RDT, 4, true>(a, st);
    if (nch <= 8) return launch_nch<HERO_I8, RDT, 8, true>(a, st);
    return HERO_ERR_UNSUPPORTED;
}

template <int XDT>
hero_status launch(const LnArgs& a, hipStream_t st) {
    switch (a.r_dt) {
    case -1: return launch_r<XDT, -1>(a, st);
    case HERO_I8: return launch_r<XDT, HERO_I8>(a, st);
    case HERO_BF16: return launch_r<XDT, HERO_BF16>(a, st);
    case HERO_F16: return launch_r<XDT, HERO_F16>(a, st);
    }
    return HERO_ERR_UNSUPPORTED;
}

hero_status ln_quant_entry(const void* x, hero_dtype x_dt, const float* x_row_scale,
                           const void* r, hero_dtype r_dt, const float* r_col_scale,
                           const float* gamma, const float* beta, float eps,
                           int64_t M, int64_t D,
                           void* y_q, int y_fp8, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream) {
    if (M < 0 || D <= 0) return HERO_ERR_SHAPE;
    if (D % 16 != 0) return HERO_ERR_UNSUPPORTED;
    if (M == 0) return HERO_OK;
    if (!x || !y_q || !y_scale) return HERO_ERR_NULL;
    // 8-bit inputs: INT8 codes or E4M3 codes (one format per call: the kernels unpack both addends the same way)
    const bool x_i8 = x_dt == HERO_I8 || x_dt == HERO_F8E4M3;
    if (!x_i8 && x_dt != HERO_BF16 && x_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (x_i8 && !x_row_scale) return HERO_ERR_NULL;
    int in_fp8 = x_dt == HERO_F8E4M3;
    if (r) {
        const bool r_8 = r_dt == HERO_I8 || r_dt == HERO_F8E4M3;
        if (!r_8 && r_dt != HERO_BF16 && r_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
        if (r_8 && !r_col_scale) return HERO_ERR_NULL;
        if (r_8 && x_i8 && r_dt != x_dt) return HERO_ERR_UNSUPPORTED;
        if (r_dt == HERO_F8E4M3) { in_fp8 = 1; r_dt = HERO_I8; }
    }
    if (!gamma && beta) return HERO_ERR_NULL;
    if (y_hp && y_hp_dt != HERO_BF16 && y_hp_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (D > (x_i8 ? 8192 : 4096)) return HERO_ERR_UNSUPPORTED;      // row must fit the register file
    if (!hero_aligned16(x) || !hero_aligned16(r) || !hero_aligned16(y_q) || !hero_aligned16(y_hp))
        return HERO_ERR_ALIGN;
    LnArgs a;
    a.x = x; a.x_row_scale = x_row_scale; a.r = r; a.r_col_scale = r_col_scale;
    a.gamma = gamma; a.beta = beta; a.eps = eps; a.M = M; a.D = (int)D;
    a.y_q = (int8_t*)y_q; a.y_scale = y_scale; a.y_hp = y_hp;
    a.x_dt = x_i8 ? (int)HERO_I8 : (int)x_dt; a.r_dt = r ? (int)r_dt : -1; a.hp_dt = y_hp ? (int)y_hp_dt : -1;
    a.y_fp8 = y_fp8; a.in_fp8 = in_fp8;
    a.x_idx = a.r_idx = a.r2_idx = nullptr; a.r2 = nullptr; a.x_rows = a.r_rows = a.r2_rows = 0;
    hipStream_t st = (hipStream_t)stream;
    if (x_i8) return launch<HERO_I8>(a, st);
    return x_dt == HERO_BF16 ? launch<HERO_BF16>(a, st) : launch<HERO_F16>(a, st);
}

}  // namespace

extern "C" hero_status hero_ln_quant(const void* x, hero_dtype x_dt, const float* x_row_scale,
                                     const void* r, hero_dtype r_dt, const float* r_col_scale,
                                     const float* gamma, const float* beta, float eps,
                                     int64_t M, int64_t D,
                                     int8_t* y_q, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream) {
    return ln_quant_entry(x, x_dt, x_row_scale, r, r_dt, r_col_scale, gamma, beta, eps, M, D, y_q, 0, y_scale, y_hp, y_hp_dt, stream);
}

extern "C" hero_status hero_ln_quant_fp8(const void* x, hero_dtype x_dt, const float* x_row_scale,
                                         const void* r, hero_dtype r_dt, const float* r_col_scale,
                                         const float* gamma, const float* beta, float eps,
                                         int64_t M, int64_t D,
                                         void* y_q, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream) {
    return ln_quant_entry(x, x_dt, x_row_scale, r, r_dt, r_col_scale, gamma, beta, eps, M, D, y_q, 1, y_scale, y_hp, y_hp_dt, stream);
}

extern "C" hero_status hero_embed_ln_quant(const int32_t* tok_ids, const int32_t* pos_ids, const int32_t* type_ids,
                                           const int8_t* tok_table, const float* tok_scale, int64_t V,
                                           const void* pos_table, int64_t P,
                                           const void* type_table, int64_t NT, hero_dtype pt_dt,
                                           const float* gamma, const float* beta, float eps,
                                           int64_t T, int64_t D, int8_t* y_q, float* y_scale, void* stream) {
    if (T < 0 || D <= 0 || V <= 0 || P <= 0 || V > 0x7fffffffLL || P > 0x7fffffffLL) return HERO_ERR_SHAPE;
    if (type_table && (NT <= 0 || NT > 0x7fffffffLL)) return HERO_ERR_SHAPE;
    if (D % 16 != 0 || D > 8192) return HERO_ERR_UNSUPPORTED;
    if (pt_dt != HERO_BF16 && pt_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (T == 0) return HERO_OK;
    if (!tok_ids || !pos_ids || !tok_table || !tok_scale || !pos_table || !gamma || !y_q || !y_scale) return HERO_ERR_NULL;
    if (type_table && !type_ids) return HERO_ERR_NULL;
    if (!hero_aligned16(tok_table) || !hero_aligned16(pos_table) || !hero_aligned16(type_table) || !hero_aligned16(y_q))
        return HERO_ERR_ALIGN;
    LnArgs a;
    a.x = tok_table; a.x_row_scale = tok_scale; a.r = pos_table; a.r_col_scale = nullptr;
    a.gamma = gamma; a.beta = beta; a.eps = eps; a.M = T; a.D = (int)D;
    a.y_q = y_q; a.y_scale = y_scale; a.y_hp = nullptr; a.y_fp8 = 0; a.in_fp8 = 0;
    a.x_dt = HERO_I8; a.r_dt = (int)pt_dt; a.hp_dt = -1;
    a.x_idx = tok_ids; a.r_idx = pos_ids; a.r2 = type_table; a.r2_idx = type_table ? type_ids : nullptr;
    a.x_rows = (int)V; a.r_rows = (int)P; a.r2_rows = type_table ? (int)NT : 0;
    hipStream_t st = (hipStream_t)stream;
    return pt_dt == HERO_BF16 ? launch_gather<HERO_BF16>(a, st) : launch_gather<HERO_F16>(a, st);
}
