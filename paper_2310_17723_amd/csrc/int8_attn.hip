// hero_int8_attn: INT8 attention, QK^T -> Softmax^quant -> PV (paper Sec. 2.2.2, quantized
// attention flow: A = d~ X_q,int8 X_k,int8^T is NOT quantized, S_p P_int8 = Softmax^quant(A)
// with unsigned codes, X_attn,int8 S_attn = S_p S_v P_int8 X_v,int8).
//
// The softmax is normalised before it is quantized, so the row maximum and the row sum
// must be known before the first code is produced: the kernel streams the keys twice
// (pass 1: QK^T, row max / row sum; pass 2: QK^T again, codes, PV).  A and P never leave
// the chip.
//
// Layout.  A block owns 128 queries of one (batch, head); each of its 4 waves owns 32 of them.
// Scores are computed TRANSPOSED, S^T = K Q^T (v_mfma_i32_32x32x32_i8 with the key
// fragment as first operand), so lane l holds query l % 32 and the keys 8g + 4(l/32) + t
// of a 32-key step in accumulator register 4g + t: a query's row statistics need one
// exchange between lanes l and l^32, and the 16 codes a lane produces are already the
// second-operand fragment of the PV MFMA (O^T = V^T P^T) provided V^T is stored in LDS with
// the same key order, which the V staging does.
// The matrix cores multiply signed bytes; codes are 0..255, so P-128 is fed and
// 128 * colsum(V) is added back, exact in int32.  Masked keys carry code 0 (fed as -128), so
// the column sums run over every staged key and are the same for all queries of the block:
// the four waves take turns adding them up from the V fragments they already hold (v_dot4
// against ones) and exchange them through LDS once, at the end.
// The kernel is bound by the plain-ALU work per score (exp2, conversion, rounding), not by
// the matrix cores, so both passes are written to spend as few vector instructions per score
// as possible (see the comment in front of pass 1).
#include "hero_common.h"
#include <atomic>
#include <type_traits>

namespace {

constexpr int BQ = 128;   // queries per block
constexpr int BKV = 64;   // keys per LDS tile

struct AttnArgs {
    const int8_t* q; const int8_t* k; const int8_t* v;
    int64_t qs[4], ks[4], vs[4];
    int B, H, Sq, Skv;
    float qk_scale, p_scale;
    const float* qk_scale_h;          // per-head d~ (online variant) or NULL
    int use_buf;                      // K / V of one (batch, head) span < 2 GB with non-negative strides
    const float* out_col_scale; int scale_is_scalar;
    int mask; const int32_t* kv_len;
    void* out; int64_t ldo;
};

// FMT = HERO_F8E4M3: the same flow with E4M3 codes (Sec. 2.1): q, k, v are E4M3 bytes, the scores and the PV sums
// are fp32 accumulators of v_mfma_f32_32x32x64_f8f6f4, the probabilities are quantized to non-negative E4M3 codes
// (saturating at 448 = p / S_p for p = 1 with S_p = 1/448), signed operands need no offset and no column sums.
// Staging, masks, tile order and the two-pass structure are those of the INT8 kernel.
template <int DH, int ODT, bool ONLINE = false, int FMT = HERO_I8>
__global__ __launch_bounds__(256, ONLINE ? (DH == 64 ? 3 : 2) : (DH == 64 ? 4 : 3)) void int8_attn_kernel(AttnArgs a) {
    constexpr bool F8 = FMT == HERO_F8E4M3;
    static_assert(!(F8 && ONLINE), "the online variant is INT8 only");
    using SACC = typename std::conditional<F8, v16f, v16i>::type;     // score / output accumulators
    constexpr int KLD = DH + 16;        // sK row stride (bytes)
    constexpr int VLD = BKV + 16;       // sVt row stride (bytes)
    constexpr int DS = DH / 32;         // 32-wide steps over the head dimension
    __shared__ __attribute__((aligned(16))) int8_t sK[2][BKV * KLD];
    __shared__ __attribute__((aligned(16))) int8_t sVt[2][DH * VLD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5, ql = lane & 31;
    // Workgroups go round-robin to the 8 XCDs; all query blocks of one (batch, head) are sent to
    // the SAME XCD, back to back, so its K / V stream hits that XCD's L2 after the first block, and
    // so are the HG = 128 / DH neighbouring heads whose K / V rows share 128-byte cache lines with it
    // in the packed [token][head][channel] layout (otherwise each XCD would fetch whole lines to use
    // a fraction of them).
    constexpr int HG = DH >= 128 ? 1 : 128 / DH;
    const int nqb = (a.Sq + BQ - 1) / BQ;
    const int slot = blockIdx.x / 8, grp = (slot / (HG * nqb)) * 8 + (blockIdx.x % 8), within = slot % (HG * nqb);
    const int bh = grp * HG + within / nqb;
    if (bh >= a.B * a.H) return;
    // The query blocks of a (batch, head) differ in length (causal: block j sees j + 1 blocks of keys; padding: the
    // blocks past the sequence's end leave at once), and the hardware places workgroups on the compute units in
    // launch order, round and round: with the same order inside every group a compute unit is handed the same kind
    // of block every time, the long ones always go to the same few, and the launch waits for those.  The order
    // inside a group therefore rotates with a hash of the group's number.
    const uint32_t rot = ((uint32_t)(slot / (HG * nqb)) * 2654435761u) >> 20;
    const int qb = (int)((within % nqb + rot) % (uint32_t)nqb);
    const int b = bh / a.H, h = bh % a.H, q0 = qb * BQ;
    const int len = a.kv_len ? min(max(a.kv_len[b], 0), a.Skv) : a.Skv;
    const int shift = len - a.Sq;                       // causal: key k visible iff k <= i + shift
    // Which 32 queries of the block a wave owns rotates with the block: with the padding mask the last sub-blocks
    // of a sequence's last block are idle, and the busy waves of co-resident blocks should not share a SIMD.
    const int wq = (wave + slot) & 3;
    const int qi = q0 + wq * 32 + ql;                   // this lane's query
    int nvis = len;
    if (a.mask == HERO_MASK_CAUSAL) nvis = min(len, qi + shift + 1);
    nvis = max(nvis, 0);
    // keys any query of the block can see -> number of key tiles
    int kmax = len;
    if (a.mask == HERO_MASK_CAUSAL) kmax = min(len, min(q0 + BQ, a.Sq) + shift);
    const int ntiles = (max(kmax, 0) + BKV - 1) / BKV;
    // PADDING mask in self-attention: the positions >= len are padding as queries too and their output rows are
    // zeros.  A block with no real query writes them and leaves; a wave with no real query keeps staging K / V
    // and meeting the barriers (and adds its share of the column sums) but computes no score.
    const int qlim = (a.mask == HERO_MASK_PADDING && a.Sq == a.Skv) ? len : a.Sq;
    if (q0 >= qlim) {
        constexpr int U = DH / 4;                              // stores of 4 elements, as the output stage below
        const int rows = min(BQ, a.Sq - q0);
        for (int idx = tid; idx < rows * U; idx += 256) {
            const int64_t e = ((int64_t)b * a.Sq + q0 + idx / U) * a.ldo + (int64_t)h * DH + (idx % U) * 4;
            if (ODT == HERO_I8 || ODT == HERO_F8E4M3) *reinterpret_cast<uint32_t*>((int8_t*)a.out + e) = 0u;
            else { v2i z = {0, 0}; *reinterpret_cast<v2i*>((uint16_t*)a.out + e) = z; }
        }
        return;
    }
    const bool wact = __builtin_amdgcn_readfirstlane(q0 + wq * 32) < qlim;     // wave-uniform

    // ---- Q fragments (second MFMA operand), kept in registers -----------------------------
    v4i qf[DS];
    {
        const int8_t* qp = a.q + (int64_t)b * a.qs[0] + (int64_t)min(qi, a.Sq - 1) * a.qs[1] + (int64_t)h * a.qs[2];
#pragma unroll
        for (int d = 0; d < DS; ++d) qf[d] = *reinterpret_cast<const v4i*>(qp + d * 32 + hh * 16);
        // The fragments pass through an empty asm statement so that they count as arrived from here on:
        // otherwise the first MFMA of every tile waits for ALL outstanding global loads (vmcnt(0)),
        // the just-issued prefetch of the next tile included.
#pragma unroll
        for (int d = 0; d < DS; ++d) asm volatile("" : "+v"(qf[d]));
    }
    const int8_t* kbase = a.k + (int64_t)b * a.ks[0] + (int64_t)h * a.ks[2];
    const int8_t* vbase = a.v + (int64_t)b * a.vs[0] + (int64_t)h * a.vs[2];

    // K / V tiles: global -> registers (next tile, in flight during the current tile's math) -> LDS
    // (double buffered, one barrier per tile).  V is written transposed, keys permuted so that the
    // PV operand fragment is one 128-bit read: key row 32kb + 8g + 4h + t -> position 32kb + 16h + 4g + t.
    constexpr int UNITS = BKV * (DH / 16) / 256;
    constexpr int VUNITS = (BKV / 4) * (DH / 4) / 256;     // V: units of 4 keys x 4 channels (one dword per key)
    v4i rk[UNITS];
    int rv[VUNITS][4];
    // K / V tiles that lie wholly inside the key range are fetched through buffer descriptors when the
    // host found that a (batch, head) operand spans less than 2 GB: the address is a wave-uniform base
    // plus a 32-bit lane offset (one add per load and tile instead of a 64-bit multiply per load).  A
    // ragged last tile, and operands beyond 2 GB, take clamped 64-bit addresses.
    __amdgpu_buffer_rsrc_t krs, vrs;
    uint32_t koff[UNITS], voff[VUNITS];
    if (a.use_buf) {
        krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(kbase), 0, (int)((int64_t)(a.Skv - 1) * a.ks[1] + DH), 0x00020000);
        vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vbase), 0, (int)((int64_t)(a.Skv - 1) * a.vs[1] + DH), 0x00020000);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int idx = tid + u * 256, row = idx / (DH / 16), ch = idx % (DH / 16);
            koff[u] = (uint32_t)row * (uint32_t)a.ks[1] + ch * 16;
        }
#pragma unroll
        for (int u = 0; u < VUNITS; ++u) {
            const int idx = tid + u * 256, kg = (idx >> 2) % (BKV / 4), cg = (idx & 3) + 4 * (idx / BKV);
            voff[u] = (uint32_t)(kg * 4) * (uint32_t)a.vs[1] + cg * 4;
        }
    }
    auto load_k = [&](int tile) {
        if (a.use_buf && (tile + 1) * BKV <= a.Skv) {
            const uint32_t tb = (uint32_t)tile * (uint32_t)(BKV * (uint32_t)a.ks[1]);
#pragma unroll
            for (int u = 0; u < UNITS; ++u)
                rk[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(krs, koff[u] + tb, 0, 0));
            return;
        }
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            int idx = tid + u * 256, row = idx / (DH / 16), ch = idx % (DH / 16);
            int key = min(tile * BKV + row, a.Skv - 1);
            rk[u] = *reinterpret_cast<const v4i*>(kbase + (int64_t)key * a.ks[1] + ch * 16);
        }
    };
    // V unit: key group kg (4 consecutive keys) x channel group cg (4 channels).  Four consecutive lanes
    // read 16 contiguous bytes of one key row; the 64 transposed dword stores of a wave (rows 4cg + j,
    // 16 key-group positions each) fall into 64 different banks.
    auto load_v = [&](int tile) {
        if (a.use_buf && (tile + 1) * BKV <= a.Skv) {
            const uint32_t tb = (uint32_t)tile * (uint32_t)(BKV * (uint32_t)a.vs[1]);
#pragma unroll
            for (int u = 0; u < VUNITS; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    rv[u][i] = (int)__builtin_amdgcn_raw_buffer_load_b32(vrs, voff[u] + tb + (uint32_t)i * (uint32_t)a.vs[1], 0, 0);
            return;
        }
#pragma unroll
        for (int u = 0; u < VUNITS; ++u) {
            const int idx = tid + u * 256, kg = (idx >> 2) % (BKV / 4), cg = (idx & 3) + 4 * (idx / BKV);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int key = min(tile * BKV + kg * 4 + i, a.Skv - 1);
                rv[u][i] = *reinterpret_cast<const int*>(vbase + (int64_t)key * a.vs[1] + cg * 4);
            }
        }
    };
    auto store_k = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            int idx = tid + u * 256, row = idx / (DH / 16), ch = idx % (DH / 16);
            *reinterpret_cast<v4i*>(&sK[buf][row * KLD + ch * 16]) = rk[u];
        }
    };
    auto store_v = [&](int buf) {
#pragma unroll
        for (int u = 0; u < VUNITS; ++u) {
            const int idx = tid + u * 256, kg = (idx >> 2) % (BKV / 4), cg = (idx & 3) + 4 * (idx / BKV);
            // 4 x 4 byte transpose in registers: dword j of the result = channel 4cg + j of keys 4kg .. 4kg + 3
            const uint32_t d0 = rv[u][0], d1 = rv[u][1], d2 = rv[u][2], d3 = rv[u][3];
            const uint32_t lo01 = __builtin_amdgcn_perm(d1, d0, 0x05010400u), hi01 = __builtin_amdgcn_perm(d1, d0, 0x07030602u);
            const uint32_t lo23 = __builtin_amdgcn_perm(d3, d2, 0x05010400u), hi23 = __builtin_amdgcn_perm(d3, d2, 0x07030602u);
            const uint32_t t[4] = {__builtin_amdgcn_perm(lo23, lo01, 0x05040100u), __builtin_amdgcn_perm(lo23, lo01, 0x07060302u),
                                   __builtin_amdgcn_perm(hi23, hi01, 0x05040100u), __builtin_amdgcn_perm(hi23, hi01, 0x07060302u)};
            // keys 4kg .. 4kg+3 sit at positions pos .. pos+3 of the permuted key order (see above)
            const int pos = ((kg * 4) & 32) + (kg & 1) * 16 + ((kg & 7) >> 1) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<uint32_t*>(&sVt[buf][(cg * 4 + j) * VLD + pos]) = t[j];
        }
    };
    // S^T for the 32-key step s of the staged tile
    auto scores = [&](int buf, int s) {
        SACC acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0;
        if constexpr (F8) {
#pragma unroll
            for (int d = 0; d < DS; d += 2) {
                const v4i k0 = *reinterpret_cast<const v4i*>(&sK[buf][(s * 32 + ql) * KLD + d * 32 + hh * 16]);
                const v4i k1 = *reinterpret_cast<const v4i*>(&sK[buf][(s * 32 + ql) * KLD + (d + 1) * 32 + hh * 16]);
                acc = mfma_wide_f8(k0, k1, qf[d], qf[d + 1], acc);
            }
        } else {
#pragma unroll
            for (int d = 0; d < DS; ++d) {
                v4i kf = *reinterpret_cast<const v4i*>(&sK[buf][(s * 32 + ql) * KLD + d * 32 + hh * 16]);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[d], acc, 0, 0, 0);
            }
        }
        return acc;
    };

    // Both passes work in the log2 domain on the raw integer scores: p = 2^(acc * c2 - m2) with
    // c2 = d~ * log2(e).  The row maximum is taken on the integers (the scale is positive), masked
    // keys are replaced by a very negative integer (only in tiles that contain one), and in pass 2
    // the normaliser and 1/S_p are folded into the exponent, so a code costs one int->float
    // conversion, one fma, one exp2 and one saturating round-to-u8.
    const float c2 = (a.qk_scale_h ? a.qk_scale_h[h] : a.qk_scale) * 1.44269504088896340736f;
    constexpr int MASKED = -0x40000000;
    // first tile in which some key is hidden from some query of this wave (wave-uniform)
    int nvis_min = nvis;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nvis_min = min(nvis_min, __shfl_xor(nvis_min, o));

    // ---- the online variant: ONE sweep.  The codes of a 64-key tile are taken against the running row
    // maximum m (so the largest weight seen so far has code 255) and stay un-normalised; the integer sums
    // of a run of tiles with an unchanged maximum are kept in int32 (oi, li); only when some query of the
    // wave raises its maximum are they folded into the fp32 accumulators (of, lf) and everything gathered
    // so far is rescaled by 2^(m_old - m_new); the division by the sum of the weights happens once, at the end.  The matrix cores take
    // signed bytes: the fragment holds 127 - code (one XOR) and a second MFMA against the constant -127
    // removes the offset, so oi = -sum_k code_k v_k exactly, with no column sums and no extra vector work.
    if constexpr (ONLINE) {
        constexpr float L255 = 7.99435343685885793770f;           // log2(255)
        v16i oi[DS];
        v16f of[DS];
        uint32_t li = 0;
        float lf = 0.0f, m2 = -INFINITY;
#pragma unroll
        for (int c = 0; c < DS; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { oi[c][r] = 0; of[c][r] = 0.0f; }
        const v4i cm127 = {(int)0x81818181u, (int)0x81818181u, (int)0x81818181u, (int)0x81818181u};
        if (ntiles > 0) { load_k(0); load_v(0); store_k(0); store_v(0); }
        __syncthreads();
        for (int tile = 0; tile < ntiles; ++tile) {
            const int buf = tile & 1;
            if (tile + 1 < ntiles) { load_k(tile + 1); load_v(tile + 1); }
            const bool edge = (tile + 1) * BKV > nvis_min;
            auto online_tile = [&](auto EDGE) {
                // the tile's maximum first; the scores are computed again for the codes (a second QK^T on
                // the idle matrix cores costs less than keeping 32 more registers alive)
                int imax = MASKED;
                auto tile_scores = [&](int s) {
                    v16i acc = scores(buf, s);
                    if constexpr (decltype(EDGE)::value) {
                        const int lim = nvis - (tile * BKV + s * 32 + hh * 4);  // key visible iff 8g + t < lim
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[r] = ((r >> 2) * 8 + (r & 3)) < lim ? acc[r] : MASKED;
                    }
                    return acc;
                };
#pragma unroll
                for (int s = 0; s < BKV / 32; ++s) {
                    const v16i acc = tile_scores(s);
#pragma unroll
                    for (int r = 0; r < 16; ++r) imax = max(imax, acc[r]);
                }
                imax = max(imax, __shfl_xor(imax, 32));
                const float mn = imax > MASKED ? fmaxf(m2, (float)imax * c2) : m2;
                if (__builtin_amdgcn_ballot_w64(mn != m2) != 0) {                // wave-uniform
                    const float alpha = mn == m2 ? 1.0f : __builtin_amdgcn_exp2f(m2 - mn);
#pragma unroll
                    for (int c = 0; c < DS; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) { of[c][r] = (of[c][r] + (float)oi[c][r]) * alpha; oi[c][r] = 0; }
                    lf = (lf + (float)li) * alpha;
                    li = 0;
                    m2 = mn;
                }
                {
                    const float off = L255 - m2;
#pragma unroll
                    for (int s = 0; s < BKV / 32; ++s) {
                        const v16i acc = scores(buf, s);
                        const int lim = nvis - (tile * BKV + s * 32 + hh * 4);
                        v4i pf;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            uint32_t w = 0;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                float e = __builtin_amdgcn_exp2f(fmaf((float)acc[4 * g + t], c2, off));
                                if constexpr (decltype(EDGE)::value) e = (g * 8 + t) < lim ? e : 0.0f;
                                w = __builtin_amdgcn_cvt_pk_u8_f32(e, t, w);
                            }
                            li = __builtin_amdgcn_sad_u8(w, 0u, li);             // + the four codes
                            pf[g] = (int)(w ^ 0x7f7f7f7fu);                      // 127 - code as signed bytes
                        }
#pragma unroll
                        for (int c = 0; c < DS; ++c) {
                            v4i vf = *reinterpret_cast<const v4i*>(&sVt[buf][(c * 32 + ql) * VLD + s * 32 + hh * 16]);
                            oi[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, oi[c], 0, 0, 0);
                            oi[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, cm127, oi[c], 0, 0, 0);
                        }
                    }
                }
            };
            if (!wact) {} else if (edge) online_tile(std::true_type{}); else online_tile(std::false_type{});
            if (tile + 1 < ntiles) { store_k(buf ^ 1); store_v(buf ^ 1); }
            __syncthreads();
        }
        if (qi >= a.Sq) return;
        float l = lf + (float)li;
        l += __shfl_xor(l, 32);
        // oi / of hold MINUS the weighted sums; y = O / L * c[j] / S_p
        const float inv = l > 0.0f ? __fdiv_rn(-1.0f, l * a.p_scale) : 0.0f;
        const int64_t orow = ((int64_t)b * a.Sq + qi) * a.ldo + (int64_t)h * DH;
#pragma unroll
        for (int c = 0; c < DS; ++c)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e0 = c * 32 + g * 8 + hh * 4;
                float y[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float sc = a.scale_is_scalar ? a.out_col_scale[0] : a.out_col_scale[h * DH + e0 + t];
                    y[t] = (of[c][4 * g + t] + (float)oi[c][4 * g + t]) * inv * sc;
                    if (qi >= qlim) y[t] = 0.0f;              // padded query: zeros
                }
                if (ODT == HERO_I8) {
                    *reinterpret_cast<uint32_t*>((int8_t*)a.out + orow + e0) = quant4_sat(y[0], y[1], y[2], y[3]);
                } else {
                    v2i w = {(int)pack2_hp<ODT>(y[0], y[1]), (int)pack2_hp<ODT>(y[2], y[3])};
                    *reinterpret_cast<v2i*>((uint16_t*)a.out + orow + e0) = w;
                }
            }
        return;
    }

    // ---- pass 1: row max and row sum ------------------------------------------------------------
    float m2 = -INFINITY, l = 0.0f;           // running max (log2 domain) and sum of 2^(a2 - m2), this lane's keys
    constexpr float FMASKED = -3.0e38f;       // E4M3 scores are floats: the mask value of that variant
    if (ntiles > 0) { load_k(0); store_k(0); }
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntiles) load_k(tile + 1);
        const bool edge = (tile + 1) * BKV > nvis_min;
        auto pass1_tile = [&](auto EDGE) {
#pragma unroll
            for (int s = 0; s < BKV / 32; ++s) {
                SACC acc = scores(buf, s);
                if constexpr (decltype(EDGE)::value) {
                    const int lim = nvis - (tile * BKV + s * 32 + hh * 4);      // key visible iff 8g + t < lim
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if constexpr (F8) acc[r] = ((r >> 2) * 8 + (r & 3)) < lim ? acc[r] : FMASKED;
                        else acc[r] = ((r >> 2) * 8 + (r & 3)) < lim ? acc[r] : MASKED;
                    }
                }
                auto smax = acc[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) smax = max(smax, acc[r]);
                smax = max(smax, __shfl_xor(smax, 32));
                if (F8 ? (float)smax > FMASKED : (int)smax > MASKED) {          // same decision in both lanes of a query
                    const float mn = fmaxf(m2, (float)smax * c2);
                    float sum = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf((float)acc[r], c2, -mn));
                    l = fmaf(l, __builtin_amdgcn_exp2f(m2 - mn), sum);
                    m2 = mn;
                }
            }
        };
        if (!wact) {} else if (edge) pass1_tile(std::true_type{}); else pass1_tile(std::false_type{});
        if (tile + 1 < ntiles) store_k(buf ^ 1);
        __syncthreads();
    }
    l += __shfl_xor(l, 32);
    // exponent offset of pass 2: 2^(acc*c2 - m2) / l / S_p = 2^(acc*c2 + off); a row that saw no key gets codes 0
    const float off = l > 0.0f ? -m2 - __log2f(l * a.p_scale) : -INFINITY;

    // ---- pass 2: codes and PV --------------------------------------------------------------------
    SACC o[DS];
    int csum[DS];                                         // this wave's share of colsum(V): channel 32c + ql, keys of half hh
#pragma unroll
    for (int c = 0; c < DS; ++c) {
        csum[c] = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) o[c][r] = 0;
    }
    if (ntiles > 0) { load_k(0); load_v(0); store_k(0); store_v(0); }
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntiles) { load_k(tile + 1); load_v(tile + 1); }
        const bool edge = (tile + 1) * BKV > nvis_min;
        auto pass2_tile = [&](auto EDGE) {
            if constexpr (F8) {
                // codes of the whole 64-key tile first (two 32-key steps), then ONE K = 64 matrix instruction per
                // 32 channels: e4m3(min(2^(acc*c2 + off), 448)), two codes per conversion instruction
                v4i pf[BKV / 32];
#pragma unroll
                for (int s = 0; s < BKV / 32; ++s) {
                    const v16f acc = scores(buf, s);
                    const int lim = nvis - (tile * BKV + s * 32 + hh * 4);
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float e[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            e[t] = fminf(__builtin_amdgcn_exp2f(fmaf(acc[4 * g + t], c2, off)), 448.0f);
                            if constexpr (decltype(EDGE)::value) e[t] = (g * 8 + t) < lim ? e[t] : 0.0f;
                        }
                        int w = __builtin_amdgcn_cvt_pk_fp8_f32(e[0], e[1], 0, false);
                        pf[s][g] = __builtin_amdgcn_cvt_pk_fp8_f32(e[2], e[3], w, true);
                    }
                }
#pragma unroll
                for (int c = 0; c < DS; ++c) {
                    const v4i v0 = *reinterpret_cast<const v4i*>(&sVt[buf][(c * 32 + ql) * VLD + hh * 16]);
                    const v4i v1 = *reinterpret_cast<const v4i*>(&sVt[buf][(c * 32 + ql) * VLD + 32 + hh * 16]);
                    o[c] = mfma_wide_f8(v0, v1, pf[0], pf[1], o[c]);
                }
            } else {
#pragma unroll
            for (int s = 0; s < BKV / 32; ++s) {
                v16i acc = scores(buf, s);
                const int lim = nvis - (tile * BKV + s * 32 + hh * 4);          // key visible iff 8g + t < lim
                v4i pf;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t w = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float e = __builtin_amdgcn_exp2f(fmaf((float)acc[4 * g + t], c2, off));
                        if constexpr (decltype(EDGE)::value) e = (g * 8 + t) < lim ? e : 0.0f;
                        w = __builtin_amdgcn_cvt_pk_u8_f32(e, t, w);     // sat_[0,255](rne(.)) into byte t
                    }
                    pf[g] = (int)(w ^ 0x80808080u);                         // codes - 128 as signed bytes
                }
#pragma unroll
                for (int c = 0; c < DS; ++c) {
                    v4i vf = *reinterpret_cast<const v4i*>(&sVt[buf][(c * 32 + ql) * VLD + s * 32 + hh * 16]);
                    o[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[c], 0, 0, 0);
                    if (((tile * (BKV / 32) + s) & 3) == wave) {         // wave-uniform: one wave per 32-key step
#pragma unroll
                        for (int w = 0; w < 4; ++w) csum[c] = __builtin_amdgcn_sdot4(vf[w], 0x01010101, csum[c], false);
                    }
                }
            }
            }
        };
        if (!wact) {
            if constexpr (!F8) {                              // only the wave's share of the column sums
#pragma unroll
                for (int s = 0; s < BKV / 32; ++s)
                    if (((tile * (BKV / 32) + s) & 3) == wave) {
#pragma unroll
                        for (int c = 0; c < DS; ++c) {
                            const v4i vf = *reinterpret_cast<const v4i*>(&sVt[buf][(c * 32 + ql) * VLD + s * 32 + hh * 16]);
#pragma unroll
                            for (int w = 0; w < 4; ++w) csum[c] = __builtin_amdgcn_sdot4(vf[w], 0x01010101, csum[c], false);
                        }
                    }
            }
        } else if (edge) pass2_tile(std::true_type{}); else pass2_tile(std::false_type{});
        if (tile + 1 < ntiles) { store_k(buf ^ 1); store_v(buf ^ 1); }
        __syncthreads();
    }

    // ---- colsum(V) of the block: every wave adds its share per channel (the loop's last barrier has
    // released the K buffers, which now hold the sums)
    int* const colsum = reinterpret_cast<int*>(&sK[0][0]);
    if constexpr (!F8) {
        for (int c = tid; c < DH; c += 256) colsum[c] = 0;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < DS; ++c) atomicAdd(&colsum[c * 32 + ql], csum[c]);
        __syncthreads();
    }

    // ---- output: lane holds query ql, channels 32c + 8g + 4hh + t -----------------------------------
    if (qi >= a.Sq) return;
    const int64_t orow = ((int64_t)b * a.Sq + qi) * a.ldo + (int64_t)h * DH;
#pragma unroll
    for (int c = 0; c < DS; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int e0 = c * 32 + g * 8 + hh * 4;
            float y[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float sc = a.scale_is_scalar ? a.out_col_scale[0] : a.out_col_scale[h * DH + e0 + t];
                if constexpr (F8) y[t] = o[c][4 * g + t] * sc;
                else y[t] = (float)(o[c][4 * g + t] + 128 * colsum[e0 + t]) * sc;
                if (qi >= qlim) y[t] = 0.0f;                  // padded query: zeros
            }
            if (ODT == HERO_I8) {
                *reinterpret_cast<uint32_t*>((int8_t*)a.out + orow + e0) = quant4_sat(y[0], y[1], y[2], y[3]);
            } else if (ODT == HERO_F8E4M3) {
                *reinterpret_cast<uint32_t*>((int8_t*)a.out + orow + e0) = fp8x4_sat(y[0], y[1], y[2], y[3]);
            } else {
                v2i w = {(int)pack2_hp<ODT>(y[0], y[1]), (int)pack2_hp<ODT>(y[2], y[3])};
                *reinterpret_cast<v2i*>((uint16_t*)a.out + orow + e0) = w;
            }
        }
}

// ------------------------------------------------------------------------------------------
// Decode (one query per sequence): HBM-bound on the K and V cache, so no matrix cores; K and
// V are each read exactly once.  One block per (batch, head); 8 lanes share a key (16 bytes of
// the row each, so a wave-level load covers 8 whole rows = 1 KB of consecutive cache).
//   phase 1: integer scores q.k (v_dot4) for every key -> LDS
//   phase 2: row max / sum in the log2 domain (block reduction), codes 0..255 -> LDS
//   phase 3: acc[e] = sum_k P[k] * v[k][e] in int32, reduced over the key groups through LDS
// ------------------------------------------------------------------------------------------
constexpr int DEC_MAX_KEYS = 16384;

// FMT = HERO_F8E4M3: E4M3 operands: the bytes are decoded two at a time (v_cvt_pk_f32_fp8), scores and PV sums are
// fp32, the probability code is e4m3(min(p / S_p, 448)) and its decoded value is what PV multiplies.
template <int DH, int ODT, int FMT = HERO_I8>
__global__ __launch_bounds__(256) void int8_attn_decode_kernel(AttnArgs a) {
    constexpr bool F8 = FMT == HERO_F8E4M3;
    using ST = typename std::conditional<F8, float, int>::type;      // score / accumulator element
    constexpr int LPK = DH / 16;                 // lanes per key
    constexpr int KPI = 256 / LPK;               // keys per block iteration
    extern __shared__ __attribute__((aligned(16))) int smem_dec[];
    ST* sc = reinterpret_cast<ST*>(smem_dec);                      // [len] scores, later codes (F8: their decoded values)
    __shared__ float red[8];
    __shared__ ST racc[KPI][DH + 4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y, h = blockIdx.x;
    const int len = a.kv_len ? min(max(a.kv_len[b], 0), a.Skv) : a.Skv;     // one query: it sees every valid key
    const int sub = tid % LPK, kg = tid / LPK;
    const int8_t* kbase = a.k + (int64_t)b * a.ks[0] + (int64_t)h * a.ks[2] + sub * 16;
    const int8_t* vbase = a.v + (int64_t)b * a.vs[0] + (int64_t)h * a.vs[2] + sub * 16;
    const v4i qv = *reinterpret_cast<const v4i*>(a.q + (int64_t)b * a.qs[0] + (int64_t)h * a.qs[2] + sub * 16);
    // 16 E4M3 bytes -> 16 floats
    auto decode16 = [](const v4i& w, float (&f)[16]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], true);
            f[4 * i] = lo[0]; f[4 * i + 1] = lo[1]; f[4 * i + 2] = hi[0]; f[4 * i + 3] = hi[1];
        }
    };
    float qf[16];
    if constexpr (F8) decode16(qv, qf);

    // ---- phase 1: scores ---------------------------------------------------------------------
    constexpr float FMASKED = -3.0e38f;
    ST lmax = F8 ? (ST)FMASKED : (ST)-0x40000000;
    auto score = [&](const v4i& kv) {
        ST d = 0;
        if constexpr (F8) {
            float kf[16];
            decode16(kv, kf);
#pragma unroll
            for (int e = 0; e < 16; ++e) d = fmaf(kf[e], qf[e], d);
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) d = __builtin_amdgcn_sdot4(kv[w], qv[w], d, false);
        }
#pragma unroll
        for (int o = 1; o < LPK; o <<= 1) d += __shfl_xor(d, o);
        return d;
    };
    // the stream is bound by the bytes in flight: UNR unconditional loads per lane are issued before the first is
    // used (whole groups of UNR * KPI keys), the ragged rest goes one guarded load at a time
    constexpr int UNR = 8;
    int k0 = 0;
    for (; k0 + UNR * KPI <= len; k0 += UNR * KPI) {
        v4i kv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) kv[u] = *reinterpret_cast<const v4i*>(kbase + (int64_t)(k0 + u * KPI + kg) * a.ks[1]);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const ST d = score(kv[u]);
            if (sub == 0) { sc[k0 + u * KPI + kg] = d; lmax = max(lmax, d); }
        }
    }
    for (; k0 < len; k0 += KPI) {
        const int key = k0 + kg;
        v4i kv = {0, 0, 0, 0};
        if (key < len) kv = *reinterpret_cast<const v4i*>(kbase + (int64_t)key * a.ks[1]);
        const ST d = score(kv);
        if (sub == 0 && key < len) { sc[key] = d; lmax = max(lmax, d); }
    }
    // block max
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lmax = max(lmax, __shfl_xor(lmax, o));
    if (lane == 0) red[wave] = F8 ? (float)lmax : __int_as_float((int)lmax);
    __syncthreads();
    const float c2 = a.qk_scale * 1.44269504088896340736f;
    float m2;
    if constexpr (F8) m2 = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * c2;
    else m2 = (float)max(max(__float_as_int(red[0]), __float_as_int(red[1])), max(__float_as_int(red[2]), __float_as_int(red[3]))) * c2;
    // ---- phase 2: sum, then codes --------------------------------------------------------------
    float lsum = 0.0f;
    for (int k = tid; k < len; k += 256) lsum += __builtin_amdgcn_exp2f(fmaf((float)sc[k], c2, -m2));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lsum += __shfl_xor(lsum, o);
    if (lane == 0) red[4 + wave] = lsum;
    __syncthreads();
    const float l = red[4] + red[5] + red[6] + red[7];
    const float off = l > 0.0f ? -m2 - __log2f(l * a.p_scale) : -INFINITY;
    for (int k = tid; k < len; k += 256) {
        const float e = __builtin_amdgcn_exp2f(fmaf((float)sc[k], c2, off));
        if constexpr (F8) sc[k] = __builtin_amdgcn_cvt_f32_fp8(__builtin_amdgcn_cvt_pk_fp8_f32(fminf(e, 448.0f), 0.0f, 0, false), 0);
        else sc[k] = (int)__builtin_amdgcn_cvt_pk_u8_f32(e, 0, 0u);
    }
    __syncthreads();
    // ---- phase 3: PV ------------------------------------------------------------------------------
    ST acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0;
    auto pv = [&](const v4i& vv, const ST p) {
        if constexpr (F8) {
            float vf[16];
            decode16(vv, vf);
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] += p * (int)(int8_t)(vv[e >> 2] >> (8 * (e & 3)));
        }
    };
    k0 = 0;
    for (; k0 + UNR * KPI <= len; k0 += UNR * KPI) {
        v4i vv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) vv[u] = *reinterpret_cast<const v4i*>(vbase + (int64_t)(k0 + u * KPI + kg) * a.vs[1]);
#pragma unroll
        for (int u = 0; u < UNR; ++u) pv(vv[u], sc[k0 + u * KPI + kg]);
    }
    for (; k0 < len; k0 += KPI) {
        const int key = k0 + kg;
        if (key < len) pv(*reinterpret_cast<const v4i*>(vbase + (int64_t)key * a.vs[1]), sc[key]);
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) racc[kg][sub * 16 + e] = acc[e];
    __syncthreads();
    if (tid < DH) {
        ST tot = 0;
        for (int g = 0; g < KPI; ++g) tot += racc[g][tid];
        const float scl = a.scale_is_scalar ? a.out_col_scale[0] : a.out_col_scale[h * DH + tid];
        const float y = (float)tot * scl;
        const int64_t oidx = (int64_t)b * a.ldo + (int64_t)h * DH + tid;
        if (ODT == HERO_I8) ((int8_t*)a.out)[oidx] = (int8_t)(rne_low_byte(__builtin_amdgcn_fmed3f(y, -127.0f, 127.0f)) & 0xff);
        else if (ODT == HERO_F8E4M3) ((uint8_t*)a.out)[oidx] = (uint8_t)(fp8x4_sat(y, 0.0f, 0.0f, 0.0f) & 0xffu);
        else ((uint16_t*)a.out)[oidx] = (uint16_t)f32_to_hp<ODT>(y);
    }
}

__global__ void zero_rows_kernel(int8_t* out, int64_t bytes) {
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 16;
    if (i < bytes) *reinterpret_cast<v4i*>(out + i) = v4i{0, 0, 0, 0};
}

// The decode kernel keeps one score per key in dynamic LDS; beyond 32 KB a kernel must be told once (per device) how
// much it may ask for.  The attribute is raised to the kernel's maximum the first time a launch needs more than the
// default, not on every call.
template <int DH, int ODT, int FMT>
bool decode_lds_ready(size_t lds) {
    static std::atomic<bool> raised[64];
    if (lds <= 32768) return true;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    if (raised[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute((const void*)int8_attn_decode_kernel<DH, ODT, FMT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            DEC_MAX_KEYS * (int)sizeof(int)) != hipSuccess) return false;
    raised[dev].store(true, std::memory_order_release);
    return true;
}

template <int DH, bool ONLINE = false, int FMT = HERO_I8>
hero_status launch(const AttnArgs& a, hero_dtype out_dt, hipStream_t st) {
    constexpr int HG = DH >= 128 ? 1 : 128 / DH;               // heads per workgroup group (see the kernel)
    const int64_t nqb = (a.Sq + BQ - 1) / BQ, hgroups = ((int64_t)a.B * a.H + HG - 1) / HG, rounds = (hgroups + 7) / 8;
    if (rounds * 8 * HG * nqb > 0x7fffffffLL) return HERO_ERR_SHAPE;
    dim3 grid((unsigned)(rounds * 8 * HG * nqb)), block(256);
    if (out_dt == HERO_BF16) hipLaunchKernelGGL((int8_attn_kernel<DH, HERO_BF16, ONLINE, FMT>), grid, block, 0, st, a);
    else if (out_dt == HERO_F16) hipLaunchKernelGGL((int8_attn_kernel<DH, HERO_F16, ONLINE, FMT>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((int8_attn_kernel<DH, FMT, ONLINE, FMT>), grid, block, 0, st, a);      // 8-bit output in the operands' format
    return hero_launch_status();
}

// argument checks and dispatch shared by the two entry points (online: the single-sweep variant)
hero_status attn_entry(const int8_t* q, const int64_t q_strides[4],
                       const int8_t* k, const int64_t k_strides[4],
                       const int8_t* v, const int64_t v_strides[4],
                       int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                       float qk_scale, const float* qk_scale_h, bool online, bool fp8,
                       float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                       hero_mask mask, const int32_t* kv_len,
                       void* out, hero_dtype out_dt, int64_t ldo, void* stream) {
    if (B < 0 || H < 0 || Sq < 0 || Skv < 0) return HERO_ERR_SHAPE;
    if (Dh != 64 && Dh != 128) return HERO_ERR_UNSUPPORTED;
    const hero_dtype dt8 = fp8 ? HERO_F8E4M3 : HERO_I8;                  // the 8-bit output format is the operands'
    if (out_dt != dt8 && out_dt != HERO_BF16 && out_dt != HERO_F16) return HERO_ERR_UNSUPPORTED;
    if (mask != HERO_MASK_NONE && mask != HERO_MASK_PADDING && mask != HERO_MASK_CAUSAL) return HERO_ERR_UNSUPPORTED;
    if (B == 0 || H == 0 || Sq == 0) return HERO_OK;
    if (!out || !out_col_scale || !q_strides || !k_strides || !v_strides) return HERO_ERR_NULL;
    if (Skv > 0 && (!q || !k || !v)) return HERO_ERR_NULL;
    if (mask == HERO_MASK_PADDING && !kv_len) return HERO_ERR_NULL;
    if (online && !qk_scale_h) return HERO_ERR_NULL;
    if (out_dt != dt8 && !out_scale_is_scalar) return HERO_ERR_UNSUPPORTED;
    if (!(p_scale > 0.0f)) return HERO_ERR_SHAPE;
    if (ldo < H * Dh) return HERO_ERR_SHAPE;
    if (B > 65535 || H > 65535 || Sq > 0x7fffffffLL || Skv > 0x7fffffffLL) return HERO_ERR_SHAPE;
    const int64_t* ss[3] = {q_strides, k_strides, v_strides};
    for (int t = 0; t < 3; ++t) {
        if (ss[t][3] != 1) return HERO_ERR_UNSUPPORTED;
        if (ss[t][0] % 16 || ss[t][1] % 16 || ss[t][2] % 16) return HERO_ERR_ALIGN;
    }
    const int64_t o_elem = out_dt == dt8 ? 1 : 2;
    if ((ldo * o_elem) % 16 != 0 || !hero_aligned16(out) || !hero_aligned16(q) || !hero_aligned16(k) || !hero_aligned16(v))
        return HERO_ERR_ALIGN;
    AttnArgs a;
    a.q = q; a.k = k; a.v = v;
    for (int t = 0; t < 4; ++t) { a.qs[t] = q_strides[t]; a.ks[t] = k_strides[t]; a.vs[t] = v_strides[t]; }
    a.B = (int)B; a.H = (int)H; a.Sq = (int)Sq; a.Skv = (int)Skv;
    a.qk_scale = qk_scale; a.qk_scale_h = qk_scale_h; a.p_scale = p_scale; a.out_col_scale = out_col_scale; a.scale_is_scalar = out_scale_is_scalar;
    a.mask = (int)mask; a.kv_len = kv_len; a.out = out; a.ldo = ldo;
    a.use_buf = Skv > 0 && k_strides[1] >= 0 && v_strides[1] >= 0 &&
                (Skv + BKV) * k_strides[1] + Dh < (1LL << 31) && (Skv + BKV) * v_strides[1] + Dh < (1LL << 31);
    hipStream_t st = (hipStream_t)stream;
    if (Skv == 0) {     // no keys at all: every query outputs 0
        const int64_t bytes = B * Sq * ldo * o_elem;                 // a multiple of 16 (ldo rule)
        const int64_t blocks = (bytes / 16 + 255) / 256;
        if (blocks > 0x7fffffffLL) return HERO_ERR_SHAPE;
        hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (int8_t*)out, bytes);
        return hero_launch_status();
    }
    if (online) return Dh == 64 ? launch<64, true>(a, out_dt, st) : launch<128, true>(a, out_dt, st);
    if (Sq == 1 && Skv <= DEC_MAX_KEYS) {          // decode: the cache-streaming kernel
        dim3 grid((unsigned)H, (unsigned)B), block(256);
        const size_t lds = (size_t)Skv * sizeof(int);
#define HERO_DEC(DH_, ODT_, FMT_) do { \
            if (!decode_lds_ready<DH_, ODT_, FMT_>(lds)) return HERO_ERR_LAUNCH; \
            hipLaunchKernelGGL((int8_attn_decode_kernel<DH_, ODT_, FMT_>), grid, block, lds, st, a); } while (0)
#define HERO_DEC_DT(DH_, FMT_) do { \
            if (out_dt == HERO_BF16) HERO_DEC(DH_, HERO_BF16, FMT_); else if (out_dt == HERO_F16) HERO_DEC(DH_, HERO_F16, FMT_); \
            else HERO_DEC(DH_, FMT_, FMT_); } while (0)
        if (fp8) { if (Dh == 64) HERO_DEC_DT(64, HERO_F8E4M3); else HERO_DEC_DT(128, HERO_F8E4M3); }
        else { if (Dh == 64) HERO_DEC_DT(64, HERO_I8); else HERO_DEC_DT(128, HERO_I8); }
#undef HERO_DEC_DT
#undef HERO_DEC
        return hero_launch_status();
    }
    if (fp8) return Dh == 64 ? launch<64, false, HERO_F8E4M3>(a, out_dt, st) : launch<128, false, HERO_F8E4M3>(a, out_dt, st);
    return Dh == 64 ? launch<64>(a, out_dt, st) : launch<128>(a, out_dt, st);
}

}  // namespace

extern "C" hero_status hero_int8_attn(const int8_t* q, const int64_t q_strides[4],
                                      const int8_t* k, const int64_t k_strides[4],
                                      const int8_t* v, const int64_t v_strides[4],
                                      int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                                      float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                                      hero_mask mask, const int32_t* kv_len,
                                      void* out, hero_dtype out_dt, int64_t ldo, void* stream) {
    return attn_entry(q, q_strides, k, k_strides, v, v_strides, B, H, Sq, Skv, Dh, qk_scale, nullptr, false, false, p_scale,
                      out_col_scale, out_scale_is_scalar, mask, kv_len, out, out_dt, ldo, stream);
}

extern "C" hero_status hero_int8_attn_online(const int8_t* q, const int64_t q_strides[4],
                                             const int8_t* k, const int64_t k_strides[4],
                                             const int8_t* v, const int64_t v_strides[4],
                                             int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                                             const float* qk_scale_h, float p_scale, const float* out_col_scale,
                                             int out_scale_is_scalar, hero_mask mask, const int32_t* kv_len,
                                             void* out, hero_dtype out_dt, int64_t ldo, void* stream) {
    return attn_entry(q, q_strides, k, k_strides, v, v_strides, B, H, Sq, Skv, Dh, 0.0f, qk_scale_h, true, false, p_scale,
                      out_col_scale, out_scale_is_scalar, mask, kv_len, out, out_dt, ldo, stream);
}

extern "C" hero_status hero_fp8_attn(const void* q, const int64_t q_strides[4],
                                     const void* k, const int64_t k_strides[4],
                                     const void* v, const int64_t v_strides[4],
                                     int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                                     float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                                     hero_mask mask, const int32_t* kv_len,
                                     void* out, hero_dtype out_dt, int64_t ldo, void* stream) {
    return attn_entry((const int8_t*)q, q_strides, (const int8_t*)k, k_strides, (const int8_t*)v, v_strides, B, H, Sq, Skv, Dh,
                      qk_scale, nullptr, false, true, p_scale, out_col_scale, out_scale_is_scalar, mask, kv_len, out, out_dt, ldo, stream);
}
