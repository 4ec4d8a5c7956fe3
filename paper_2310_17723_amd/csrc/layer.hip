// hero_layer_fwd: one W8A8 transformer layer (paper Sec. 2.2.2 attention module and
// Sec. 2.2.3 MLP module chained; Sec. 2.3 / Table 1 per-module INT8 / BF16 switch).
// The host only enqueues kernels on the caller's stream; there is no synchronisation and
// no allocation: intermediates live in the caller's workspace.
//
// POST_LN (BERT):  X_in,int8 S_in -> QKV -> attention -> W_o -> LN^quant(X_in, X_o)
//                  -> FC1 + GELU^quant -> FC2 -> LN^quant(X_mid, X_2) -> X_out,int8 S_out
// PRE_LN (GPT):    h (16-bit) -> LN^quant -> QKV -> attention -> W_o (+h) -> LN^quant
//                  -> FC1 + GELU^quant -> FC2 (+h); h is updated in place.
// Every module is INT8 or 16-bit (bf16, or fp16 with HERO_M_F16) as its mode bit says; a tensor between two
// modules is INT8 codes when its consumer is INT8 and 16-bit values otherwise (LN^quant writes its 16-bit copy
// beside the codes when the next linear is 16-bit).
#include "hero_common.h"
#include <algorithm>

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    size_t xin_q, xin_s, xin_hp, qkv, attn, xo, mid_q, mid_s, mid_hp, a, x2, gemm_ws, gemm_ws_bytes, total;
};

Workspace plan(const hero_layer_desc* d, int64_t T) {
    Workspace w;
    const bool pre = d->arch == HERO_ARCH_PRE_LN;
    const size_t e_qkv = (d->mode_mask & HERO_M_ATTN) ? 1 : 2;
    const size_t e_attn = (d->mode_mask & HERO_M_ATTN_OUT) ? 1 : 2;
    const size_t e_a = (d->mode_mask & HERO_M_FC2) ? 1 : 2;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    w.xin_q = take(pre ? (size_t)T * d->d : 0);
    w.xin_s = take(pre ? (size_t)T * 4 : 0);
    w.xin_hp = take(pre && !(d->mode_mask & HERO_M_QKV) ? (size_t)T * d->d * 2 : 0);   // 16-bit LN output for a 16-bit QKV
    w.qkv = take((size_t)T * 3 * d->d * e_qkv);
    w.attn = take((size_t)T * d->d * e_attn);
    w.xo = take(pre ? 0 : (size_t)T * d->d * e_attn);
    w.mid_q = take((size_t)T * d->d);
    w.mid_s = take((size_t)T * 4);
    w.mid_hp = take(!(d->mode_mask & HERO_M_FC1) ? (size_t)T * d->d * 2 : 0);          // 16-bit X_mid for a 16-bit FC1
    w.a = take((size_t)T * d->f * e_a);
    w.x2 = take(pre ? 0 : (size_t)T * d->d * e_a);
    // split-K scratch of the skinny (decode) GEMMs: the largest of the four shapes, shared (stream order);
    // none in the FP8 variant (fp32 partial sums would not commute)
    size_t g = 0;
    if (!(d->mode_mask & HERO_M_FP8)) {
        g = hero_int8_gemm_workspace_bytes(T, 3 * (int64_t)d->d, d->d);
        g = std::max(g, hero_int8_gemm_workspace_bytes(T, d->d, d->d));
        g = std::max(g, hero_int8_gemm_workspace_bytes(T, d->f, d->d));
        g = std::max(g, hero_int8_gemm_workspace_bytes(T, d->d, d->f));
    }
    w.gemm_ws_bytes = g;
    w.gemm_ws = take(g);
    w.total = off;
    return w;
}

// Copy this call's K and V codes from the fused QKV buffer [T, 3d] into the INT8 KV cache
// [B, H, Smax, Dh] at positions kv_len[b]-S .. kv_len[b]-1.  One thread moves 16 bytes.
__global__ void kv_append_kernel(const int8_t* qkv, int8_t* kc, int8_t* vc, const int32_t* kv_len,
                                 int B, int S, int H, int Dh, int64_t Smax) {
    const int d = H * Dh, cpr = d / 16;                              // 16-byte chunks per row
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)B * S * cpr) return;
    const int c = (int)(idx % cpr);
    const int64_t t = idx / cpr;
    const int b = (int)(t / S), s = (int)(t % S);
    const int pos = kv_len[b] - S + s;
    if (pos < 0 || pos >= Smax) return;
    const int h = (c * 16) / Dh, e = (c * 16) % Dh;
    const int64_t dst = (((int64_t)b * H + h) * Smax + pos) * Dh + e;
    const int8_t* src = qkv + t * 3 * d + c * 16;
    *reinterpret_cast<v4i*>(kc + dst) = *reinterpret_cast<const v4i*>(src + d);
    *reinterpret_cast<v4i*>(vc + dst) = *reinterpret_cast<const v4i*>(src + 2 * d);
}

hero_status check(const hero_layer_desc* d) {
    if (d->arch != HERO_ARCH_POST_LN && d->arch != HERO_ARCH_PRE_LN) return HERO_ERR_UNSUPPORTED;
    if (d->d <= 0 || d->H <= 0 || d->Dh <= 0 || d->f <= 0 || (int64_t)d->H * d->Dh != d->d) return HERO_ERR_SHAPE;
    const uint32_t m = d->mode_mask;
    // a 16-bit module hands 16-bit values on, and there is no stand-alone quantization kernel (the method removes
    // it): INT8 attention needs an INT8 QKV, an INT8 output linear an INT8 attention, an INT8 FC2 an INT8 FC1
    if ((m & HERO_M_ATTN) && !(m & HERO_M_QKV)) return HERO_ERR_UNSUPPORTED;
    if ((m & HERO_M_ATTN_OUT) && !(m & HERO_M_ATTN)) return HERO_ERR_UNSUPPORTED;
    if ((m & HERO_M_FC2) && !(m & HERO_M_FC1)) return HERO_ERR_UNSUPPORTED;
    if (m & ~(uint32_t)(HERO_MODE_M3 | HERO_M_FP8 | HERO_M_F16)) return HERO_ERR_UNSUPPORTED;
    if ((m & HERO_M_FP8) && (m & (HERO_MODE_M3 | HERO_M_F16)) != HERO_MODE_M3) return HERO_ERR_UNSUPPORTED;   // FP8: every module 8-bit
    return HERO_OK;
}

#define HERO_TRY(expr) do { hero_status s_ = (expr); if (s_ != HERO_OK) return s_; } while (0)

}  // namespace

extern "C" const char* hero_strerror(hero_status s) {
    switch (s) {
    case HERO_OK: return "ok";
    case HERO_ERR_NULL: return "a required pointer is NULL";
    case HERO_ERR_SHAPE: return "invalid or inconsistent size";
    case HERO_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case HERO_ERR_UNSUPPORTED: return "unsupported shape, dtype or mode";
    case HERO_ERR_WORKSPACE: return "workspace missing, misaligned, too small, or larger than the built-in scratch";
    case HERO_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

extern "C" const char* hero_build_arch(void) { return HERO_BUILD_ARCH; }

extern "C" size_t hero_layer_workspace_bytes(const hero_layer_desc* desc, int64_t B, int64_t S) {
    if (!desc || B < 0 || S < 0 || check(desc) != HERO_OK) return 0;
    return plan(desc, B * S).total;
}

extern "C" hero_status hero_layer_fwd(const hero_layer_desc* desc, const hero_layer_weights* w, const hero_layer_io* io,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc || !w || !io) return HERO_ERR_NULL;
    HERO_TRY(check(desc));
    const int64_t B = io->B, S = io->S, T = B * S;
    if (B < 0 || S < 0) return HERO_ERR_SHAPE;
    if (T == 0) return HERO_OK;
    const Workspace ws = plan(desc, T);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws.total) return HERO_ERR_WORKSPACE;
    const bool pre = desc->arch == HERO_ARCH_PRE_LN;
    const uint32_t mode = desc->mode_mask;
    const bool q_i8 = mode & HERO_M_QKV, attn_i8 = mode & HERO_M_ATTN, o_i8 = mode & HERO_M_ATTN_OUT;
    const bool fc1_i8 = mode & HERO_M_FC1, fc2_i8 = mode & HERO_M_FC2;
    const hero_dtype HP = (mode & HERO_M_F16) ? HERO_F16 : HERO_BF16;     // the layer's 16-bit type
    const int64_t d = desc->d, f = desc->f, H = desc->H, Dh = desc->Dh;
    const bool cache = io->k_cache || io->v_cache;
    // ---- everything that can be checked is checked before the first launch
    if (pre ? !io->h : (!io->out_q || !io->out_scale || (q_i8 ? (!io->x_q || !io->x_scale) : !io->x_hp))) return HERO_ERR_NULL;
    if (!w->ln1_g || !w->ln2_g) return HERO_ERR_NULL;
    if (q_i8 ? (!w->w_qkv || !w->w_qkv_s) : !w->w_qkv_hp) return HERO_ERR_NULL;
    if (fc1_i8 ? (!w->w_1 || !w->w_1_s) : !w->w_1_hp) return HERO_ERR_NULL;
    if (attn_i8 && !w->attn_out_scale) return HERO_ERR_NULL;
    if (o_i8 ? (!w->w_o || !w->w_o_s) : !w->w_o_bf16) return HERO_ERR_NULL;
    if (fc2_i8 ? (!w->w_2 || !w->w_2_s || !w->S_a) : !w->w_2_bf16) return HERO_ERR_NULL;
    if (!pre && ((o_i8 && !w->S_o) || (fc2_i8 && !w->S_x2))) return HERO_ERR_NULL;
    if (cache) {
        if (!io->k_cache || !io->v_cache || !io->kv_len) return HERO_ERR_NULL;
        if (!attn_i8) return HERO_ERR_UNSUPPORTED;            // the cache holds INT8 (SQ) codes
        if (io->Smax < S) return HERO_ERR_SHAPE;
    }
    if (desc->mask == HERO_MASK_PADDING && !io->kv_len) return HERO_ERR_NULL;
    if (Dh != 64 && Dh != 128) return HERO_ERR_UNSUPPORTED;
    if (d % 64 || f % 64) return HERO_ERR_UNSUPPORTED;
    // what the chained entry points would refuse only after earlier stages had been enqueued (and, pre-LN, after
    // h had been partly updated in place): the GeMM^quant row bound, the LN^quant row width (a row lives in one
    // wavefront's registers: 8192 columns behind INT8 addends, 4096 behind the 16-bit residual stream), alignment
    if (T >= (1LL << 23)) return HERO_ERR_SHAPE;
    if (d > ((pre || !q_i8 || !fc1_i8) ? 4096 : 8192)) return HERO_ERR_UNSUPPORTED;
    {
        const void* const ptrs[] = {w->w_qkv, w->w_o, w->w_1, w->w_2, w->w_o_bf16, w->w_2_bf16, w->w_qkv_hp, w->w_1_hp,
                                    io->x_q, io->out_q, io->h, io->k_cache, io->v_cache, io->x_hp, io->out_hp};
        for (const void* p : ptrs) if (!hero_aligned16(p)) return HERO_ERR_ALIGN;
    }

    char* base = (char*)workspace;
    int8_t* xin_q = pre ? (int8_t*)(base + ws.xin_q) : const_cast<int8_t*>(io->x_q);
    float* xin_s = pre ? (float*)(base + ws.xin_s) : const_cast<float*>(io->x_scale);
    void* xin_hp = pre ? (void*)(base + ws.xin_hp) : const_cast<void*>(io->x_hp);    // read only when QKV is 16-bit
    void* mid_hp = base + ws.mid_hp;
    void* qkv = base + ws.qkv;
    void* attn = base + ws.attn;
    void* xo = base + ws.xo;
    int8_t* mid_q = (int8_t*)(base + ws.mid_q);
    float* mid_s = (float*)(base + ws.mid_s);
    void* act = base + ws.a;
    void* x2 = base + ws.x2;
    hipStream_t st = (hipStream_t)stream;
    void* gws = ws.gemm_ws_bytes ? (void*)(base + ws.gemm_ws) : nullptr;   // split-K scratch of the skinny GEMMs

    // ---- the FP8 variant (Sec. 2.1): the same chain with E4M3 codes in every 8-bit buffer
    if (mode & HERO_M_FP8) {
        const hero_dtype F8 = HERO_F8E4M3;
        if (pre)
            HERO_TRY(hero_ln_quant_fp8(io->h, HERO_BF16, nullptr, nullptr, F8, nullptr, w->ln1_g, w->ln1_b, desc->eps,
                                       T, d, xin_q, xin_s, nullptr, HERO_BF16, stream));
        HERO_TRY(hero_fp8_gemm_prefetching(xin_q, d, xin_s, w->w_qkv, d, w->w_qkv_s, w->b_qkv, nullptr, HERO_BF16, 0,
                                           HERO_EPI_REQUANT, nullptr, qkv, F8, 3 * d, T, 3 * d, d, stream, w->w_o, (size_t)(d * d)));
        const int64_t qs[4] = {S * 3 * d, 3 * d, Dh, 1};
        const int8_t* qp = (const int8_t*)qkv;
        const int8_t *kp = qp + d, *vp = qp + 2 * d;
        int64_t ks[4] = {qs[0], qs[1], qs[2], qs[3]};
        int64_t Skv = S;
        if (cache) {                                              // the cache holds E4M3 (SQ) codes: a byte copy
            const int64_t n = T * (d / 16);
            hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                               qp, io->k_cache, io->v_cache, io->kv_len, (int)B, (int)S, (int)H, (int)Dh, io->Smax);
            HERO_TRY(hero_launch_status());
            kp = io->k_cache; vp = io->v_cache; Skv = io->Smax;
            ks[0] = H * io->Smax * Dh; ks[1] = Dh; ks[2] = io->Smax * Dh; ks[3] = 1;
        }
        HERO_TRY(hero_fp8_attn(qp, qs, kp, ks, vp, ks, B, H, S, Skv, Dh, w->qk_scale, w->p_scale,
                               w->attn_out_scale, 0, (hero_mask)desc->mask, io->kv_len, attn, F8, d, stream));
        if (!pre) {
            HERO_TRY(hero_fp8_gemm_prefetching(attn, d, nullptr, w->w_o, d, w->w_o_s, w->b_o, nullptr, HERO_BF16, 0,
                                               HERO_EPI_REQUANT, nullptr, xo, F8, d, T, d, d, stream, w->w_1, (size_t)(f * d)));
            HERO_TRY(hero_ln_quant_fp8(xin_q, F8, xin_s, xo, F8, w->S_o, w->ln1_g, w->ln1_b, desc->eps, T, d,
                                       mid_q, mid_s, nullptr, HERO_BF16, stream));
        } else {
            HERO_TRY(hero_fp8_gemm_prefetching(attn, d, nullptr, w->w_o, d, w->w_o_s, w->b_o, io->h, HERO_BF16, d,
                                               HERO_EPI_DEQUANT, nullptr, io->h, HERO_BF16, d, T, d, d, stream, w->w_1, (size_t)(f * d)));
            HERO_TRY(hero_ln_quant_fp8(io->h, HERO_BF16, nullptr, nullptr, F8, nullptr, w->ln2_g, w->ln2_b, desc->eps,
                                       T, d, mid_q, mid_s, nullptr, HERO_BF16, stream));
        }
        HERO_TRY(hero_fp8_gemm_prefetching(mid_q, d, mid_s, w->w_1, d, w->w_1_s, w->b_1, nullptr, HERO_BF16, 0,
                                           HERO_EPI_GELU_REQUANT, w->S_a, act, F8, f, T, f, d, stream, w->w_2, (size_t)(d * f)));
        if (!pre) {
            HERO_TRY(hero_fp8_gemm_prefetching(act, f, nullptr, w->w_2, f, w->w_2_s, w->b_2, nullptr, HERO_BF16, 0,
                                               HERO_EPI_REQUANT, nullptr, x2, F8, d, T, d, f, stream, io->next_read, io->next_read_bytes));
            HERO_TRY(hero_ln_quant_fp8(mid_q, F8, mid_s, x2, F8, w->S_x2, w->ln2_g, w->ln2_b, desc->eps, T, d,
                                       io->out_q, io->out_scale, nullptr, HERO_BF16, stream));
        } else {
            HERO_TRY(hero_fp8_gemm_prefetching(act, f, nullptr, w->w_2, f, w->w_2_s, w->b_2, io->h, HERO_BF16, d,
                                               HERO_EPI_DEQUANT, nullptr, io->h, HERO_BF16, d, T, d, f, stream, io->next_read, io->next_read_bytes));
        }
        return HERO_OK;
    }

    // (1) PRE_LN: LN^quant of the residual stream (with its 16-bit copy when the QKV module is 16-bit)
    if (pre)
        HERO_TRY(hero_ln_quant(io->h, HP, nullptr, nullptr, HERO_I8, nullptr, w->ln1_g, w->ln1_b, desc->eps,
                               T, d, xin_q, xin_s, q_i8 ? nullptr : xin_hp, HP, stream));
    // (2) QKV: SQ codes for an INT8 attention (bare Round), 16-bit values otherwise
    if (q_i8)
        HERO_TRY(hero_int8_gemm_prefetching(xin_q, d, xin_s, w->w_qkv, d, w->w_qkv_s, w->b_qkv, nullptr, HP, 0,
                                            attn_i8 ? HERO_EPI_REQUANT : HERO_EPI_DEQUANT, nullptr,
                                            qkv, attn_i8 ? HERO_I8 : HP, 3 * d, T, 3 * d, d, gws, ws.gemm_ws_bytes, stream,
                                            o_i8 ? w->w_o : nullptr, (size_t)(d * d)));
    else
        HERO_TRY(hero_hp_gemm(xin_hp, d, w->w_qkv_hp, d, w->b_qkv, nullptr, 0, 0, qkv, 3 * d, T, 3 * d, d, HP, stream));
    // (3) attention
    const int64_t qs[4] = {S * 3 * d, 3 * d, Dh, 1};
    if (attn_i8) {
        const int8_t* qp = (const int8_t*)qkv;
        const int8_t *kp = qp + d, *vp = qp + 2 * d;
        int64_t ks[4] = {qs[0], qs[1], qs[2], qs[3]};
        int64_t Skv = S;
        if (cache) {
            const int64_t n = T * (d / 16);
            hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                               qp, io->k_cache, io->v_cache, io->kv_len, (int)B, (int)S, (int)H, (int)Dh, io->Smax);
            HERO_TRY(hero_launch_status());
            kp = io->k_cache; vp = io->v_cache; Skv = io->Smax;
            ks[0] = H * io->Smax * Dh; ks[1] = Dh; ks[2] = io->Smax * Dh; ks[3] = 1;
        }
        HERO_TRY(hero_int8_attn(qp, qs, kp, ks, vp, ks, B, H, S, Skv, Dh, w->qk_scale, w->p_scale,
                                w->attn_out_scale, o_i8 ? 0 : 1, (hero_mask)desc->mask, io->kv_len,
                                attn, o_i8 ? HERO_I8 : HP, d, stream));
    } else {
        const uint16_t* qp = (const uint16_t*)qkv;
        HERO_TRY(hero_hp_attn(qp, qs, qp + d, qs, qp + 2 * d, qs, B, H, S, S, Dh, w->qk_scale,
                              (hero_mask)desc->mask, io->kv_len, attn, d, HP, stream));
    }
    // (4) attention-output linear and the LN^quant that closes the attention module; X_mid also as 16-bit values
    // when FC1 is 16-bit
    const void* x1 = q_i8 ? (const void*)xin_q : (const void*)xin_hp;      // the layer input as LN^quant's first addend
    const hero_dtype x1_dt = q_i8 ? HERO_I8 : HP;
    if (!pre) {
        if (o_i8)
            HERO_TRY(hero_int8_gemm_prefetching((const int8_t*)attn, d, nullptr, w->w_o, d, w->w_o_s, w->b_o, nullptr, HP, 0,
                                                HERO_EPI_REQUANT, nullptr, xo, HERO_I8, d, T, d, d, gws, ws.gemm_ws_bytes, stream,
                                                fc1_i8 ? w->w_1 : nullptr, (size_t)(f * d)));
        else
            HERO_TRY(hero_hp_gemm(attn, d, w->w_o_bf16, d, w->b_o, nullptr, 0, 0, xo, d, T, d, d, HP, stream));
        HERO_TRY(hero_ln_quant(x1, x1_dt, q_i8 ? xin_s : nullptr, xo, o_i8 ? HERO_I8 : HP, o_i8 ? w->S_o : nullptr,
                               w->ln1_g, w->ln1_b, desc->eps, T, d, mid_q, mid_s, fc1_i8 ? nullptr : mid_hp, HP, stream));
    } else {
        if (o_i8)
            HERO_TRY(hero_int8_gemm_prefetching((const int8_t*)attn, d, nullptr, w->w_o, d, w->w_o_s, w->b_o, io->h, HP, d,
                                                HERO_EPI_DEQUANT, nullptr, io->h, HP, d, T, d, d, gws, ws.gemm_ws_bytes, stream,
                                                fc1_i8 ? w->w_1 : nullptr, (size_t)(f * d)));
        else
            HERO_TRY(hero_hp_gemm(attn, d, w->w_o_bf16, d, w->b_o, io->h, d, 0, io->h, d, T, d, d, HP, stream));
        HERO_TRY(hero_ln_quant(io->h, HP, nullptr, nullptr, HERO_I8, nullptr, w->ln2_g, w->ln2_b, desc->eps,
                               T, d, mid_q, mid_s, fc1_i8 ? nullptr : mid_hp, HP, stream));
    }
    // (5) FC1 + GELU: GELU^quant codes for an INT8 FC2 (X_1 stays in registers), 16-bit values otherwise
    if (fc1_i8)
        HERO_TRY(hero_int8_gemm_prefetching(mid_q, d, mid_s, w->w_1, d, w->w_1_s, w->b_1, nullptr, HP, 0,
                                            fc2_i8 ? HERO_EPI_GELU_REQUANT : HERO_EPI_DEQUANT_GELU, w->S_a,
                                            act, fc2_i8 ? HERO_I8 : HP, f, T, f, d, gws, ws.gemm_ws_bytes, stream,
                                            fc2_i8 ? w->w_2 : nullptr, (size_t)(d * f)));
    else
        HERO_TRY(hero_hp_gemm(mid_hp, d, w->w_1_hp, d, w->b_1, nullptr, 0, 1, act, f, T, f, d, HP, stream));
    // (6) FC2 and the closing LN^quant (POST_LN) or residual add (PRE_LN)
    if (!pre) {
        if (fc2_i8)
            HERO_TRY(hero_int8_gemm_prefetching((const int8_t*)act, f, nullptr, w->w_2, f, w->w_2_s, w->b_2, nullptr, HP, 0,
                                                HERO_EPI_REQUANT, nullptr, x2, HERO_I8, d, T, d, f, gws, ws.gemm_ws_bytes, stream,
                                                io->next_read, io->next_read_bytes));
        else
            HERO_TRY(hero_hp_gemm(act, f, w->w_2_bf16, f, w->b_2, nullptr, 0, 0, x2, d, T, d, f, HP, stream));
        HERO_TRY(hero_ln_quant(fc1_i8 ? (const void*)mid_q : (const void*)mid_hp, fc1_i8 ? HERO_I8 : HP, fc1_i8 ? mid_s : nullptr,
                               x2, fc2_i8 ? HERO_I8 : HP, fc2_i8 ? w->S_x2 : nullptr, w->ln2_g, w->ln2_b, desc->eps, T, d,
                               io->out_q, io->out_scale, io->out_hp, HP, stream));
    } else {
        if (fc2_i8)
            HERO_TRY(hero_int8_gemm_prefetching((const int8_t*)act, f, nullptr, w->w_2, f, w->w_2_s, w->b_2, io->h, HP, d,
                                                HERO_EPI_DEQUANT, nullptr, io->h, HP, d, T, d, f, gws, ws.gemm_ws_bytes, stream,
                                                io->next_read, io->next_read_bytes));
        else
            HERO_TRY(hero_hp_gemm(act, f, w->w_2_bf16, f, w->b_2, io->h, d, 0, io->h, d, T, d, f, HP, stream));
    }
    return HERO_OK;
}
