"""Oracle: the paper's layer dataflow, offline preparation and the unquantized model.

TEST INFRASTRUCTURE (see ``oracle/__init__.py``).  Written from the equations of
Sec. 2.2.2 (attention module), Sec. 2.2.3 (MLP module) and Sec. 2.3 / Table 1 (modes),
in the paper's notation:

    X_in,int8 S_in  --QKV-->  X_{q,k,v},int8 (SQ)  --attention-->  X_attn,int8 S_attn (FWQ)
    --W_o-->  X_o,int8 S_o (FWQ)  --LN^quant(X_in, X_o)-->  X_mid,int8 S_mid (TWQ)
    --W_1, GELU^quant-->  A_int8 S_a (FWQ)  --W_2-->  X_2,int8 S_x2 (FWQ)
    --LN^quant(X_mid, X_2)-->  X_out,int8 S_out (TWQ)

The pre-LN (GPT) variant, the bias, the masks and the KV cache are not in the paper; the
readings taken are listed in the design document.  Everything numeric is done by the C++
operators in ``hero_oracle.cpp``; numpy fp64 is used for the unquantized model, the
calibration statistics and the scale folding.
"""
from __future__ import annotations

import math

import numpy as np

import oracle as O

POST_LN, PRE_LN = 0, 1
# One bit per switchable module (Table 1 columns after "Embedding"); 1 = INT8, 0 = BF16.
M_QKV, M_ATTN, M_ATTN_OUT, M_FC1, M_FC2 = 1, 2, 4, 8, 16
MODE_M3 = M_QKV | M_ATTN | M_ATTN_OUT | M_FC1 | M_FC2
MODE_M2 = M_QKV | M_ATTN | M_ATTN_OUT | M_FC1
MODE_M1 = M_QKV | M_FC1
MODE_M0 = 0          # every module 16-bit: the layer of Table 2's FP16 row
S_P = np.float32(1.0 / 255.0)
S_P_FP8 = np.float32(1.0 / 448.0)     # the FP8 variant: p = 1 is the largest E4M3 code


# ------------------------------------------------------------------ unquantized model (fp64)
def _gelu64(x):
    from scipy.special import erf
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def _ln64(x, g, b, eps):
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def _visible(mask, i, Sq, length):
    last = length - 1
    if mask == O.MASK_CAUSAL:
        last = min(last, i + (length - Sq))
    return last + 1


def fp64_attention(q, k, v, B, Sq, Skv, H, Dh, mask, kv_len):
    """softmax(Q K^T / sqrt(Dh)) V per (batch, head); q [B*Sq, d], k/v [B*Skv, d]."""
    out = np.zeros((B * Sq, H * Dh))
    for b in range(B):
        length = Skv if kv_len is None else min(int(kv_len[b]), Skv)
        for h in range(H):
            qs = q[b * Sq:(b + 1) * Sq, h * Dh:(h + 1) * Dh]
            ks = k[b * Skv:(b + 1) * Skv, h * Dh:(h + 1) * Dh]
            vs = v[b * Skv:(b + 1) * Skv, h * Dh:(h + 1) * Dh]
            a = qs @ ks.T / math.sqrt(Dh)
            for i in range(Sq):
                n = _visible(mask, i, Sq, length)
                if n <= 0:
                    continue
                e = np.exp(a[i, :n] - a[i, :n].max())
                out[b * Sq + i, h * Dh:(h + 1) * Dh] = (e / e.sum()) @ vs[:n]
    return out


def fp64_layer(p, x, shape, B, S, kv_len=None):
    """The unquantized layer (Sec. 2.2.2 first equation block, Sec. 2.2.3 first block).
    x: [B*S, d] float64, the layer input (post-LN: already normalised; pre-LN: the
    residual stream).  Returns every intermediate the calibration needs."""
    d, H, Dh = shape.d, shape.H, shape.Dh
    P = {k_: np.asarray(v_, np.float64) for k_, v_ in p.items()}
    t = {}
    xin = _ln64(x, P["ln1_g"], P["ln1_b"], shape.eps) if shape.arch == PRE_LN else x
    qkv = xin @ P["w_qkv"] + P["b_qkv"]
    t["q"], t["k"], t["v"] = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    t["attn"] = fp64_attention(t["q"], t["k"], t["v"], B, S, S, H, Dh, shape.mask, kv_len)
    t["o"] = t["attn"] @ P["w_o"] + P["b_o"]
    if shape.arch == POST_LN:
        mid = _ln64(x + t["o"], P["ln1_g"], P["ln1_b"], shape.eps)
        x1 = mid @ P["w_1"] + P["b_1"]
    else:
        mid = x + t["o"]
        x1 = _ln64(mid, P["ln2_g"], P["ln2_b"], shape.eps) @ P["w_1"] + P["b_1"]
    t["mid"] = mid
    t["a"] = _gelu64(x1)
    t["x2"] = t["a"] @ P["w_2"] + P["b_2"]
    t["out"] = _ln64(mid + t["x2"], P["ln2_g"], P["ln2_b"], shape.eps) if shape.arch == POST_LN else mid + t["x2"]
    return t


# ------------------------------------------------------------------ calibration + preparation
def _absmax_scale(a, axis=None, qmax=127.0):
    """Static scale = absmax / qmax over the calibration tokens (no truncation, Sec. 3
    discussion); qmax = 127 for INT8 codes, 448 for E4M3; a zero range gets scale 1."""
    m = np.abs(a).max(axis=axis)
    s = np.where(m == 0.0, qmax, m) / qmax
    return np.float32(s) if axis is None else s.astype(np.float32)


def calibrate(p, x_calib, shape, B, S, kv_len=None, fp8=False):
    """Static scales from a forward pass of the unquantized layer on calibration tokens:
    SQ scalars for X_q, X_k, X_v; FWQ vectors for X_attn, X_o, A, X_2; S_p = 1/255 (fp8: every range is
    mapped to the largest E4M3 value 448 instead of 127, and S_p = 1/448)."""
    t = fp64_layer(p, np.asarray(x_calib, np.float64), shape, B, S, kv_len)
    qm = 448.0 if fp8 else 127.0
    sc = {"S_q": _absmax_scale(t["q"], None, qm), "S_k": _absmax_scale(t["k"], None, qm), "S_v": _absmax_scale(t["v"], None, qm),
          "S_attn": _absmax_scale(t["attn"], 0, qm), "S_o": _absmax_scale(t["o"], 0, qm),
          "S_a": _absmax_scale(t["a"], 0, qm), "S_x2": _absmax_scale(t["x2"], 0, qm), "S_p": S_P_FP8 if fp8 else S_P}
    return sc, t["out"]


def _hp(a, dt):
    return O.f32_to_hp(np.asarray(a, np.float32), dt)


def check_mode(mode):
    """Which module subsets are a layer (Sec. 2.3: every module has an INT8 / 16-bit switch).  A 16-bit module
    hands 16-bit values on, and the method has no stand-alone quantization kernel, so an INT8 attention needs an
    INT8 QKV in front of it (SQ codes), an INT8 attention-output linear an INT8 attention (FWQ codes), an INT8 FC2
    an INT8 FC1 (GELU^quant codes).  Table 1's M1 / M2 / M3 and the all-16-bit layer satisfy this."""
    if (mode & M_ATTN) and not (mode & M_QKV):
        raise ValueError("an INT8 attention needs an INT8 QKV GeMM in front of it")
    if (mode & M_ATTN_OUT) and not (mode & M_ATTN):
        raise ValueError("an INT8 attention-output linear needs INT8 attention in front of it")
    if (mode & M_FC2) and not (mode & M_FC1):
        raise ValueError("an INT8 FC2 needs an INT8 FC1 (GELU^quant) in front of it")


def prepare(p, sc, shape, mode=MODE_M3, fp8=False, hp_dt=O.BF16):
    """Fold the static scales into the weights, then quantize column-wise (Sec. 2.2.2:
    W~_q = W_q / S_q and W~_o = S_attn W_o / S_o;  Sec. 2.2.3: W~_2 = S_a W_2 / S_x2).
    Biases fold with the output scale.  Folding is done in fp64, cast to fp32 once, then
    quantized.  BF16 modules keep the unfolded weights cast to bf16, stored [N][K].
    fp8: the FP8 variant of Sec. 2.1 (every module 8-bit): the same folds, E4M3 weight codes with column scale
    max / 448; the scales in ``sc`` must come from calibrate(..., fp8=True)."""
    d = shape.d
    P = {k_: np.asarray(v_, np.float64) for k_, v_ in p.items()}
    w = {"mode": mode, "S_p": sc["S_p"], "fp8": bool(fp8), "hp_dt": hp_dt}
    if fp8 and mode != MODE_M3:
        raise ValueError("the FP8 variant runs every module in 8 bits")
    if hp_dt not in (O.BF16, O.F16):
        raise ValueError("the 16-bit side is BF16 or FP16")
    check_mode(mode)
    fold_quant = O.weight_fold_quant_fp8 if fp8 else O.weight_fold_quant
    # --- QKV (INT8 in every mode of Table 1; 16-bit in the all-16-bit layer).  INT8 attention consumes SQ
    # codes, so S_{q,k,v} are folded; a 16-bit attention consumes dequantized values, so nothing is folded.
    if mode & M_ATTN:
        div = np.concatenate([np.full(d, float(sc["S_q"])), np.full(d, float(sc["S_k"])), np.full(d, float(sc["S_v"]))])
    else:
        div = np.ones(3 * d)
    if mode & M_QKV:
        w["wq_qkv"], w["s_qkv"] = fold_quant(P["w_qkv"], None, div)
    else:
        w["wb_qkv"] = _hp(P["w_qkv"].T.copy(), hp_dt)
    w["b_qkv"] = (P["b_qkv"] / div).astype(np.float32)
    w["qk_scale"] = np.float32(float(sc["S_q"]) * float(sc["S_k"]) / math.sqrt(shape.Dh))
    w["bf16_qk_scale"] = np.float32(1.0 / math.sqrt(shape.Dh))
    # attention output scale: FWQ codes when W_o is INT8, plain values when it is BF16
    pv = float(sc["S_p"]) * float(sc["S_v"])
    w["attn_out_scale"] = (pv / sc["S_attn"].astype(np.float64)).astype(np.float32)
    w["attn_out_scalar"] = np.array([pv], np.float32)
    # --- attention output linear
    post = shape.arch == POST_LN
    if mode & M_ATTN_OUT:
        bo = P["b_o"]
        if post:
            bo = bo / sc["S_o"].astype(np.float64)
        w["wq_o"], w["s_o_w"] = fold_quant(P["w_o"], sc["S_attn"], sc["S_o"] if post else None)
        w["b_o"] = bo.astype(np.float32)
    else:
        w["wb_o"] = _hp(P["w_o"].T.copy(), hp_dt)
        w["b_o"] = P["b_o"].astype(np.float32)
    w["S_o"] = sc["S_o"]
    # --- FC1 (INT8 in every mode of Table 1); GELU^quant divides by S_a, nothing to fold
    if mode & M_FC1:
        w["wq_1"], w["s_1"] = fold_quant(P["w_1"])
    else:
        w["wb_1"] = _hp(P["w_1"].T.copy(), hp_dt)
    w["b_1"] = P["b_1"].astype(np.float32)
    w["S_a"] = sc["S_a"]
    # --- FC2
    if mode & M_FC2:
        b2 = P["b_2"]
        if post:
            b2 = b2 / sc["S_x2"].astype(np.float64)
        w["wq_2"], w["s_2_w"] = fold_quant(P["w_2"], sc["S_a"], sc["S_x2"] if post else None)
        w["b_2"] = b2.astype(np.float32)
    else:
        w["wb_2"] = _hp(P["w_2"].T.copy(), hp_dt)
        w["b_2"] = P["b_2"].astype(np.float32)
    w["S_x2"] = sc["S_x2"]
    for k_ in ("ln1_g", "ln1_b", "ln2_g", "ln2_b"):
        w[k_] = np.asarray(p[k_], np.float32)
    return w


# ------------------------------------------------------------------ the quantized layer
def _heads(a2d, B, S, H, Dh, part, parts=3):
    """[B*S, parts*H*Dh] buffer -> strided [B,S,H,Dh] view of one of its column blocks."""
    return a2d.reshape(B, S, parts, H, Dh)[:, :, part]


def layer_fwd(w, shape, B, S, *, x_q=None, x_s=None, x_hp=None, h=None, kv_len=None, cache=None, trace=None):
    """One layer, every module INT8 or 16-bit as the mode mask says (Sec. 2.3).
    POST_LN: input (x_q int8 [T,d], x_s f32 [T]) when the QKV GeMM is INT8, else x_hp (16-bit bit patterns [T,d]);
    returns (out_q, out_s); the 16-bit copy of the output a 16-bit successor would read is trace["out_hp"].
    PRE_LN: input h (16-bit bit patterns [T,d]) -> new h.  ``cache`` (INT8 attention only) is a dict
    {k, v: int8 [B,H,Smax,Dh]}; the S new key/value rows are written at positions kv_len[b]-S .. kv_len[b]-1 and
    attention runs over the cache.  ``trace`` (a dict) receives every intermediate.  The 16-bit type is
    w["hp_dt"] (BF16 or F16)."""
    if w.get("fp8"):
        return layer_fwd_fp8(w, shape, B, S, x_q=x_q, x_s=x_s, h=h, kv_len=kv_len, cache=cache, trace=trace)
    d, H, Dh, mode = shape.d, shape.H, shape.Dh, w["mode"]
    hp = w.get("hp_dt", O.BF16)
    tr = trace if trace is not None else {}
    post = shape.arch == POST_LN
    check_mode(mode)
    q_i8, attn_i8, o_i8 = bool(mode & M_QKV), bool(mode & M_ATTN), bool(mode & M_ATTN_OUT)
    f1_i8, f2_i8 = bool(mode & M_FC1), bool(mode & M_FC2)
    if cache is not None and not attn_i8:
        raise ValueError("the KV cache holds INT8 (SQ) codes: it needs the INT8 attention")
    # ---- the layer input as the QKV GeMM reads it
    if post:
        xin_q, xin_s, xin_hp = (x_q, x_s, None) if q_i8 else (None, None, x_hp)
    else:
        xin_q, xin_s, xin_hp = O.ln_quant(h, hp, None, None, 0, None, w["ln1_g"], w["ln1_b"], shape.eps,
                                          y_hp_dt=None if q_i8 else hp)
    tr["xin_q"], tr["xin_s"], tr["xin_hp"] = xin_q, xin_s, xin_hp
    # ---- QKV: SQ codes (the bare Round of the folded weights) for an INT8 attention, 16-bit values otherwise
    if q_i8:
        qkv = O.int8_gemm(xin_q, w["wq_qkv"], a_row_scale=xin_s, b_col_scale=w["s_qkv"], bias=w["b_qkv"],
                          epi=O.EPI_REQUANT if attn_i8 else O.EPI_DEQUANT, c_dt=O.I8 if attn_i8 else hp)
    else:
        qkv = O.hp_gemm(xin_hp, w["wb_qkv"], bias=w["b_qkv"], dt=hp)
    tr["qkv"] = qkv
    qv = _heads(qkv, B, S, H, Dh, 0)
    if cache is not None:
        kn, vn = _heads(qkv, B, S, H, Dh, 1), _heads(qkv, B, S, H, Dh, 2)
        for b in range(B):
            p0 = int(kv_len[b]) - S
            cache["k"][b, :, p0:p0 + S, :] = kn[b].transpose(1, 0, 2)
            cache["v"][b, :, p0:p0 + S, :] = vn[b].transpose(1, 0, 2)
        kv, vv = cache["k"].transpose(0, 2, 1, 3), cache["v"].transpose(0, 2, 1, 3)   # [B,Smax,H,Dh] views
    else:
        kv, vv = _heads(qkv, B, S, H, Dh, 1), _heads(qkv, B, S, H, Dh, 2)
    mask = shape.mask
    # ---- attention
    if attn_i8:
        attn = O.int8_attn(qv, kv, vv, qk_scale=float(w["qk_scale"]), p_scale=float(w["S_p"]),
                           out_col_scale=w["attn_out_scale"] if o_i8 else w["attn_out_scalar"],
                           out_scale_is_scalar=not o_i8, mask=mask, kv_len=kv_len,
                           out_dt=O.I8 if o_i8 else hp)
    else:
        attn = O.hp_attn(qv, kv, vv, scale=float(w["bf16_qk_scale"]), mask=mask, kv_len=kv_len, dt=hp)
    tr["attn"] = attn
    # ---- attention output linear, then (post-LN) LN^quant of the two addends
    x_in = (xin_q, O.I8, xin_s) if q_i8 else (xin_hp, hp, None)
    if post:
        if o_i8:
            xo = O.int8_gemm(attn, w["wq_o"], b_col_scale=w["s_o_w"], bias=w["b_o"], epi=O.EPI_REQUANT, c_dt=O.I8)
            r_in = (xo, O.I8, w["S_o"])
        else:
            xo = O.hp_gemm(attn, w["wb_o"], bias=w["b_o"], dt=hp)
            r_in = (xo, hp, None)
        tr["xo"] = xo
        mid_q, mid_s, mid_hp = O.ln_quant(x_in[0], x_in[1], x_in[2], r_in[0], r_in[1], r_in[2], w["ln1_g"], w["ln1_b"],
                                          shape.eps, y_hp_dt=None if f1_i8 else hp)
    else:
        if o_i8:
            h1 = O.int8_gemm(attn, w["wq_o"], b_col_scale=w["s_o_w"], bias=w["b_o"], residual=h, res_dt=hp,
                             epi=O.EPI_DEQUANT, c_dt=hp)
        else:
            h1 = O.hp_gemm(attn, w["wb_o"], bias=w["b_o"], residual=h, dt=hp)
        tr["h1"] = h1
        mid_q, mid_s, mid_hp = O.ln_quant(h1, hp, None, None, 0, None, w["ln2_g"], w["ln2_b"], shape.eps,
                                          y_hp_dt=None if f1_i8 else hp)
    tr["mid_q"], tr["mid_s"], tr["mid_hp"] = mid_q, mid_s, mid_hp
    # ---- FC1 + GELU (GELU^quant when FC2 is INT8)
    if f1_i8:
        a = O.int8_gemm(mid_q, w["wq_1"], a_row_scale=mid_s, b_col_scale=w["s_1"], bias=w["b_1"],
                        epi=O.EPI_GELU_REQUANT if f2_i8 else O.EPI_DEQUANT_GELU,
                        out_col_scale=w["S_a"] if f2_i8 else None, c_dt=O.I8 if f2_i8 else hp)
    else:
        a = O.hp_gemm(mid_hp, w["wb_1"], bias=w["b_1"], gelu=True, dt=hp)
    tr["a"] = a
    # ---- FC2 and the closing LN^quant (post-LN) or residual add (pre-LN)
    if post:
        if f2_i8:
            x2 = O.int8_gemm(a, w["wq_2"], b_col_scale=w["s_2_w"], bias=w["b_2"], epi=O.EPI_REQUANT, c_dt=O.I8)
            r2 = (x2, O.I8, w["S_x2"])
        else:
            x2 = O.hp_gemm(a, w["wb_2"], bias=w["b_2"], dt=hp)
            r2 = (x2, hp, None)
        m_in = (mid_q, O.I8, mid_s) if f1_i8 else (mid_hp, hp, None)
        out_q, out_s, out_hp = O.ln_quant(m_in[0], m_in[1], m_in[2], r2[0], r2[1], r2[2], w["ln2_g"], w["ln2_b"],
                                          shape.eps, y_hp_dt=hp)
        tr["x2"] = x2
        tr["out_q"], tr["out_s"], tr["out_hp"] = out_q, out_s, out_hp
        return out_q, out_s
    if f2_i8:
        h2 = O.int8_gemm(a, w["wq_2"], b_col_scale=w["s_2_w"], bias=w["b_2"], residual=h1, res_dt=hp,
                         epi=O.EPI_DEQUANT, c_dt=hp)
    else:
        h2 = O.hp_gemm(a, w["wb_2"], bias=w["b_2"], residual=h1, dt=hp)
    tr["h2"] = h2
    return h2


def layer_fwd_fp8(w, shape, B, S, *, x_q=None, x_s=None, h=None, kv_len=None, cache=None, trace=None):
    """The same layer with E4M3 as the 8-bit format of every module (Sec. 2.1: the method works for FP8 as for
    INT8): the dataflow, scale granularities (TWQ / FWQ / SQ) and folds of layer_fwd, with the FP8 operators.
    POST_LN: (x_q uint8 E4M3 [T,d], x_s f32 [T]) -> (out_q, out_s); PRE_LN: h (bf16 bit patterns) -> new h.
    ``cache`` holds E4M3 bytes [B,H,Smax,Dh]."""
    d, H, Dh = shape.d, shape.H, shape.Dh
    tr = trace if trace is not None else {}
    post = shape.arch == POST_LN
    sp = float(w["S_p"])
    if post:
        xin_q, xin_s = x_q, x_s
    else:
        xin_q, xin_s, _ = O.ln_quant(h, O.BF16, None, None, 0, None, w["ln1_g"], w["ln1_b"], shape.eps, fp8=True)
    tr["xin_q"], tr["xin_s"] = xin_q, xin_s
    qkv = O.fp8_gemm(xin_q, w["wq_qkv"], a_row_scale=xin_s, b_col_scale=w["s_qkv"], bias=w["b_qkv"],
                     epi=O.EPI_REQUANT, c_dt=O.F8)
    tr["qkv"] = qkv
    qv = _heads(qkv, B, S, H, Dh, 0)
    if cache is not None:
        kn, vn = _heads(qkv, B, S, H, Dh, 1), _heads(qkv, B, S, H, Dh, 2)
        for b in range(B):
            p0 = int(kv_len[b]) - S
            cache["k"][b, :, p0:p0 + S, :] = kn[b].transpose(1, 0, 2)
            cache["v"][b, :, p0:p0 + S, :] = vn[b].transpose(1, 0, 2)
        kv, vv = cache["k"].transpose(0, 2, 1, 3), cache["v"].transpose(0, 2, 1, 3)
    else:
        kv, vv = _heads(qkv, B, S, H, Dh, 1), _heads(qkv, B, S, H, Dh, 2)
    attn = O.fp8_attn(qv, kv, vv, qk_scale=float(w["qk_scale"]), p_scale=sp, out_col_scale=w["attn_out_scale"],
                      mask=shape.mask, kv_len=kv_len, out_dt=O.F8)
    tr["attn"] = attn
    if post:
        xo = O.fp8_gemm(attn, w["wq_o"], b_col_scale=w["s_o_w"], bias=w["b_o"], epi=O.EPI_REQUANT, c_dt=O.F8)
        tr["xo"] = xo
        mid_q, mid_s, _ = O.ln_quant(xin_q, O.F8, xin_s, xo, O.F8, w["S_o"], w["ln1_g"], w["ln1_b"], shape.eps, fp8=True)
    else:
        h1 = O.fp8_gemm(attn, w["wq_o"], b_col_scale=w["s_o_w"], bias=w["b_o"], residual=h, res_dt=O.BF16,
                        epi=O.EPI_DEQUANT, c_dt=O.BF16)
        tr["h1"] = h1
        mid_q, mid_s, _ = O.ln_quant(h1, O.BF16, None, None, 0, None, w["ln2_g"], w["ln2_b"], shape.eps, fp8=True)
    tr["mid_q"], tr["mid_s"] = mid_q, mid_s
    a = O.fp8_gemm(mid_q, w["wq_1"], a_row_scale=mid_s, b_col_scale=w["s_1"], bias=w["b_1"],
                   epi=O.EPI_GELU_REQUANT, out_col_scale=w["S_a"], c_dt=O.F8)
    tr["a"] = a
    if post:
        x2 = O.fp8_gemm(a, w["wq_2"], b_col_scale=w["s_2_w"], bias=w["b_2"], epi=O.EPI_REQUANT, c_dt=O.F8)
        tr["x2"] = x2
        out_q, out_s, _ = O.ln_quant(mid_q, O.F8, mid_s, x2, O.F8, w["S_x2"], w["ln2_g"], w["ln2_b"], shape.eps, fp8=True)
        tr["out_q"], tr["out_s"] = out_q, out_s
        return out_q, out_s
    h2 = O.fp8_gemm(a, w["wq_2"], b_col_scale=w["s_2_w"], bias=w["b_2"], residual=h1, res_dt=O.BF16,
                    epi=O.EPI_DEQUANT, c_dt=O.BF16)
    tr["h2"] = h2
    return h2
