"""Offline preparation of a layer's parameters for libhero (host-side tool, not on the hot
path): calibrate the static scales with a forward pass of the unquantized layer, fold
them into the weights, quantize the weights column-wise.

Paper: Sec. 2.1 (column-wise weight quantization W = W_int8 Diag(S_w); FWQ / SQ scales are
calibrated in a pre-processing phase), Sec. 2.2.2 (W~_q = W_q / S_q, d~ = S_q S_k / sqrt(d),
W~_o = S_attn W_o / S_o), Sec. 2.2.3 (W~_2 = S_a W_2 / S_x2), Sec. 3 (calibration is a
forward pass recording min/max, no truncation).

The unquantized reference forward is plain torch fp64 on the GPU; the calibration statistic
(column maxima) and the fold + column-wise weight quantization run in the library's own load-time
operators (hero_absmax_cols, hero_weight_fold_quant[_fp8]) -- there is one route, and it needs the
loaded library.  Produces the tensors `hero_layer_weights` points to.  The hot path never calls it.
"""
from __future__ import annotations

import math

import torch

from . import binding as HB


def _ln(x, g, b, eps):
    return torch.nn.functional.layer_norm(x, (x.shape[-1],), g, b, eps)


def _attention(q, k, v, B, S, H, Dh, mask, kv_len):
    q, k, v = (t.view(B, S, H, Dh).permute(0, 2, 1, 3) for t in (q, k, v))
    a = (q @ k.transpose(-1, -2)) / math.sqrt(Dh)
    idx = torch.arange(S, device=q.device)
    vis = torch.ones((B, 1, S, S), dtype=torch.bool, device=q.device)
    if kv_len is not None:
        vis = vis & (idx[None, None, None, :] < kv_len.view(B, 1, 1, 1))
    if mask == HB.MASK_CAUSAL:
        L = kv_len.view(B, 1, 1, 1) if kv_len is not None else S
        vis = vis & (idx[None, None, None, :] <= idx[None, None, :, None] + (L - S))
    a = a.masked_fill(~vis, float("-inf"))
    p = torch.softmax(a, dim=-1)
    p = torch.nan_to_num(p, nan=0.0)                      # rows that see no key
    return (p @ v).permute(0, 2, 1, 3).reshape(B * S, H * Dh)


def reference_layer(p, x, arch, H, Dh, eps, mask, B, S, kv_len=None):
    """Unquantized layer forward (fp64 on the given device); returns the intermediates
    whose ranges the static scales are calibrated on, and the layer output."""
    P = {k: v.double() for k, v in p.items()}
    x = x.double()
    d = x.shape[1]
    xin = _ln(x, P["ln1_g"], P["ln1_b"], eps) if arch == HB.ARCH_PRE_LN else x
    qkv = xin @ P["w_qkv"] + P["b_qkv"]
    t = {"q": qkv[:, :d], "k": qkv[:, d:2 * d], "v": qkv[:, 2 * d:]}
    t["attn"] = _attention(t["q"], t["k"], t["v"], B, S, H, Dh, mask, kv_len)
    t["o"] = t["attn"] @ P["w_o"] + P["b_o"]
    if arch == HB.ARCH_POST_LN:
        mid = _ln(x + t["o"], P["ln1_g"], P["ln1_b"], eps)
        x1 = mid @ P["w_1"] + P["b_1"]
    else:
        mid = x + t["o"]
        x1 = _ln(mid, P["ln2_g"], P["ln2_b"], eps) @ P["w_1"] + P["b_1"]
    t["a"] = torch.nn.functional.gelu(x1)
    t["x2"] = t["a"] @ P["w_2"] + P["b_2"]
    t["out"] = _ln(mid + t["x2"], P["ln2_g"], P["ln2_b"], eps) if arch == HB.ARCH_POST_LN else mid + t["x2"]
    return t


def calibrate(p, x_calib, arch, H, Dh, eps, mask, B, S, kv_len=None, *, hero, fp8=False):
    """Static scales: SQ scalars for X_q, X_k, X_v; FWQ vectors for X_attn, X_o, A, X_2.  The column maxima
    come from hero_absmax_cols of the loaded library `hero` (a maximum is exact in any precision).
    fp8: the FP8 variant (Sec. 2.1): ranges are mapped to the largest E4M3 value 448, S_p = 1/448."""
    t = reference_layer(p, x_calib, arch, H, Dh, eps, mask, B, S, kv_len)
    qmax = 448.0 if fp8 else 127.0

    def scale(a, dim=None):
        m = hero.hero_absmax_cols(a.float().contiguous()).double()
        m = m.amax() if dim is None else m
        m = torch.where(m == 0, torch.full_like(m, qmax), m)
        return (m / qmax).float()
    sc = {"S_q": scale(t["q"]), "S_k": scale(t["k"]), "S_v": scale(t["v"]),
          "S_attn": scale(t["attn"], 0), "S_o": scale(t["o"], 0), "S_a": scale(t["a"], 0),
          "S_x2": scale(t["x2"], 0),
          "S_p": torch.tensor(1.0 / 448.0 if fp8 else 1.0 / 255.0, dtype=torch.float32, device=x_calib.device)}
    return sc, t["out"]


def check_mode(mode):
    """The subsets of the per-module switch the layer driver runs (Sec. 2.3): a module can be 8-bit only when the
    module that produces its codes is (attention needs the QKV GEMM's SQ codes, the attention-output linear the
    attention's FWQ codes, FC2 the GELU^quant codes of FC1)."""
    m = mode & ~(HB.M_FP8 | HB.M_F16)
    if (m & HB.M_ATTN and not m & HB.M_QKV) or (m & HB.M_ATTN_OUT and not m & HB.M_ATTN) or (m & HB.M_FC2 and not m & HB.M_FC1):
        raise ValueError("this subset of the switch needs a stand-alone quantization kernel, which the method removes")
    if mode & HB.M_FP8 and (m != HB.MODE_M3 or mode & HB.M_F16):
        raise ValueError("the FP8 variant runs every module in 8 bits")


def prepare(p, sc, arch, d, Dh, mode=HB.MODE_M3, *, hero, fp8=False):
    """Fold the static scales into the weights and quantize.  Returns (tensors, qk_scale,
    p_scale): `tensors` is keyed by the field names of hero_layer_weights.  The fold + column-wise
    quantization runs in hero_weight_fold_quant of the loaded library `hero`, on the weights' device.
    mode: any admissible subset of the module bits (Table 1's rows, the all-16-bit layer MODE_M0 and what lies
    between); a 16-bit module gets its unfolded weight, transposed to [N][K], in BF16 or (HB.M_F16) FP16.
    fp8 (mode M3, scales from calibrate(fp8=True)): E4M3 weights for a layer run with M_FP8."""
    check_mode(mode | (HB.M_FP8 if fp8 else 0))
    P = {k: v.double() for k, v in p.items()}
    post = arch == HB.ARCH_POST_LN
    hp = torch.float16 if mode & HB.M_F16 else torch.bfloat16
    t = {}
    f32 = lambda a: None if a is None else a.float().contiguous()
    as_hp = lambda name: P[name].t().contiguous().to(hp)             # [in][out] -> [N][K], one rounding from fp64

    def quantize_folded(name, rm, cd):
        return hero.hero_weight_fold_quant(p[name].float().contiguous(), f32(rm), f32(cd), fp8=fp8)
    if mode & HB.M_ATTN:
        div = torch.cat([sc["S_q"].double().expand(d), sc["S_k"].double().expand(d), sc["S_v"].double().expand(d)])
        qk_scale = float(sc["S_q"].double() * sc["S_k"].double() / math.sqrt(Dh))
    else:
        div = torch.ones(3 * d, dtype=torch.float64, device=P["w_qkv"].device)
        qk_scale = 1.0 / math.sqrt(Dh)
    if mode & HB.M_QKV:
        t["w_qkv"], t["w_qkv_s"] = quantize_folded("w_qkv", None, div if mode & HB.M_ATTN else None)
    else:
        t["w_qkv_hp"] = as_hp("w_qkv")
    t["b_qkv"] = (P["b_qkv"] / div).float()
    pv = sc["S_p"].double() * sc["S_v"].double()
    if mode & HB.M_ATTN_OUT:
        t["attn_out_scale"] = (pv / sc["S_attn"].double()).float()
        bo = P["b_o"] / sc["S_o"].double() if post else P["b_o"]
        t["w_o"], t["w_o_s"] = quantize_folded("w_o", sc["S_attn"], sc["S_o"] if post else None)
        t["b_o"] = bo.float()
    else:
        t["attn_out_scale"] = pv.float().reshape(1)
        t["w_o_bf16"] = as_hp("w_o")
        t["b_o"] = P["b_o"].float()
    if mode & HB.M_FC1:
        t["w_1"], t["w_1_s"] = quantize_folded("w_1", None, None)
    else:
        t["w_1_hp"] = as_hp("w_1")
    t["b_1"] = P["b_1"].float()
    if mode & HB.M_FC2:
        b2 = P["b_2"] / sc["S_x2"].double() if post else P["b_2"]
        t["w_2"], t["w_2_s"] = quantize_folded("w_2", sc["S_a"], sc["S_x2"] if post else None)
        t["b_2"] = b2.float()
    else:
        t["w_2_bf16"] = as_hp("w_2")
        t["b_2"] = P["b_2"].float()
    for k in ("S_o", "S_x2", "S_a"):
        t[k] = sc[k].float().contiguous()
    for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b"):
        t[k] = p[k].float().contiguous()
    return t, qk_scale, float(sc["S_p"])
