"""End-to-end parity of hero_layer_fwd against the oracle's layer chain at the REAL widths of the five
workloads (the per-kernel tests and the 256-wide layers of test_gpu_layer.py do not reach these code paths
together): BERT-base in full, one GPT prefill layer on one 512-token sequence, GPT decode steps against a
2048-key INT8 cache (the split-K linear included), BERT-large through all 24 layers, and BERT-large in the
mixed mode M1 at width 1024.  Slices are the ones the oracle finishes in seconds to a minute.

Thresholds are set from the values measured on MI355X (printed by every test; the numbers and their margins are
listed in the design document), not from the generic 2e-2 / 97 % defaults."""
import json
import os

import numpy as np
import pytest
import torch

import oracle as O
from oracle import layer as OL
from paper_2310_17723_amd import binding as HB
from paper_2310_17723_amd import synth
from parity import dev, rel_err, to_np, upload_weights

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _record(name, obj):
    """Measured parity figures go to stdout and, when the scratch folder exists, to a JSON file beside the logs."""
    print(f"[parity] {name}: {json.dumps(obj)}", flush=True)
    out = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out):
        with open(os.path.join(out, f"parity_{name}.json"), "w") as f:
            json.dump(obj, f, indent=1)


def _calib_input(seed, shape, tokens):
    hc = synth.activations(seed, shape, tokens, stream=1).astype(np.float64)
    if shape.arch == synth.POST_LN:
        emb = synth.embedding_ln_params(seed, shape)
        hc = OL._ln64(hc, emb["g"].astype(np.float64), emb["b"].astype(np.float64), shape.eps)
    return hc


def _prepare_stack(seed, shape, mode, layers, Bc, Sc):
    """Oracle-prepared weights of `layers` layers: static scales calibrated on Bc x Sc tokens pushed through the
    unquantized fp64 stack layer by layer (the padding mask is dropped for calibration)."""
    cal = synth.small(shape, mask=synth.MASK_NONE if shape.mask == synth.MASK_PADDING else shape.mask)
    xc = _calib_input(seed, shape, Bc * Sc)
    ws = []
    for l in range(layers):
        p = synth.layer_params(seed, shape, l)
        sc, xc = OL.calibrate(p, xc, cal, Bc, Sc)
        ws.append(OL.prepare(p, sc, shape, mode))
    return ws


def _post_ln_input(seed, shape, T):
    emb = synth.embedding_ln_params(seed, shape)
    xq, xs, _ = O.ln_quant(synth.activations(seed, shape, T), O.F32, None, None, 0, None, emb["g"], emb["b"], shape.eps)
    return xq, xs


def _code_stats(gq, gs, oq, os_, valid=None):
    if valid is not None:
        gq, gs, oq, os_ = gq[valid], gs[valid], oq[valid], os_[valid]
    d = np.abs(gq.astype(np.int32) - oq.astype(np.int32))
    ref = oq.astype(np.float32) * os_[:, None]
    got = gq.astype(np.float32) * gs[:, None]
    return {"identical": float(np.mean(d == 0)), "max_code_diff": int(d.max()),
            "scale_rel": float(np.max(np.abs(gs - os_) / os_)), "rel_err": rel_err(got, ref)}


def _run_post_ln(hero, desc, W, B, S, xq, xs, kv_len, ws):
    T = B * S
    out_q = torch.empty((T, xq.shape[1]), dtype=torch.int8, device="cuda")
    out_s = torch.empty((T,), dtype=torch.float32, device="cuda")
    hero.hero_layer_fwd(desc, W, B, S, ws, x_q=xq, x_scale=xs, out_q=out_q, out_scale=out_s, kv_len=kv_len)
    return out_q, out_s


def test_config0_bert_base_layer_full(hero):
    """Config 0 in full: 1 x 128 tokens, d 768 (the padded-row LN^quant path: 768 is not a multiple of 512),
    12 x 64 heads, f 3072, eps 1e-12, no mask, every module INT8."""
    shape = synth.CONFIGS[0]
    B, S, T = shape.B, shape.S, shape.B * shape.S
    (w,) = _prepare_stack(2310, shape, OL.MODE_M3, 1, 2, 128)
    xq, xs = _post_ln_input(2310, shape, T)
    tr = {}
    oq, os_ = OL.layer_fwd(w, shape, B, S, x_q=xq, x_s=xs, trace=tr)
    desc = hero.layer_desc(shape.arch, shape.d, shape.H, shape.Dh, shape.f, shape.eps, shape.mask, HB.MODE_M3)
    W, keep = upload_weights(hero, w)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, S), dtype=torch.uint8, device="cuda")
    out_q, out_s = _run_post_ln(hero, desc, W, B, S, dev(xq), dev(xs), None, ws)
    st = _code_stats(to_np(out_q), to_np(out_s), oq, os_)
    _record("config0_bert_base", st)
    # measured on MI355X: every code identical, scales equal to 2e-7; the margin allows a handful of +-1 LSB
    # flips of the LayerNorm / GELU / softmax stages (their class) and what they do to a row scale
    assert st["max_code_diff"] <= 1 and st["identical"] >= 0.999 and st["scale_rel"] <= 1e-3


def _stage_codes(name, got, ref, max_frac):
    d = np.abs(to_np(got).astype(np.int32) - ref.astype(np.int32))
    assert d.max() <= 1 and np.mean(d != 0) <= max_frac, (name, int(d.max()), float(np.mean(d != 0)))
    return float(np.mean(d != 0))


def test_config3_gpt_prefill_layer_one_sequence(hero):
    """Config 3, one sequence of 512 tokens through one layer at the real width: d 4096, 32 x 128 heads,
    f 16384, pre-LN, causal; K = 4096 and K = 16384 GEMMs with the in-place bf16 residual.
    (1) Every stage on the ORACLE's input (its trace): the integer stages bit for bit, the LayerNorm / GELU
    stages in their +-1 LSB class.  (2) The layer driver end to end.  The layer is not a continuous function
    of its input at the level of one code: a flipped LN^quant code (8e-6 of them flip) moves ~15 % of that
    token's SQ codes of Q, K, V, one V step is up to S_v / S_attn[j] ~ 7 steps of an attention output channel,
    and so on; at the end 57 % of the bf16 outputs sit on the neighbouring bf16 value (relative L2 1.6e-3, the
    size of the bf16 rounding itself).  Hence the end-to-end bar is the 16-bit output class (2e-2) plus an L2
    bound, and the sharp comparison is (1)."""
    shape = synth.small(synth.CONFIGS[3], B=1, S=512)
    B, S, T = shape.B, shape.S, shape.B * shape.S
    d, H, Dh = shape.d, shape.H, shape.Dh
    (w,) = _prepare_stack(2311, shape, OL.MODE_M3, 1, 1, 128)
    hb = O.f32_to_bf16(synth.activations(2311, shape, T))
    tr = {}
    ref = OL.layer_fwd(w, shape, B, S, h=hb, trace=tr)
    D = {k: dev(v) for k, v in w.items() if isinstance(v, np.ndarray)}
    st = {}
    # ---- (1) stage by stage on the oracle's intermediates
    q, s, _ = hero.hero_ln_quant(dev(hb), None, None, None, D["ln1_g"], D["ln1_b"], shape.eps)
    st["ln1_flips"] = _stage_codes("ln1", q, tr["xin_q"], 1e-4)                     # measured 8e-6
    assert np.allclose(to_np(s), tr["xin_s"], rtol=1e-6)
    qkv = hero.hero_int8_gemm(dev(tr["xin_q"]), D["wq_qkv"], dev(tr["xin_s"]), D["s_qkv"], D["b_qkv"],
                              epi=HB.EPI_REQUANT, out_dtype=torch.int8)
    assert np.array_equal(to_np(qkv), tr["qkv"])
    dq = dev(tr["qkv"]).view(B, S, 3, H, Dh)
    at = hero.hero_int8_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], float(w["qk_scale"]), float(w["S_p"]),
                             D["attn_out_scale"], mask=shape.mask)
    st["attn_flips"] = _stage_codes("attn", at, tr["attn"], 1e-3)                   # measured 0
    h1 = hero.hero_int8_gemm(dev(tr["attn"]), D["wq_o"], None, D["s_o_w"], D["b_o"], residual=dev(hb),
                             epi=HB.EPI_DEQUANT, out_dtype=torch.bfloat16)
    assert np.array_equal(to_np(h1), tr["h1"])
    q2, s2, _ = hero.hero_ln_quant(dev(tr["h1"]), None, None, None, D["ln2_g"], D["ln2_b"], shape.eps)
    st["ln2_flips"] = _stage_codes("ln2", q2, tr["mid_q"], 1e-4)                    # measured 7e-6
    a = hero.hero_int8_gemm(dev(tr["mid_q"]), D["wq_1"], dev(tr["mid_s"]), D["s_1"], D["b_1"],
                            epi=HB.EPI_GELU_REQUANT, out_col_scale=D["S_a"], out_dtype=torch.int8)
    st["gelu_flips"] = _stage_codes("fc1", a, tr["a"], 1e-4)                        # measured 4e-6
    h2 = hero.hero_int8_gemm(dev(tr["a"]), D["wq_2"], None, D["s_2_w"], D["b_2"], residual=dev(tr["h1"]),
                             epi=HB.EPI_DEQUANT, out_dtype=torch.bfloat16)
    assert np.array_equal(to_np(h2), tr["h2"])
    # ---- (2) the layer driver
    desc = hero.layer_desc(shape.arch, d, H, Dh, shape.f, shape.eps, shape.mask, HB.MODE_M3)
    W, keep = upload_weights(hero, w)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, S), dtype=torch.uint8, device="cuda")
    h = dev(hb)
    hero.hero_layer_fwd(desc, W, B, S, ws, h=h)
    got, want = O.bf16_to_f32(to_np(h)), O.bf16_to_f32(ref)
    st.update({"rel_err": rel_err(got, want), "identical_bf16": float(np.mean(to_np(h) == ref)),
               "rel_l2": float(np.sqrt(((got.astype(np.float64) - want) ** 2).sum() / (want.astype(np.float64) ** 2).sum()))})
    _record("config3_gpt_prefill", st)
    # measured: rel_err 1.29e-2, relative L2 1.6e-3
    assert st["rel_err"] <= 2e-2 and st["rel_l2"] <= 4e-3


def test_config4_gpt_decode_steps_against_2048_key_cache(hero):
    """Config 4, two batch rows, four one-token steps at d 4096 against a 2048-key INT8 cache: kv_append, the
    cache-streaming one-query attention, the four-K-group skinny GEMMs and the split-K FC2 in one chain."""
    base = synth.CONFIGS[4]
    shape = synth.small(base, B=2)
    B, d, H, Dh, f = shape.B, shape.d, shape.H, shape.Dh, shape.f
    steps, L0 = 4, base.cache_len
    Smax = L0 + steps
    cal = synth.small(shape, mask=synth.MASK_CAUSAL, S=128)
    p = synth.layer_params(2312, shape, 0)
    sc, _ = OL.calibrate(p, _calib_input(2312, shape, 128), cal, 1, 128)
    w = OL.prepare(p, sc, shape, OL.MODE_M3)
    # the split-K path is what this layer's FC2 takes: a scratch size is reported for its shape and is part
    # of the layer workspace
    assert hero.hero_int8_gemm_workspace_bytes(B, d, f) > 0
    desc = hero.layer_desc(shape.arch, d, H, Dh, f, shape.eps, shape.mask, HB.MODE_M3)
    act_bytes = B * (d + 4 + 3 * d + d + d + 4 + f)
    assert hero.hero_layer_workspace_bytes(desc, B, 1) >= act_bytes + hero.hero_int8_gemm_workspace_bytes(B, d, f)
    cache = {"k": synth.int8_codes(2312, (B, H, Smax, Dh), 0), "v": synth.int8_codes(2312, (B, H, Smax, Dh), 1)}
    W, keep = upload_weights(hero, w)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, 1), dtype=torch.uint8, device="cuda")
    kc, vc = dev(cache["k"]), dev(cache["v"])
    kv = np.full(B, L0, np.int32)
    worst = {"rel_err": 0.0, "rel_l2": 0.0, "cache_identical": 1.0}
    for step in range(steps):
        hb = O.f32_to_bf16(synth.activations(2312, shape, B, stream=10 + step))
        kv = kv + 1
        ref = OL.layer_fwd(w, shape, B, 1, h=hb, kv_len=kv, cache=cache)
        h = dev(hb)
        hero.hero_layer_fwd(desc, W, B, 1, ws, h=h, kv_len=dev(kv), k_cache=kc, v_cache=vc)
        got, want = O.bf16_to_f32(to_np(h)), O.bf16_to_f32(ref)
        worst["rel_err"] = max(worst["rel_err"], rel_err(got, want))
        worst["rel_l2"] = max(worst["rel_l2"], float(np.sqrt(((got.astype(np.float64) - want) ** 2).sum() / (want.astype(np.float64) ** 2).sum())))
    # the rows appended by the four steps
    gk, gv = to_np(kc)[:, :, L0:], to_np(vc)[:, :, L0:]
    worst["cache_identical"] = float(min(np.mean(gk == cache["k"][:, :, L0:]), np.mean(gv == cache["v"][:, :, L0:])))
    worst["cache_max_diff"] = int(max(np.abs(gk.astype(int) - cache["k"][:, :, L0:].astype(int)).max(),
                                      np.abs(gv.astype(int) - cache["v"][:, :, L0:].astype(int)).max()))
    _record("config4_gpt_decode", worst)
    # measured: rel_err 5.1e-3, relative L2 1.2e-3 (the size of the bf16 rounding: see the config 3 test), appended
    # cache rows identical
    assert worst["rel_err"] <= 2e-2 and worst["rel_l2"] <= 3e-3
    assert worst["cache_max_diff"] <= 1 and worst["cache_identical"] >= 0.999
    assert np.array_equal(to_np(kc)[:, :, :L0], cache["k"][:, :, :L0])        # the old rows are untouched


def _snr_db(x, ref):
    e = np.asarray(x, np.float64) - ref
    return float(10.0 * np.log10((ref * ref).sum() / max((e * e).sum(), 1e-300)))


def test_config2_bert_large_24_layers(hero):
    """Config 2, one sequence of 512 tokens through all 24 layers in M3 (padding mask, 400 real tokens).
    Three views.  (1) Teacher-forced: every layer runs on the ORACLE's input, which gives each layer's own
    parity at depth (tight).  (2) Free-running: each side feeds its own output forward.  The quantized layer is
    a discontinuous function of its input (a +-1 LSB flip of one LN^quant code moves ~15 % of that token's SQ
    codes of Q, K, V; see the config 3 test), so the two chains separate code by code within a few layers;
    the per-layer fraction of identical codes and the largest code difference are recorded.  (3) What a user of
    the method cares about: both chains are EQUALLY good evaluations of the unquantized model -- their
    signal-to-noise ratios against the fp64 stack agree at every depth."""
    shape = synth.small(synth.CONFIGS[2], B=1)
    B, S, T, L = shape.B, shape.S, shape.B * shape.S, synth.CONFIGS[2].layers
    ws_o = _prepare_stack(2313, shape, OL.MODE_M3, L, 2, 128)
    xq, xs = _post_ln_input(2313, shape, T)
    kv_len = np.array([400], np.int32)
    valid = (np.arange(S)[None, :] < kv_len[:, None]).ravel()
    vmask = torch.from_numpy(~valid).cuda()
    desc = hero.layer_desc(shape.arch, shape.d, shape.H, shape.Dh, shape.f, shape.eps, shape.mask, HB.MODE_M3)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, S), dtype=torch.uint8, device="cuda")
    dkv = dev(kv_len)
    emb = synth.embedding_ln_params(2313, shape)
    x64 = OL._ln64(synth.activations(2313, shape, T).astype(np.float64), emb["g"].astype(np.float64),
                   emb["b"].astype(np.float64), shape.eps)
    oq, os_ = xq, xs
    gq, gs = dev(xq), dev(xs)
    forced, free = [], []
    for l in range(L):
        W, keep = upload_weights(hero, ws_o[l])
        fq, fs = _run_post_ln(hero, desc, W, B, S, dev(oq), dev(os_), dkv, ws)        # teacher-forced
        gq, gs = _run_post_ln(hero, desc, W, B, S, gq, gs, dkv, ws)                    # free-running
        oq, os_ = OL.layer_fwd(ws_o[l], shape, B, S, x_q=oq, x_s=os_, kv_len=kv_len)
        x64 = OL.fp64_layer(synth.layer_params(2313, shape, l), x64, shape, B, S, kv_len)["out"]
        forced.append(_code_stats(to_np(fq), to_np(fs), oq, os_, valid))
        st = _code_stats(to_np(gq), to_np(gs), oq, os_, valid)
        deq_o = oq[valid].astype(np.float64) * os_[valid, None]
        deq_g = to_np(gq)[valid].astype(np.float64) * to_np(gs)[valid, None].astype(np.float64)
        st.update({"snr_oracle_db": _snr_db(deq_o, x64[valid]), "snr_gpu_db": _snr_db(deq_g, x64[valid]),
                   "snr_gpu_vs_oracle_db": _snr_db(deq_g, deq_o)})
        free.append(st)
        # padded rows carry no meaning (the mask hides them as keys) and differ freely: the free-running chain
        # takes the oracle's values there so that only real tokens are compared
        gq = gq.clone(); gs = gs.clone()
        gq[vmask] = dev(oq)[vmask]
        gs[vmask] = dev(os_)[vmask]
        del W, keep
    _record("config2_depth24", {"teacher_forced": forced, "free_running": free})
    # (1) measured over the 24 layers: identical 0.99924 .. 0.99999, max code difference 1 (2 in two layers),
    # row scales within 2.6e-3
    for l, st in enumerate(forced):
        assert st["max_code_diff"] <= 3 and st["identical"] >= 0.998 and st["scale_rel"] <= 6e-3, (l, st)
    # (2) on record, not a bar: identical codes 0.9999 -> 0.96 -> 0.84 -> 0.67 -> 0.50 -> ... -> 0.14-0.19 from layer
    # 10 on, largest code difference 26 (rows whose scale is set by a x20 outlier channel).
    # (3) the bar.  Measured: SNR against the fp64 stack 22.7 dB after layer 0 falling to 13.5 dB after layer 23,
    # the SAME for both chains to 0.04 dB at every depth; GPU chain against oracle chain >= 19.9 dB, i.e. the two
    # are 4-9 dB closer to each other than either is to the unquantized model
    for l, st in enumerate(free):
        assert abs(st["snr_gpu_db"] - st["snr_oracle_db"]) <= 0.25, (l, st)
        assert st["snr_gpu_vs_oracle_db"] >= st["snr_oracle_db"] + 3.0, (l, st)


def test_config2_bert_large_layer_mixed_mode_m1(hero):
    """Config 2's second mode at the real width: attention core, attention-output linear and FC2 in BF16
    (Table 1, M1), QKV and FC1 INT8 with 16-bit outputs; one layer, two sequences."""
    shape = synth.small(synth.CONFIGS[2], B=2)
    B, S, T = shape.B, shape.S, shape.B * shape.S
    (w,) = _prepare_stack(2314, shape, OL.MODE_M1, 1, 2, 128)
    xq, xs = _post_ln_input(2314, shape, T)
    kv_len = synth.kv_lengths(2314, shape)
    oq, os_ = OL.layer_fwd(w, shape, B, S, x_q=xq, x_s=xs, kv_len=kv_len)
    desc = hero.layer_desc(shape.arch, shape.d, shape.H, shape.Dh, shape.f, shape.eps, shape.mask, HB.MODE_M1)
    W, keep = upload_weights(hero, w)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, S), dtype=torch.uint8, device="cuda")
    out_q, out_s = _run_post_ln(hero, desc, W, B, S, dev(xq), dev(xs), dev(kv_len), ws)
    valid = (np.arange(S)[None, :] < kv_len[:, None]).ravel()
    st = _code_stats(to_np(out_q), to_np(out_s), oq, os_, valid)
    _record("config2_m1_width1024", st)
    # the bf16 GEMMs (K = 1024 and 4096) accumulate in fp32 in another order than the oracle's fp64 sums and the
    # attention core runs on bf16 probabilities, so more values cross a rounding boundary than in M3 --
    # measured: identical 0.9925, max code difference 2, scale rel 6.0e-3
    assert st["max_code_diff"] <= 3 and st["identical"] >= 0.985 and st["scale_rel"] <= 1.5e-2
