"""GPU parity: each HIP entry point against the CPU oracle, element by element, on the
same seeded inputs, at sizes that span several tiles and a ragged tail.  All calls go
through the C ABI (ctypes binding)."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import layer as OL
from paper_2310_17723_amd import binding as HB
from paper_2310_17723_amd import synth
from parity import (assert_codes, assert_exact, assert_fp8_attn_codes, assert_fp8_attn_values, assert_fp8_codes, assert_scales, dev,
                    fp8_attn_flip_bound, rel_err, to_np)

pytestmark = pytest.mark.gpu


# ============================================================ LN^quant
def _ln_inputs(seed, M, D):
    g = synth.rng(seed)
    xq = g.integers(-127, 128, (M, D), dtype=np.int8)
    rq = g.integers(-127, 128, (M, D), dtype=np.int8)
    xs = g.uniform(0.005, 0.05, M).astype(np.float32)
    rc = g.uniform(0.001, 0.02, D).astype(np.float32)
    gam = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
    bet = (0.02 * g.standard_normal(D)).astype(np.float32)
    hb = O.f32_to_bf16(synth.activations(seed, synth.small(synth.CONFIGS[3], d=D), M))
    return xq, rq, xs, rc, gam, bet, hb


@pytest.mark.parametrize("M,D", [(37, 768), (130, 1024), (67, 4096), (9, 48), (21, 8192), (300, 1536)])
def test_ln_quant_int8_pair(hero, M, D):
    """Post-LN form: TWQ INT8 input + FWQ INT8 second addend (Sec. 2.2.2 last line)."""
    xq, rq, xs, rc, gam, bet, _ = _ln_inputs(100 + D, M, D)
    rq_o, rs_o, _ = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, 1e-12)
    q, s, _ = hero.hero_ln_quant(dev(xq), dev(xs), dev(rq), dev(rc), dev(gam), dev(bet), 1e-12)
    assert_scales(to_np(s), rs_o, "y_scale")
    assert_codes(to_np(q), rq_o, "y_q")


@pytest.mark.parametrize("M,D", [(131, 4096), (40, 1024), (17, 512), (5, 16)])
def test_ln_quant_bf16_single_and_hp_copy(hero, M, D):
    """Pre-LN form: one bf16 input; also the bf16 copy of y and a bf16 second addend."""
    xq, rq, xs, rc, gam, bet, hb = _ln_inputs(200 + D, M, D)
    rq_o, rs_o, hp_o = O.ln_quant(hb, O.BF16, None, None, 0, None, gam, bet, 1e-5, y_hp_dt=O.BF16)
    q, s, hp = hero.hero_ln_quant(dev(hb), None, None, None, dev(gam), dev(bet), 1e-5, y_hp_dtype=torch.bfloat16)
    assert_scales(to_np(s), rs_o)
    assert_codes(to_np(q), rq_o, "y_q")
    assert rel_err(O.bf16_to_f32(to_np(hp)), O.bf16_to_f32(hp_o)) <= 2e-2
    # INT8 x + bf16 addend (a BF16 module feeding the LayerNorm), f16 copy of y
    rb = O.f32_to_bf16(synth.rng(3).standard_normal((M, D)).astype(np.float32))
    rq_o, rs_o, hp_o = O.ln_quant(xq, O.I8, xs, rb, O.BF16, None, gam, None, 1e-5, y_hp_dt=O.F16)
    q, s, hp = hero.hero_ln_quant(dev(xq), dev(xs), dev(rb), None, dev(gam), None, 1e-5, y_hp_dtype=torch.float16)
    assert_scales(to_np(s), rs_o)
    assert_codes(to_np(q), rq_o)
    assert rel_err(O.f16_to_f32(to_np(hp)), O.f16_to_f32(hp_o)) <= 2e-2


def test_ln_quant_pure_per_token_quant_is_bit_exact(hero):
    """gamma == NULL: no float reduction besides absmax, so scales and codes are exact."""
    M, D = 150, 1024
    _, _, _, _, _, _, hb = _ln_inputs(7, M, D)
    hb[3] = 0                                                     # an all-zero row: scale 1, codes 0
    rq_o, rs_o, _ = O.ln_quant(hb, O.BF16, None, None, 0, None, None, None, 0.0)
    q, s, _ = hero.hero_ln_quant(dev(hb), None, None, None, None, None, 0.0)
    assert_exact(to_np(s), rs_o, "scale")
    assert_exact(to_np(q), rq_o, "codes")
    assert to_np(s)[3] == 1.0 and not to_np(q)[3].any()
    hf = O.f32_to_f16(O.bf16_to_f32(hb))
    rq_o, rs_o, _ = O.ln_quant(hf, O.F16, None, None, 0, None, None, None, 0.0)
    q, s, _ = hero.hero_ln_quant(dev(hf, torch.float16), None, None, None, None, None, 0.0)
    assert_exact(to_np(s), rs_o)
    assert_exact(to_np(q), rq_o)


@pytest.mark.parametrize("M,D", [(70, 1024), (33, 4096), (200, 48), (9, 8192)])
def test_ln_quant_fp8_output(hero, M, D):
    """hero_ln_quant_fp8: token-wise E4M3 output (scale max|y| / 448).  Behind a LayerNorm the codes are in the
    tolerance class of the INT8 form (equal on all but 0.1 %, the rest adjacent E4M3 values: y itself differs in
    its last bits); without one (gamma NULL) the quotient is the IEEE one and the codes are exact.  The result
    feeds hero_fp8_gemm as A / a_row_scale."""
    xq, rq, xs, rc, gam, bet, hb = _ln_inputs(1500 + D, M, D)
    q_o, s_o, _ = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, 1e-12, fp8=True)
    q, s, _ = hero.hero_ln_quant(dev(xq), dev(xs), dev(rq), dev(rc), dev(gam), dev(bet), 1e-12, fp8=True)
    assert_scales(to_np(s), s_o, "y_scale fp8")
    assert_fp8_codes(to_np(q), q_o, O.e4m3_to_f32, "LN fp8", max_frac=max(1e-3, 2.5 / q_o.size))
    if D <= 4096:
        q_o, s_o, hp_o = O.ln_quant(hb, O.BF16, None, None, 0, None, gam, bet, 1e-5, y_hp_dt=O.BF16, fp8=True)
        q, s, hp = hero.hero_ln_quant(dev(hb), None, None, None, dev(gam), dev(bet), 1e-5, y_hp_dtype=torch.bfloat16, fp8=True)
        assert_scales(to_np(s), s_o)
        assert_fp8_codes(to_np(q), q_o, O.e4m3_to_f32, "LN fp8, bf16 input", max_frac=max(1e-3, 2.5 / q_o.size))
        assert rel_err(O.bf16_to_f32(to_np(hp)), O.bf16_to_f32(hp_o)) <= 2e-2
        # pure per-token FP8 quantization of a bf16 tensor: exact
        q_o, s_o, _ = O.ln_quant(hb, O.BF16, None, None, 0, None, None, None, 0.0, fp8=True)
        q, s, _ = hero.hero_ln_quant(dev(hb), None, None, None, None, None, 0.0, fp8=True)
        assert_exact(to_np(s), s_o, "fp8 twq scale")
        assert_exact(to_np(q), q_o, "fp8 twq codes")
        # ... and the chain LN^quant(FP8) -> FP8 GeMM^quant against the oracle's chain
        if D == 1024:
            g = synth.rng(1501)
            N = 136
            W = (g.standard_normal((N, D)) * 0.05).astype(np.float32)
            cs = (np.abs(W).max(axis=1) / 448).astype(np.float32)
            Bt = O.f32_to_e4m3((W / cs[:, None]).astype(np.float32))
            ref = O.fp8_gemm(q_o, Bt, a_row_scale=s_o, b_col_scale=cs, epi=O.EPI_DEQUANT, c_dt=O.BF16)
            got = hero.hero_fp8_gemm(q, dev(Bt), s, dev(cs), epi=HB.EPI_DEQUANT, out_dtype=torch.bfloat16)
            assert rel_err(O.bf16_to_f32(to_np(got)), O.bf16_to_f32(ref)) <= 2e-2


@pytest.mark.parametrize("M,D", [(70, 1024), (9, 8192), (200, 48)])
def test_ln_quant_e4m3_addends(hero, M, D):
    """The 8-bit addends as E4M3 codes (the FP8 layer's LN^quant(S_in X_in, X_o S_o)): same scales, same classes;
    an INT8 output from E4M3 addends is served too; INT8 and E4M3 addends in one call are refused."""
    g = synth.rng(1600 + D)
    x8 = O.f32_to_e4m3((g.standard_normal((M, D)) * 60).astype(np.float32))
    r8 = O.f32_to_e4m3((g.standard_normal((M, D)) * 60).astype(np.float32))
    _, _, xs, rc, gam, bet, _ = _ln_inputs(1601 + D, M, D)
    f8 = lambda a: dev(a).view(torch.float8_e4m3fn)
    q_o, s_o, _ = O.ln_quant(x8, O.F8, xs, r8, O.F8, rc, gam, bet, 1e-5, fp8=True)
    q, s, _ = hero.hero_ln_quant(f8(x8), dev(xs), f8(r8), dev(rc), dev(gam), dev(bet), 1e-5, fp8=True)
    assert_scales(to_np(s), s_o, "y_scale")
    assert_fp8_codes(to_np(q), q_o, O.e4m3_to_f32, "LN fp8 <- fp8", max_frac=max(1e-3, 2.5 / q_o.size))
    q_o, s_o, _ = O.ln_quant(x8, O.F8, xs, r8, O.F8, rc, gam, bet, 1e-5)
    q, s, _ = hero.hero_ln_quant(f8(x8), dev(xs), f8(r8), dev(rc), dev(gam), dev(bet), 1e-5)
    assert_scales(to_np(s), s_o, "y_scale")
    assert_codes(to_np(q), q_o, "LN int8 <- fp8", max_frac=max(1e-3, 2.5 / q_o.size))
    # no LayerNorm: the decoded, scaled codes quantized per token, exact
    q_o, s_o, _ = O.ln_quant(x8, O.F8, xs, None, 0, None, None, None, 0.0, fp8=True)
    q, s, _ = hero.hero_ln_quant(f8(x8), dev(xs), None, None, None, None, 0.0, fp8=True)
    assert_exact(to_np(s), s_o, "twq scale")
    assert_exact(to_np(q), q_o, "twq codes")
    with pytest.raises(HB.HeroError):
        hero.hero_ln_quant(f8(x8), dev(xs), dev(r8.view(np.int8)), dev(rc), dev(gam), dev(bet), 1e-5, fp8=True)


def test_ln_quant_rejects_bad_arguments(hero):
    x = torch.zeros((4, 40), dtype=torch.int8, device="cuda")
    with pytest.raises(HB.HeroError) as e:
        hero.hero_ln_quant(x, torch.ones(4, device="cuda"))
    assert e.value.status == 4                                    # D % 16 != 0
    x = torch.zeros((4, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(HB.HeroError) as e:
        hero.hero_ln_quant(x, None)
    assert e.value.status == 1                                    # INT8 input without a row scale
    q, s, _ = hero.hero_ln_quant(x[:0], torch.ones(0, device="cuda"))     # empty: no-op
    assert q.shape == (0, 64)


# ============================================================ model-load-time operators
@pytest.mark.parametrize("K,N", [(768, 2304), (100, 37), (1024, 4096), (4096, 1024), (65, 130)])
def test_weight_fold_quant_bit_exact(hero, K, N):
    """Fold (fp64, multiply then divide, one cast) + column-wise quantization: codes and scales bit-exact."""
    g = synth.rng(900 + K)
    W = (g.standard_normal((K, N)) * 0.02).astype(np.float32)
    W[:, min(3, N - 1)] = 0                                              # an all-zero column: scale 1, codes 0
    rm = g.uniform(0.001, 0.05, K).astype(np.float32)
    cd = g.uniform(0.002, 0.3, N).astype(np.float32)
    for a, b in ((rm, cd), (None, cd), (rm, None), (None, None)):
        q_o, s_o = O.weight_fold_quant(W, a, b)
        q, s = hero.hero_weight_fold_quant(dev(W), dev(a), dev(b))
        assert_exact(to_np(s), s_o, "column scales")
        assert_exact(to_np(q), q_o, "codes")
        # the FP8 variant: E4M3 codes, scale max / 448, the same fold: bit-exact as well
        q_o, s_o = O.weight_fold_quant_fp8(W, a, b)
        q, s = hero.hero_weight_fold_quant(dev(W), dev(a), dev(b), fp8=True)
        assert_exact(to_np(s), s_o, "fp8 column scales")
        assert_exact(to_np(q), q_o, "fp8 codes")
    # a strided view (leading dimension > N)
    Wbig = dev(np.concatenate([W, W], axis=1))
    q, s = hero.hero_weight_fold_quant(Wbig[:, :N], dev(rm), dev(cd))
    q_o, s_o = O.weight_fold_quant(W, rm, cd)
    assert_exact(to_np(q), q_o) and assert_exact(to_np(s), s_o)


@pytest.mark.parametrize("T,D,dt", [(1000, 768, "f32"), (37, 50, "bf16"), (4096, 1024, "bf16"), (513, 4096, "f16"), (1, 16, "f32")])
def test_absmax_cols_exact_and_running(hero, T, D, dt):
    g = synth.rng(950 + D)
    x = (g.standard_normal((T, D)) * g.uniform(0.1, 30, D)).astype(np.float32)
    if dt == "f32":
        xd, xr = dev(x), x
    elif dt == "bf16":
        xb = O.f32_to_bf16(x); xd, xr = dev(xb, torch.bfloat16), O.bf16_to_f32(xb)
    else:
        xb = O.f32_to_f16(x); xd, xr = dev(xb, torch.float16), O.f16_to_f32(xb)
    m = hero.hero_absmax_cols(xd)
    assert_exact(to_np(m), O.absmax_cols(xr), "first batch")
    x2 = (xr * np.float32(0.5)); x2[T // 2, D // 3] = np.float32(1e4)
    m2 = hero.hero_absmax_cols(dev(x2), m)                               # running maximum, second batch in f32
    assert_exact(to_np(m2), O.absmax_cols(x2, O.absmax_cols(xr)), "running maximum")


# ============================================================ embedding LN^quant
@pytest.mark.parametrize("B,S,d,V,typed,dt", [(3, 50, 768, 1000, True, "bf16"), (2, 37, 1024, 333, True, "f16"),
                                                (5, 16, 48, 64, False, "bf16"), (1, 9, 4096, 100, True, "bf16"),
                                                (8, 128, 1536, 2000, False, "f16")])
def test_embed_ln_quant(hero, B, S, d, V, typed, dt):
    """Sec. 2.2.1: INT8 token table with per-row scales + 16-bit position / type tables -> LN -> TWQ INT8;
    +-1 LSB class like every LayerNorm-fused path."""
    tb = synth.embedding_tables(40 + d, d, V, S + 3, 2)
    ids = synth.embedding_ids(41 + d, B, S, V, 2)
    tq, ts = O.quant_twq(tb["tok"])
    odt, tdt = (O.BF16, torch.bfloat16) if dt == "bf16" else (O.F16, torch.float16)
    cvt = O.f32_to_bf16 if dt == "bf16" else O.f32_to_f16
    pos16, typ16 = cvt(tb["pos"]), cvt(tb["type"])
    g = synth.rng(42 + d)
    gam = (1 + 0.1 * g.standard_normal(d)).astype(np.float32)
    bet = (0.02 * g.standard_normal(d)).astype(np.float32)
    q_o, s_o = O.embed_ln_quant(ids["tok"], ids["pos"], ids["type"] if typed else None, tq, ts, pos16,
                                typ16 if typed else None, odt, gam, bet, 1e-12)
    q, s = hero.hero_embed_ln_quant(dev(ids["tok"]), dev(ids["pos"]), dev(ids["type"]) if typed else None, dev(tq), dev(ts),
                                    dev(pos16, tdt), dev(typ16, tdt) if typed else None, dev(gam), dev(bet), 1e-12)
    assert_scales(to_np(s), s_o, "y_scale")
    assert_codes(to_np(q), q_o, "y_q")
    # an index outside its table is clamped (no fault, the other rows unaffected)
    bad = ids["tok"].copy(); bad[0] = V + 7; bad[1] = -3
    q2, s2 = hero.hero_embed_ln_quant(dev(bad), dev(ids["pos"]), dev(ids["type"]) if typed else None, dev(tq), dev(ts),
                                      dev(pos16, tdt), dev(typ16, tdt) if typed else None, dev(gam), dev(bet), 1e-12)
    assert np.array_equal(to_np(q2)[2:], to_np(q)[2:])
    with pytest.raises(HB.HeroError):
        hero.hero_embed_ln_quant(dev(ids["tok"]), dev(ids["pos"]), None, dev(tq), dev(ts), dev(pos16, tdt),
                                 dev(typ16, tdt), dev(gam), dev(bet), 1e-12)           # type table without type ids


# ============================================================ GeMM^quant
GEMM_SHAPES = [(128, 128, 64), (200, 200, 256), (512, 384, 1024), (77, 1000, 192), (1, 64, 4096), (300, 72, 768)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_raw_int32_bit_exact(hero, M, N, K):
    c = synth.gemm_case(300 + M, M, K, N)
    ref = O.gemm_i32(c["A"], c["Bt"])
    got = hero.hero_int8_gemm(dev(c["A"]), dev(c["Bt"]))
    assert_exact(to_np(got), ref, "acc")


def test_gemm_one_hot_probes_operand_layout(hero):
    """A one-hot A row picks single weight entries: fails on any mistake in the MFMA
    operand or accumulator lane mapping."""
    M, N, K = 160, 192, 128
    g = synth.rng(5)
    Bt = g.integers(-127, 128, (N, K), dtype=np.int8)
    A = np.zeros((M, K), np.int8)
    ks = g.integers(0, K, M)
    A[np.arange(M), ks] = 1
    got = to_np(hero.hero_int8_gemm(dev(A), dev(Bt)))
    assert_exact(got, Bt[:, ks].T.astype(np.int32))
    # extreme magnitude: K = 16384 of 127 * -127
    A = np.full((3, 16384), 127, np.int8)
    Bt = np.full((8, 16384), -127, np.int8)
    assert (to_np(hero.hero_int8_gemm(dev(A), dev(Bt))) == -127 * 127 * 16384).all()


@pytest.mark.parametrize("outlier", [False, True])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES[1:4])
def test_gemm_requant_and_dequant_bit_exact(hero, M, N, K, outlier):
    """REQUANT / DEQUANT: pure fp32 arithmetic on exact integers in a pinned order."""
    c = synth.gemm_case(400 + M, M, K, N, outlier_rows=outlier)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    dA, dB, drs, dcs, db = map(dev, (A, Bt, rs, cs, bias))
    for dt, tdt in ((O.F16, torch.float16), (O.BF16, torch.bfloat16)):
        ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=dt)
        got = hero.hero_int8_gemm(dA, dB, drs, dcs, db, epi=HB.EPI_DEQUANT, out_dtype=tdt)
        assert_exact(to_np(got), ref, f"dequant {dt}")
    # static output scale folded into the column scale (the paper's bare Round)
    y = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y[~np.isin(np.arange(M), np.argsort(rs)[-max(1, M // 100):])]).max() / 127)
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, drs, dev(cs2), dev(b2), epi=HB.EPI_REQUANT, out_dtype=torch.int8)
    assert_exact(to_np(got), ref, "requant")
    if outlier:
        assert (np.abs(ref) == 127).sum() > 0                     # saturation is exercised
    # no row scale, no bias (FWQ input whose scale is folded into the weight)
    ref = O.int8_gemm(A, Bt, b_col_scale=cs2 * np.float32(0.01), epi=O.EPI_REQUANT, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, None, dev(cs2 * np.float32(0.01)), None, epi=HB.EPI_REQUANT, out_dtype=torch.int8)
    assert_exact(to_np(got), ref, "requant no row scale")
    # residual add (in place: C aliases the residual)
    res = O.f32_to_bf16(synth.rng(9).standard_normal((M, N)).astype(np.float32))
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                      epi=O.EPI_DEQUANT, c_dt=O.BF16)
    dres = dev(res)
    got = hero.hero_int8_gemm(dA, dB, drs, dcs, db, residual=dres, epi=HB.EPI_DEQUANT, C_out=dres)
    assert_exact(to_np(got), ref, "dequant + residual in place")


@pytest.mark.parametrize("M,N,K", [(256, 512, 256), (130, 200, 768)])
def test_gemm_gelu_epilogues(hero, M, N, K):
    """GELU^quant (Sec. 2.2.3): fp32 erf on the GPU vs fp64 in the oracle -> +-1 LSB class."""
    c = synth.gemm_case(500 + M, M, K, N)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    cs = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)      # pre-activations of a few units
    g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(g).max(axis=0) / 127).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
    got = hero.hero_int8_gemm(dev(A), dev(Bt), dev(rs), dev(cs), dev(bias), epi=HB.EPI_GELU_REQUANT,
                              out_col_scale=dev(s_a), out_dtype=torch.int8)
    assert_codes(to_np(got), ref, "gelu requant")
    refb = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.BF16)
    gotb = hero.hero_int8_gemm(dev(A), dev(Bt), dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT_GELU, out_dtype=torch.bfloat16)
    assert rel_err(O.bf16_to_f32(to_np(gotb)), O.bf16_to_f32(refb)) <= 2e-2


@pytest.mark.parametrize("M,N,K", [(3300, 3400, 320), (2560, 2560, 256), (4000, 1700, 704), (3300, 3400, 384), (3500, 3100, 640)])
def test_gemm_many_tiles_ragged_edges(hero, M, N, K):
    """Enough 256 x 256 tiles for the large-problem kernels (the persistent one included: several tiles
    per workgroup, ragged last row and column panels, K of 4 / 5 / 6 / 10 / 11 slabs: odd counts take the
    one-tile-per-workgroup kernel, fewer than 160 tiles the 128 x 128 one), strided operands and output;
    every epilogue: REQUANT / DEQUANT / residual / raw bit-exact, GELU^quant in the +-1 LSB class, with and
    without the optional vectors."""
    c = synth.gemm_case(700 + M, M, K + 64, N)
    A_full, rs, cs, bias = c["A"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    A, Bt = A_full[:, :K], c["Bt"][:, :K]
    dA, dB = dev(A_full)[:, :K], dev(c["Bt"])[:, :K]
    y = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y).max() / 127)
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.I8)
    ref_plain = O.int8_gemm(A, Bt, b_col_scale=cs2 * np.float32(0.01), epi=O.EPI_REQUANT, c_dt=O.I8)
    csg = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)
    g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(g).max(axis=0) / 127).astype(np.float32)
    ref_g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
    ref_raw = O.gemm_i32(A, Bt)
    ref_f16 = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F16)
    res = O.f32_to_bf16(synth.rng(11).standard_normal((M, N)).astype(np.float32))
    ref_res = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                          epi=O.EPI_DEQUANT, c_dt=O.BF16)
    for tile in (None, 1, 7, 8):             # default choice, one tile per workgroup, persistent 256 x 256 and 128 x 128
        Cbuf = torch.full((M, N + 16), -7, dtype=torch.int8, device="cuda")
        hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(b2), epi=HB.EPI_REQUANT, C_out=Cbuf[:, :N], tile=tile)
        assert_exact(to_np(Cbuf[:, :N]), ref, f"requant tile={tile}")
        assert (to_np(Cbuf[:, N:]) == -7).all()
        got = hero.hero_int8_gemm(dA, dB, None, dev(cs2 * np.float32(0.01)), None, epi=HB.EPI_REQUANT, out_dtype=torch.int8, tile=tile)
        assert_exact(to_np(got), ref_plain, f"requant, no row scale, no bias, tile={tile}")
        got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_GELU_REQUANT,
                                  out_col_scale=dev(s_a), out_dtype=torch.int8, tile=tile)
        assert_codes(to_np(got), ref_g, f"gelu requant tile={tile}")
        assert_exact(to_np(hero.hero_int8_gemm(dA, dB, tile=tile)), ref_raw, f"raw tile={tile}")
        got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT, out_dtype=torch.float16, tile=tile)
        assert_exact(to_np(got), ref_f16, f"dequant f16 tile={tile}")
        dres = dev(res)
        got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), residual=dres, epi=HB.EPI_DEQUANT, C_out=dres, tile=tile)
        assert_exact(to_np(got), ref_res, f"dequant + residual in place tile={tile}")


@pytest.mark.parametrize("M,N,K", [(3300, 3400, 1024), (4200, 4100, 1152), (2100, 6200, 2048)])
def test_gemm_overlapped_epilogue_kernel(hero, M, N, K):
    """The persistent 256 x 128 kernel whose epilogue runs inside the next tile's main loop (tile code 9; the
    default choice from 320 such tiles and K >= 1024 on): one to three tiles per workgroup, ragged last row and
    column panels, K of exactly 16 slabs (no slab without an epilogue step), 18 and 32 slabs; an output whose
    rows are 8-element aligned (plain wide stores in the interior tiles) and one whose rows are not (the careful
    store path everywhere), with canary columns.  REQUANT / DEQUANT / raw bit-exact, GELU^quant in its +-1 LSB class."""
    c = synth.gemm_case(900 + M, M, K, N)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    dA, dB = dev(A), dev(Bt)
    y = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y).max() / 127)
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.I8)
    for pad in (16, 12):                                       # row stride N + 16 (8-aligned) and N + 12 (not)
        Cbuf = torch.full((M, N + pad), -7, dtype=torch.int8, device="cuda")
        hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(b2), epi=HB.EPI_REQUANT, C_out=Cbuf[:, :N], tile=9)
        assert_exact(to_np(Cbuf[:, :N]), ref, f"requant, row stride N+{pad}")
        assert (to_np(Cbuf[:, N:]) == -7).all()
    ref_plain = O.int8_gemm(A, Bt, b_col_scale=cs2 * np.float32(0.01), epi=O.EPI_REQUANT, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, None, dev(cs2 * np.float32(0.01)), None, epi=HB.EPI_REQUANT, out_dtype=torch.int8, tile=9)
    assert_exact(to_np(got), ref_plain, "requant, no row scale, no bias")
    csg = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)
    gl = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(gl).max(axis=0) / 127).astype(np.float32)
    ref_g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_GELU_REQUANT, out_col_scale=dev(s_a),
                              out_dtype=torch.int8, tile=9)
    assert_codes(to_np(got), ref_g, "gelu requant")
    assert_exact(to_np(hero.hero_int8_gemm(dA, dB, tile=9)), O.gemm_i32(A, Bt), "raw")
    for dt, tdt in ((O.F16, torch.float16), (O.BF16, torch.bfloat16)):
        ref16 = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=dt)
        Cb = torch.zeros((M, N + 4), dtype=tdt, device="cuda")          # row stride not 8-aligned
        hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT, C_out=Cb[:, :N], tile=9)
        assert_exact(to_np(Cb[:, :N]), ref16, f"dequant {tdt}")
        assert (to_np(Cb[:, N:]) == 0).all()
    ref_gl = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.BF16)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_DEQUANT_GELU, out_dtype=torch.bfloat16, tile=9)
    assert rel_err(O.bf16_to_f32(to_np(got)), O.bf16_to_f32(ref_gl)) <= 2e-2
    assert np.mean(to_np(got) == ref_gl) > 0.999               # fp32 GELU against the definition's fp64: a last-bit flip now and then


def test_gemm_overlapped_epilogue_kernel_at_the_bench_shapes(hero):
    """At the FC1 shape of config 2 and two M = 8192 shapes of the config-1 sweep the overlapped kernel, the
    persistent 256 x 256 kernel and the default choice give the same bytes (integer contraction, the same fp32
    epilogue); with GELU^quant the overlapped kernel multiplies by the correctly rounded 1 / S_a where the
    others use v_rcp_f32, so a code may differ by one step now and then."""
    for (M, N, K) in ((16384, 4096, 1024), (8192, 3072, 1024), (8192, 1024, 4096)):
        c = synth.gemm_case(950, M, K, N)
        dA, dB, rs, cs, bias = (dev(c[k]) for k in ("A", "Bt", "a_row_scale", "b_col_scale", "bias"))
        cs = cs * (30.0 / K ** 0.5)
        sa = torch.full((N,), 0.03, dtype=torch.float32, device="cuda")
        outs = [hero.hero_int8_gemm(dA, dB, rs, cs, bias, epi=HB.EPI_GELU_REQUANT, out_col_scale=sa, out_dtype=torch.int8, tile=t)
                for t in (None, 9, 7)]
        for o in (outs[0], outs[2]):
            d = (outs[1].to(torch.int16) - o.to(torch.int16)).abs()
            assert int(d.max()) <= 1 and float((d != 0).float().mean()) <= 1e-4
        for epi, dt in ((HB.EPI_DEQUANT, torch.float16), (HB.EPI_REQUANT, torch.int8)):
            o = [hero.hero_int8_gemm(dA, dB, rs, cs * 0.05, bias, epi=epi, out_dtype=dt, tile=t) for t in (None, 9, 7)]
            assert torch.equal(o[0].view(torch.int8), o[1].view(torch.int8)) and torch.equal(o[1].view(torch.int8), o[2].view(torch.int8))


@pytest.mark.parametrize("M,N,K", [(64, 4096, 16384), (33, 1000, 8704), (100, 2304, 8192), (1, 512, 16384), (64, 1024, 8192)])
def test_gemm_skinny_split_k_workspace(hero, M, N, K):
    """hero_int8_gemm_ws: K split over several workgroups per tile with int32 partial sums in a caller-owned
    scratch.  Integer sums commute, so every epilogue stays in its class (raw / REQUANT / DEQUANT / residual
    bit-exact); the scratch needs no initialisation (it starts out as garbage here) and serves calls of other shapes."""
    nbytes = hero.hero_int8_gemm_workspace_bytes(M, N, K)
    assert nbytes > 0
    assert hero.hero_int8_gemm_workspace_bytes(4096, N, K) == 0        # not skinny: no split
    assert hero.hero_int8_gemm_workspace_bytes(M, 1024, 512) == 0      # small weights: no split either
    assert hero.hero_int8_gemm_workspace_bytes(64, 12288, 4096) == 0   # K = 4096: the one-pass kernels are faster
    ws = torch.full((max(nbytes, hero.hero_int8_gemm_workspace_bytes(64, 4096, 16384)),), 0xA5, dtype=torch.uint8, device="cuda")
    c = synth.gemm_case(800 + M, M, K, N)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    dA, dB = dev(A), dev(Bt)
    assert_exact(to_np(hero.hero_int8_gemm(dA, dB, workspace=ws)), O.gemm_i32(A, Bt), "raw")
    y = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y).max() / 127)
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(b2), epi=HB.EPI_REQUANT, out_dtype=torch.int8, workspace=ws)
    assert_exact(to_np(got), ref, "requant")
    res = O.f32_to_bf16(synth.rng(12).standard_normal((M, N)).astype(np.float32))
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                      epi=O.EPI_DEQUANT, c_dt=O.BF16)
    dres = dev(res)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), residual=dres, epi=HB.EPI_DEQUANT, C_out=dres, workspace=ws)
    assert_exact(to_np(got), ref, "dequant + residual in place")
    csg = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)
    g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(g).max(axis=0) / 127 + 1e-6).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_GELU_REQUANT, out_col_scale=dev(s_a),
                              out_dtype=torch.int8, workspace=ws)
    assert_codes(to_np(got), ref, "gelu requant")
    with pytest.raises(HB.HeroError):                                   # misaligned scratch
        hero.hero_int8_gemm(dA, dB, workspace=ws[16:])


@pytest.mark.parametrize("M,N,K", [(64, 4096, 4096), (37, 1000, 2048), (64, 12288, 4096), (5, 8264, 2176), (64, 8200, 2112), (1, 16384, 4096)])
def test_gemm_skinny_one_pass_forms(hero, M, N, K):
    """One row of tiles (M <= 64, a decode step) without a scratch: 64 x 32 tiles with eight slabs in flight up to
    128 tiles of 64 x 64, two K groups per workgroup beyond (the last shape has an odd slab count and takes the plain
    tile).  Every epilogue in its class: raw / REQUANT / DEQUANT (+ residual, in place) bit-exact, GELU^quant +-1."""
    c = synth.gemm_case(900 + M + N % 97, M, K, N)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    dA, dB = dev(A), dev(Bt)
    assert_exact(to_np(hero.hero_int8_gemm(dA, dB)), O.gemm_i32(A, Bt), "raw")
    y = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y).max() / 127)
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(b2), epi=HB.EPI_REQUANT, out_dtype=torch.int8)
    assert_exact(to_np(got), ref, "requant")
    assert np.abs(ref).max() == 127
    res = O.f32_to_bf16(synth.rng(13).standard_normal((M, N)).astype(np.float32))
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                      epi=O.EPI_DEQUANT, c_dt=O.BF16)
    dres = dev(res)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), residual=dres, epi=HB.EPI_DEQUANT, C_out=dres)
    assert_exact(to_np(got), ref, "dequant + residual in place")
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F16)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT, out_dtype=torch.float16)
    assert_exact(to_np(got), ref, "dequant f16")
    csg = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)
    g = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(g).max(axis=0) / 127 + 1e-6).astype(np.float32)
    ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
    got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_GELU_REQUANT, out_col_scale=dev(s_a),
                              out_dtype=torch.int8)
    assert_codes(to_np(got), ref, "gelu requant", max_frac=max(1e-3, 2.5 / ref.size))


def test_gemm_strided_operands_and_errors(hero):
    """Leading dimensions larger than the logical width; invalid combinations are refused."""
    M, N, K = 96, 80, 128
    c = synth.gemm_case(600, M, K + 64, N + 16)
    A_full, B_full = dev(c["A"]), dev(c["Bt"])
    A, Bt = A_full[:, :K], B_full[:N, :K]
    Cbuf = torch.full((M, N + 48), -7, dtype=torch.int32, device="cuda")
    hero.hero_int8_gemm(A, Bt, C_out=Cbuf[:, :N])
    assert_exact(to_np(Cbuf[:, :N]), O.gemm_i32(c["A"][:, :K], c["Bt"][:N, :K]))
    assert (to_np(Cbuf[:, N:]) == -7).all()                        # nothing written past N
    with pytest.raises(HB.HeroError) as e:
        hero.hero_int8_gemm(A, Bt, epi=HB.EPI_REQUANT, out_dtype=torch.int8)     # no column scale
    assert e.value.status == 1
    with pytest.raises(HB.HeroError) as e:
        hero.hero_int8_gemm(A, Bt, None, torch.ones(N, device="cuda"), epi=HB.EPI_REQUANT, out_dtype=torch.float16)
    assert e.value.status == 4
    with pytest.raises(HB.HeroError) as e:
        hero.hero_int8_gemm(A_full[:, :K - 16], B_full[:N, :K - 16])             # K % 64 != 0
    assert e.value.status == 4


# ============================================================ INT8 attention
def _attn_case(seed, B, Sq, Skv, H, Dh):
    g = synth.rng(seed)
    # q/k/v codes with the spread of SQ-quantized N(0,1)-ish activations (|code| mostly < 60)
    mk = lambda s: np.clip(np.rint(g.standard_normal(s) * 30), -127, 127).astype(np.int8)
    q, k, v = mk((B, Sq, H, Dh)), mk((B, Skv, H, Dh)), mk((B, Skv, H, Dh))
    qk_scale = np.float32(4.0 / (30 * 30 * np.sqrt(Dh)) / np.sqrt(Dh) * 6)       # logits of a few units
    cs = g.uniform(0.8, 1.2, H * Dh).astype(np.float32) * np.float32(1.0 / (255 * 30) * 127 / 2.5)
    return q, k, v, float(qk_scale), cs


ATTN_SHAPES = [(2, 200, 200, 2, 64), (1, 128, 128, 3, 128), (2, 77, 300, 2, 64), (1, 513, 513, 1, 128)]


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
@pytest.mark.parametrize("B,Sq,Skv,H,Dh", ATTN_SHAPES)
def test_int8_attn_matches_oracle(hero, B, Sq, Skv, H, Dh, mask):
    q, k, v, qk_scale, cs = _attn_case(700 + Sq + Dh, B, Sq, Skv, H, Dh)
    kv_len = None
    if mask == O.MASK_PADDING:
        kv_len = np.int32([Skv - 3, 0][:B]) if B == 2 else np.int32([Skv // 2 + 1])
    if mask == O.MASK_CAUSAL and Sq != Skv:
        kv_len = np.int32([Skv, Skv - 50][:B])
    ref = O.int8_attn(q, k, v, qk_scale=qk_scale, p_scale=float(OL.S_P), out_col_scale=cs, mask=mask, kv_len=kv_len)
    got = hero.hero_int8_attn(dev(q), dev(k), dev(v), qk_scale, float(OL.S_P), dev(cs), mask=mask, kv_len=dev(kv_len))
    assert np.abs(ref).max() > 40                                  # the case is not degenerate
    assert_codes(to_np(got), ref, "X_attn")
    # 16-bit float output (the consumer is a BF16 attention-output linear)
    sc = np.float32([cs[0]])
    refb = O.int8_attn(q, k, v, qk_scale=qk_scale, p_scale=float(OL.S_P), out_col_scale=sc, out_scale_is_scalar=True,
                       mask=mask, kv_len=kv_len, out_dt=O.BF16)
    gotb = hero.hero_int8_attn(dev(q), dev(k), dev(v), qk_scale, float(OL.S_P), dev(sc), out_scale_is_scalar=True,
                               mask=mask, kv_len=dev(kv_len), out_dtype=torch.bfloat16)
    assert rel_err(O.bf16_to_f32(to_np(gotb)), O.bf16_to_f32(refb)) <= 2e-2


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
@pytest.mark.parametrize("B,Sq,Skv,H,Dh", ATTN_SHAPES + [(2, 1, 150, 2, 64)])
def test_int8_attn_online_matches_oracle(hero, B, Sq, Skv, H, Dh, mask):
    """The single-sweep variant (codes against the running 64-key-block maximum, normalised at the end) against
    its own oracle; per-head score scales; the output classes of the two-pass operator."""
    q, k, v, qk_scale, cs = _attn_case(1400 + Sq + Dh, B, Sq, Skv, H, Dh)
    dts = (np.float32(qk_scale) * np.linspace(0.7, 1.6, H)).astype(np.float32)
    kv_len = None
    if mask == O.MASK_PADDING:
        kv_len = np.int32([Skv - 3, 0][:B]) if B == 2 else np.int32([Skv // 2 + 1])
    if mask == O.MASK_CAUSAL and Sq != Skv:
        kv_len = np.int32([Skv, Skv - 50][:B])
    sp = float(OL.S_P)
    ref = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len, kv_block=64)
    got = hero.hero_int8_attn_online(dev(q), dev(k), dev(v), dev(dts), sp, dev(cs), mask=mask, kv_len=dev(kv_len))
    assert np.abs(ref).max() > 40
    assert_codes(to_np(got), ref, "X_attn online", max_frac=3e-3 if ref.size < 2000 else 1e-3)
    sc = np.float32([cs[0]])
    refb = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=sc, out_scale_is_scalar=True,
                              mask=mask, kv_len=kv_len, out_dt=O.BF16, kv_block=64)
    gotb = hero.hero_int8_attn_online(dev(q), dev(k), dev(v), dev(dts), sp, dev(sc), out_scale_is_scalar=True,
                                      mask=mask, kv_len=dev(kv_len), out_dtype=torch.bfloat16)
    assert rel_err(O.bf16_to_f32(to_np(gotb)), O.bf16_to_f32(refb)) <= 2e-2


def test_int8_attn_online_views_errors_and_long_rows(hero):
    """Fused-buffer views, a long causal row set (many flushes and many tiles without one), no keys, bad arguments."""
    B, S, H, Dh = 2, 1100, 2, 64
    d = H * Dh
    g = synth.rng(1450)
    qkv = np.clip(np.rint(g.standard_normal((B * S, 3 * d)) * 30), -127, 127).astype(np.int8)
    _, _, _, qk_scale, cs = _attn_case(1451, 1, 1, 1, H, Dh)
    dts = np.float32([qk_scale, 2 * qk_scale])
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    sp = float(OL.S_P)
    ref = O.int8_attn_online(qv, kv, vv, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, mask=O.MASK_CAUSAL)
    dq = dev(qkv).view(B, S, 3, H, Dh)
    got = hero.hero_int8_attn_online(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], dev(dts), sp, dev(cs), mask=HB.MASK_CAUSAL)
    assert_codes(to_np(got), ref, "online, fused-buffer views, causal 1100")
    z = hero.hero_int8_attn_online(dq[:, :4, 0], dq[:, :0, 1], dq[:, :0, 2], dev(dts), sp, dev(cs))
    assert not to_np(z).any()
    with pytest.raises(HB.HeroError):
        hero.hero_int8_attn_online(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], None, sp, dev(cs))


def test_int8_attn_strided_views_cache_and_decode(hero):
    """Operands as views into a fused [T,3d] buffer and a [B,H,Smax,Dh] cache; one-query decode."""
    B, S, H, Dh = 3, 70, 2, 64
    d = H * Dh
    g = synth.rng(800)
    qkv = np.clip(np.rint(g.standard_normal((B * S, 3 * d)) * 30), -127, 127).astype(np.int8)
    _, _, _, qk_scale, cs = _attn_case(801, 1, 1, 1, H, Dh)
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    ref = O.int8_attn(qv, kv, vv, qk_scale=qk_scale, p_scale=float(OL.S_P), out_col_scale=cs, mask=O.MASK_CAUSAL)
    dq = dev(qkv).view(B, S, 3, H, Dh)
    got = hero.hero_int8_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], qk_scale, float(OL.S_P), dev(cs), mask=HB.MASK_CAUSAL)
    assert_codes(to_np(got), ref, "fused-buffer views")
    Smax = 96
    kc = np.zeros((B, H, Smax, Dh), np.int8)
    vc = np.zeros((B, H, Smax, Dh), np.int8)
    kc[:, :, :S], vc[:, :, :S] = kv.transpose(0, 2, 1, 3), vv.transpose(0, 2, 1, 3)
    lens = np.int32([S, S - 9, 1])
    q1 = np.ascontiguousarray(qv[:, -1:, :, :])
    ref = O.int8_attn(q1, kc.transpose(0, 2, 1, 3), vc.transpose(0, 2, 1, 3), qk_scale=qk_scale, p_scale=float(OL.S_P),
                      out_col_scale=cs, mask=O.MASK_PADDING, kv_len=lens)
    dk, dv = dev(kc), dev(vc)
    got = hero.hero_int8_attn(dev(q1), dk.permute(0, 2, 1, 3), dv.permute(0, 2, 1, 3), qk_scale, float(OL.S_P), dev(cs),
                              mask=HB.MASK_PADDING, kv_len=dev(lens))
    assert_codes(to_np(got), ref, "decode against the cache", max_frac=3e-3)    # 384 outputs: 1 flip = 0.26 %
    # no keys at all -> zeros
    z = hero.hero_int8_attn(dev(q1), dk.permute(0, 2, 1, 3)[:, :0], dv.permute(0, 2, 1, 3)[:, :0], qk_scale,
                            float(OL.S_P), dev(cs))
    assert not to_np(z).any()


@pytest.mark.parametrize("Dh", [64, 128])
@pytest.mark.parametrize("Skv", [16384, 16400])
def test_one_query_attention_at_the_longest_cache(hero, Dh, Skv):
    """One query against 16384 keys (the longest cache the cache-streaming kernel takes: 64 KB of scores in LDS on
    top of its static buffers) and against 16400 (served by the general kernel), INT8 and E4M3 codes."""
    B, H = 2, 2
    g = synth.rng(3000 + Dh + Skv)
    mk = lambda s: np.clip(np.rint(g.standard_normal(s) * 30), -127, 127).astype(np.int8)
    q, kc, vc = mk((B, 1, H, Dh)), mk((B, H, Skv, Dh)), mk((B, H, Skv, Dh))
    lens = np.int32([Skv, Skv - 777])
    qk_scale = float(np.float32(4.5 / (900.0 * np.sqrt(Dh))))       # peaked rows: over 16384 keys a diffuse row has only zero codes
    cs = (g.uniform(0.8, 1.2, H * Dh) / (255 * 30) * 400).astype(np.float32)
    ref = O.int8_attn(q, kc.transpose(0, 2, 1, 3), vc.transpose(0, 2, 1, 3), qk_scale=qk_scale, p_scale=float(OL.S_P),
                      out_col_scale=cs, mask=O.MASK_PADDING, kv_len=lens)
    dk, dv = dev(kc), dev(vc)
    got = hero.hero_int8_attn(dev(q), dk.permute(0, 2, 1, 3), dv.permute(0, 2, 1, 3), qk_scale, float(OL.S_P), dev(cs),
                              mask=HB.MASK_PADDING, kv_len=dev(lens))
    assert np.abs(ref).max() > 20
    assert_codes(to_np(got), ref, "one query, longest cache", max_frac=2.5 / ref.size)
    q8, k8, v8 = (O.f32_to_e4m3(t.astype(np.float32)) for t in (q, kc, vc))            # the same values as E4M3 codes
    sp = float(OL.S_P_FP8)
    cs8 = (cs * np.float32(255.0 / 448.0)).astype(np.float32)
    ref8 = O.fp8_attn(q8, k8.transpose(0, 2, 1, 3), v8.transpose(0, 2, 1, 3), qk_scale=qk_scale, p_scale=sp, out_col_scale=cs8,
                      mask=O.MASK_PADDING, kv_len=lens)
    got8 = hero.hero_fp8_attn(dev(q8), dev(k8).permute(0, 2, 1, 3), dev(v8).permute(0, 2, 1, 3), qk_scale, sp, dev(cs8),
                              mask=HB.MASK_PADDING, kv_len=dev(lens))
    D = fp8_attn_flip_bound(q8, k8.transpose(0, 2, 1, 3), v8.transpose(0, 2, 1, 3), qk_scale, sp, cs8, mask=1, kv_len=lens)
    assert_fp8_attn_codes(to_np(got8.view(torch.uint8)), ref8, O.e4m3_to_f32, "one query, longest cache, fp8", flip_bound=D)


@pytest.mark.parametrize("M,N,K", [(8192, 4096, 1024), (2048 + 77, 3072 + 8, 1024), (8192, 1024, 4096)])
def test_gemm_full_size_sampled_rows(hero, M, N, K):
    """The benchmark's launch configuration (256x256 direct-to-LDS kernel, XCD-aware tile
    order) at the sweep's full sizes: sampled output rows against the oracle, bit-exact, for
    the raw accumulators, REQUANT and DEQUANT; every tile row-panel and a ragged edge are hit."""
    c = synth.gemm_case(900 + M, M, K, N, outlier_rows=True)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    g = synth.rng(901)
    rows = np.unique(np.concatenate([g.integers(0, M, 48), [0, 255, 256, M - 1], np.arange(M // 256) * 256 + 131]))
    dA, dB = dev(A), dev(Bt)
    raw = to_np(hero.hero_int8_gemm(dA, dB))
    assert_exact(raw[rows], O.gemm_i32(A[rows], Bt), "acc rows")
    cs2 = (cs * np.float32(3000.0 / np.sqrt(K))).astype(np.float32)
    got = to_np(hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(bias), epi=HB.EPI_REQUANT, out_dtype=torch.int8))
    ref = O.int8_gemm(A[rows], Bt, a_row_scale=rs[rows], b_col_scale=cs2, bias=bias, epi=O.EPI_REQUANT, c_dt=O.I8)
    assert_exact(got[rows], ref, "requant rows")
    assert 0 < np.mean(np.abs(ref) == 127) < 0.5
    got = to_np(hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT, out_dtype=torch.float16))
    ref = O.int8_gemm(A[rows], Bt, a_row_scale=rs[rows], b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F16)
    assert_exact(got[rows], ref, "dequant rows")
    # property that holds at any size: column sums of the raw accumulators
    colsum = A.astype(np.int64).sum(axis=0) @ Bt.astype(np.int64).T
    assert np.array_equal(raw.astype(np.int64).sum(axis=0), colsum)


# ============================================================ FP8 variant
@pytest.mark.parametrize("M,N,K,tile", [(200, 136, 256, None), (64, 72, 192, None), (300, 520, 1024, None), (3300, 3400, 384, None),
                                         (3300, 3400, 384, "8"), (2500, 2600, 256, None), (2500, 2600, 256, "7"),
                                         (100, 264, 2304, None)])
def test_fp8_gemm_matches_oracle(hero, M, N, K, tile):
    """hero_fp8_gemm (Sec. 2.1: FP8 as the 8-bit format): E4M3 operands, fp32 accumulation on the matrix cores
    (the oracle carries the exact sum), the INT8 path's epilogue.  16-bit outputs within 2e-2, E4M3 outputs equal
    up to an adjacent code on <= 0.5 %.  The large shapes run the persistent kernels with ragged edges: by
    default the 256 x 256 one (182 tiles) and the 128 x 128 one (110 tiles of 256 x 256), then each the other one.
    The last shape (few tiles, K = 2304) runs the workgroup with four K groups: fp32 partial sums added through LDS."""
    tile = None if tile is None else int(tile)
    g = synth.rng(1300 + M)
    X = (g.standard_normal((M, K)) * g.uniform(0.5, 4, (M, 1))).astype(np.float32)
    W = (g.standard_normal((K, N)) * 0.05).astype(np.float32)
    A, rs = O.quant_twq_fp8(X)                                            # token-wise FP8 activations
    wmax = np.abs(W).max(axis=0)
    cs = (wmax / 448).astype(np.float32)
    Bt = O.f32_to_e4m3((W / cs[None, :]).T.astype(np.float32))            # column-wise FP8 weights, [N][K]
    bias = (0.1 * g.standard_normal(N)).astype(np.float32)
    dA, dB = dev(A), dev(Bt)
    for dt, tdt, cvt in ((O.BF16, torch.bfloat16, O.bf16_to_f32), (O.F16, torch.float16, O.f16_to_f32)):
        ref = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=dt)
        got = hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT, out_dtype=tdt, tile=tile)
        assert rel_err(cvt(to_np(got)), cvt(ref)) <= 2e-2
    res = O.f32_to_bf16(g.standard_normal((M, N)).astype(np.float32))
    ref = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16, epi=O.EPI_DEQUANT, c_dt=O.BF16)
    dres = dev(res)
    got = hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), residual=dres, epi=HB.EPI_DEQUANT, C_out=dres, tile=tile)
    assert rel_err(O.bf16_to_f32(to_np(got)), O.bf16_to_f32(ref)) <= 2e-2
    ref = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.BF16)
    got = hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_DEQUANT_GELU, out_dtype=torch.bfloat16, tile=tile)
    assert rel_err(O.bf16_to_f32(to_np(got)), O.bf16_to_f32(ref)) <= 2e-2
    # 8-bit outputs: a static output scale folded into the column scale (REQUANT), GELU^quant with S_a
    y = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    s_out = np.float32(np.abs(y).max() / 448 * 0.9)                       # a little saturation
    cs2, b2 = (cs / s_out).astype(np.float32), (bias / s_out).astype(np.float32)
    ref = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=b2, epi=O.EPI_REQUANT, c_dt=O.F8)
    got = hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs2), dev(b2), epi=HB.EPI_REQUANT, out_dtype=torch.float8_e4m3fn, tile=tile)
    # The FP8 matrix instruction adds each lane's group of 8 products after aligning them to the group's largest
    # with 13 fractional bits, truncating (measured on gfx950: 256 + 2^-5 survives, 256 + 2^-6 does not), so a dot
    # product carries a relative error of ~1e-4 where the exact sum of the definition has none; E4M3's grid is
    # 1/8 .. 1/16 of the value, so ~16 x 1e-4 of the outputs sit that close to a rounding boundary.  The error
    # scales with the typical product, so outputs far below the typical magnitude may move by 1e-3 of the rms.
    assert_fp8_codes(to_np(got), ref, O.e4m3_to_f32, "requant", max_frac=5e-3, acc_rel=1e-3)
    assert (ref & 0x7F == 0x7E).sum() > 0
    gl = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    s_a = (np.abs(gl).max(axis=0) / 448 + 1e-6).astype(np.float32)
    ref = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.F8)
    got = hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), epi=HB.EPI_GELU_REQUANT, out_col_scale=dev(s_a), tile=tile,
                             out_dtype=torch.float8_e4m3fn)
    # the same bound; in addition the kernel's GELU is accurate to 1.1e-7 ABSOLUTE (built for the INT8 grid)
    # while E4M3 resolves small values down to a step of 2^-9 S_a.
    assert_fp8_codes(to_np(got), ref, O.e4m3_to_f32, "gelu requant", max_frac=5e-3, acc_rel=1e-3)
    with pytest.raises(HB.HeroError):
        hero.hero_fp8_gemm(dA, dB, dev(rs), dev(cs), epi=HB.EPI_REQUANT, out_dtype=torch.bfloat16)


def _fp8_attn_case(seed, B, Sq, Skv, H, Dh):
    g = synth.rng(seed)
    mk = lambda s: O.f32_to_e4m3((g.standard_normal(s) * 40).astype(np.float32))     # E4M3 codes of SQ-scaled activations
    q, k, v = mk((B, Sq, H, Dh)), mk((B, Skv, H, Dh)), mk((B, Skv, H, Dh))
    qk_scale = float(np.float32(1.5 / (40 * 40 * np.sqrt(Dh))))                       # logits of a few units
    sp = np.float32(1.0 / 448.0)
    cs = g.uniform(0.8, 1.2, H * Dh).astype(np.float32) * sp * np.float32(4.0)
    return q, k, v, qk_scale, float(sp), cs


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
@pytest.mark.parametrize("B,Sq,Skv,H,Dh", ATTN_SHAPES)
def test_fp8_attn_matches_oracle(hero, B, Sq, Skv, H, Dh, mask):
    """hero_fp8_attn (Sec. 2.2.2 flow with E4M3 codes) against its oracle.  A probability code may land on the
    neighbouring E4M3 value only where the oracle's own p / S_p is next to a rounding boundary; the bound on what those
    flips can do to each output (parity.fp8_attn_flip_bound) is the tolerance, plus one step of the output grid (E4M3
    output) or the 16-bit rounding; rows without such a probability must carry the oracle's codes."""
    q, k, v, qk_scale, sp, cs = _fp8_attn_case(2000 + Sq + Dh, B, Sq, Skv, H, Dh)
    kv_len = None
    if mask == O.MASK_PADDING:
        kv_len = np.int32([Skv - 3, 0][:B]) if B == 2 else np.int32([Skv // 2 + 1])
    if mask == O.MASK_CAUSAL and Sq != Skv:
        kv_len = np.int32([Skv, Skv - 50][:B])
    ref = O.fp8_attn(q, k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len)
    got = hero.hero_fp8_attn(dev(q), dev(k), dev(v), qk_scale, sp, dev(cs), mask=mask, kv_len=dev(kv_len))
    assert got.dtype == torch.float8_e4m3fn and np.abs(O.e4m3_to_f32(ref)).max() > 100      # not degenerate
    D = fp8_attn_flip_bound(q, k, v, qk_scale, sp, cs, mask=mask, kv_len=kv_len)
    clean, diff = assert_fp8_attn_codes(to_np(got.view(torch.uint8)), ref, O.e4m3_to_f32, "X_attn fp8", flip_bound=D)
    print(f"[parity] fp8 attention {B}x{Sq}x{Skv}x{H}x{Dh} mask {mask}: {clean:.3f} of the outputs have no probability near a boundary, "
          f"{diff:.2e} of all codes differ")
    if mask == O.MASK_PADDING and B == 2:
        assert not to_np(got.view(torch.uint8))[Sq:].any()               # the batch row without keys
    sc = np.float32([cs[0]])
    for odt, tdt, cvt in ((O.BF16, torch.bfloat16, O.bf16_to_f32), (O.F16, torch.float16, O.f16_to_f32)):
        refb = O.fp8_attn(q, k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=sc, out_scale_is_scalar=True,
                          mask=mask, kv_len=kv_len, out_dt=odt)
        gotb = hero.hero_fp8_attn(dev(q), dev(k), dev(v), qk_scale, sp, dev(sc), out_scale_is_scalar=True,
                                  mask=mask, kv_len=dev(kv_len), out_dtype=tdt)
        assert_fp8_attn_values(cvt(to_np(gotb)), cvt(refb), "16-bit output", flip_bound=D / cs[None, :] * sc[0])


def test_fp8_attn_views_cache_one_query_and_errors(hero):
    """Operands as views into a fused [T,3d] buffer and a [B,H,Smax,Dh] cache with one query per sequence; no keys;
    argument errors (INT8 output type, per-column scales with a 16-bit output, unsupported head size)."""
    B, S, H, Dh = 3, 70, 2, 64
    d = H * Dh
    g = synth.rng(2100)
    qkv = O.f32_to_e4m3((g.standard_normal((B * S, 3 * d)) * 40).astype(np.float32))
    _, _, _, qk_scale, sp, cs = _fp8_attn_case(2101, 1, 1, 1, H, Dh)
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    ref = O.fp8_attn(qv, kv, vv, qk_scale=qk_scale, p_scale=sp, out_col_scale=cs, mask=O.MASK_CAUSAL)
    dq = dev(qkv).view(B, S, 3, H, Dh)
    got = hero.hero_fp8_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], qk_scale, sp, dev(cs), mask=HB.MASK_CAUSAL)
    D = fp8_attn_flip_bound(qv, kv, vv, qk_scale, sp, cs, mask=2)
    assert_fp8_attn_codes(to_np(got.view(torch.uint8)), ref, O.e4m3_to_f32, "fused-buffer views", flip_bound=D)
    Smax = 96
    kc = np.zeros((B, H, Smax, Dh), np.uint8)
    vc = np.zeros((B, H, Smax, Dh), np.uint8)
    kc[:, :, :S], vc[:, :, :S] = kv.transpose(0, 2, 1, 3), vv.transpose(0, 2, 1, 3)
    lens = np.int32([S, S - 9, 1])
    q1 = np.ascontiguousarray(qv[:, -1:, :, :])
    ref = O.fp8_attn(q1, kc.transpose(0, 2, 1, 3), vc.transpose(0, 2, 1, 3), qk_scale=qk_scale, p_scale=sp,
                     out_col_scale=cs, mask=O.MASK_PADDING, kv_len=lens)
    dk, dv = dev(kc), dev(vc)
    got = hero.hero_fp8_attn(dev(q1), dk.permute(0, 2, 1, 3), dv.permute(0, 2, 1, 3), qk_scale, sp, dev(cs),
                             mask=HB.MASK_PADDING, kv_len=dev(lens))
    D = fp8_attn_flip_bound(q1, kc.transpose(0, 2, 1, 3), vc.transpose(0, 2, 1, 3), qk_scale, sp, cs, mask=1, kv_len=lens)
    assert_fp8_attn_codes(to_np(got.view(torch.uint8)), ref, O.e4m3_to_f32, "one query against the cache", flip_bound=D)
    z = hero.hero_fp8_attn(dev(q1), dk.permute(0, 2, 1, 3)[:, :0], dv.permute(0, 2, 1, 3)[:, :0], qk_scale, sp, dev(cs))
    assert not to_np(z.view(torch.uint8)).any()
    with pytest.raises(HB.HeroError):
        hero.hero_fp8_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], qk_scale, sp, dev(cs), out_dtype=torch.bfloat16)   # needs a scalar scale
    with pytest.raises(HB.HeroError):
        st = hero.lib.hero_fp8_attn(dq.data_ptr(), HB._strides4(dq[:, :, 0]), dq.data_ptr(), HB._strides4(dq[:, :, 1]),
                                    dq.data_ptr(), HB._strides4(dq[:, :, 2]), B, H, S, S, Dh, qk_scale, sp,
                                    dev(cs).data_ptr(), 0, 0, None, got.data_ptr(), HB.I8, d, None)
        hero._check(st)                                                   # INT8 is not an output type of the FP8 flow
    with pytest.raises(HB.HeroError):
        bad = dev(qkv[:, :3 * 2 * 32]).view(B, S, 3, 2, 32)
        hero.hero_fp8_attn(bad[:, :, 0], bad[:, :, 1], bad[:, :, 2], qk_scale, sp, dev(cs[:64]))


# ============================================================ 16-bit side of a switched module (BF16 / FP16)
@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(200, 136, 256), (130, 512, 1024), (64, 72, 96), (2500, 2600, 160), (2560, 2560, 128), (2500, 2600, 192)])
def test_hp_gemm_matches_oracle(hero, M, N, K, dt):
    """hero_hp_gemm (Sec. 2.3: a switched module runs in FP16 / BF16) in both 16-bit types.  The last three shapes
    have enough tiles for the persistent kernels (ragged edges, 5 / 4 / 6 slabs, several tiles per workgroup): the
    default choice, then the 256 x 256 and the 128 x 128 form forced."""
    odt, tdt = (O.BF16, torch.bfloat16) if dt == "bf16" else (O.F16, torch.float16)
    enc = lambda a: O.f32_to_hp(a.astype(np.float32), odt)
    dec = lambda u: O.hp_to_f32(u, odt)
    g = synth.rng(1000 + M)
    A, Wt = enc(g.standard_normal((M, K))), enc(g.standard_normal((N, K)) * 0.05)
    bias = (0.1 * g.standard_normal(N)).astype(np.float32)
    res = enc(g.standard_normal((M, N)))
    big = K % 64 == 0 and -(-M // 128) * -(-N // 128) >= 192
    for gelu, r in ((False, None), (True, None), (False, res), (True, res)):
        ref = O.hp_gemm(A, Wt, bias=bias, residual=r, gelu=gelu, dt=odt)
        for tile in (None, 7, 8) if big else (None,):
            got = hero.hero_hp_gemm(dev(A, tdt), dev(Wt, tdt), dev(bias), residual=dev(r, tdt), gelu=gelu, tile=tile)
            assert got.dtype == tdt
            assert rel_err(dec(to_np(got)), dec(ref)) <= 2e-2, (gelu, r is not None, tile)
    if dt == "bf16":                                           # the BF16-only name is the same call
        a = hero.hero_bf16_gemm(dev(A), dev(Wt), dev(bias), residual=dev(res), gelu=True)
        b = hero.hero_hp_gemm(dev(A), dev(Wt), dev(bias), residual=dev(res), gelu=True)
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
@pytest.mark.parametrize("B,S,H,Dh", [(2, 150, 2, 64), (1, 200, 2, 128)])
def test_hp_attn_matches_oracle(hero, B, S, H, Dh, mask, dt):
    odt, tdt = (O.BF16, torch.bfloat16) if dt == "bf16" else (O.F16, torch.float16)
    g = synth.rng(1100 + S)
    qkv = O.f32_to_hp(g.standard_normal((B * S, 3 * H * Dh)).astype(np.float32), odt)
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    kv_len = np.int32([S - 7, 3][:B]) if mask == O.MASK_PADDING else None
    ref = O.hp_attn(qv, kv, vv, scale=1.0 / np.sqrt(Dh), mask=mask, kv_len=kv_len, dt=odt)
    dq = dev(qkv, tdt).view(B, S, 3, H, Dh)
    got = hero.hero_hp_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], 1.0 / np.sqrt(Dh), mask=mask, kv_len=dev(kv_len))
    assert rel_err(O.hp_to_f32(to_np(got), odt), O.hp_to_f32(ref, odt)) <= 2e-2
    if dt == "bf16":
        b = hero.hero_bf16_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], 1.0 / np.sqrt(Dh), mask=mask, kv_len=dev(kv_len))
        assert torch.equal(got.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("Dh", [64, 128])
def test_attention_padded_positions_ask_nothing(hero, Dh):
    """Padding mask in self-attention: the positions i >= kv_len[b] are padding as queries too and their output rows
    are zeros (all bits), in every attention entry point; lengths on and next to the 32-query and 128-query
    boundaries of the kernels' work split, a full row and an empty one; the real rows in their usual classes; the
    outputs are pre-filled so that rows nobody writes would show.  With Sq != Skv the queries are not the padded
    positions and every one of them is answered."""
    B, S, H = 8, 384, 2
    kv_len = np.int32([384, 300, 129, 128, 97, 33, 1, 0])
    pad = (np.arange(S)[None, :] >= kv_len[:, None]).reshape(-1)              # [B*S] rows that are padding
    q, k, v, qk_scale, cs = _attn_case(4100 + Dh, B, S, S, H, Dh)
    sp, sc = float(OL.S_P), np.float32([cs[0]])
    kw = dict(mask=O.MASK_PADDING, kv_len=kv_len)
    dkw = dict(mask=O.MASK_PADDING, kv_len=dev(kv_len))
    fill8 = lambda: torch.full((B * S, H * Dh), 77, dtype=torch.int8, device="cuda")
    fill16 = lambda: torch.full((B * S, H * Dh), 3.0, dtype=torch.bfloat16, device="cuda")
    # two-pass INT8
    ref = O.int8_attn(q, k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=cs, **kw)
    got = to_np(hero.hero_int8_attn(dev(q), dev(k), dev(v), qk_scale, sp, dev(cs), out=fill8(), **dkw))
    assert not ref[pad].any() and not got[pad].any() and np.abs(got[~pad]).max() > 40
    assert_codes(got, ref, "X_attn")
    refb = O.int8_attn(q, k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=sc, out_scale_is_scalar=True, out_dt=O.BF16, **kw)
    gotb = to_np(hero.hero_int8_attn(dev(q), dev(k), dev(v), qk_scale, sp, dev(sc), out_scale_is_scalar=True,
                                     out_dtype=torch.bfloat16, out=fill16(), **dkw))
    assert not refb[pad].any() and not gotb[pad].any()
    assert rel_err(O.bf16_to_f32(gotb), O.bf16_to_f32(refb)) <= 2e-2
    # online variant
    dts = (np.float32(qk_scale) * np.linspace(0.8, 1.3, H)).astype(np.float32)
    ref = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, kv_block=64, **kw)
    got = to_np(hero.hero_int8_attn_online(dev(q), dev(k), dev(v), dev(dts), sp, dev(cs), out=fill8(), **dkw))
    assert not ref[pad].any() and not got[pad].any()
    assert_codes(got, ref, "X_attn online")
    # FP8
    q8, k8, v8, qs8, sp8, cs8 = _fp8_attn_case(4200 + Dh, B, S, S, H, Dh)
    ref = O.fp8_attn(q8, k8, v8, qk_scale=qs8, p_scale=sp8, out_col_scale=cs8, **kw)
    got = to_np(hero.hero_fp8_attn(dev(q8), dev(k8), dev(v8), qs8, sp8, dev(cs8),
                                   out=fill8().view(torch.float8_e4m3fn), **dkw).view(torch.uint8))
    assert not ref[pad].any() and not got[pad].any() and got[~pad].any()
    assert_fp8_attn_codes(got, ref, O.e4m3_to_f32, "X_attn fp8", flip_bound=fp8_attn_flip_bound(q8, k8, v8, qs8, sp8, cs8, mask=1, kv_len=kv_len))
    # 16-bit attention
    g = synth.rng(4300 + Dh)
    for odt, tdt in ((O.BF16, torch.bfloat16), (O.F16, torch.float16)):
        qkv = O.f32_to_hp(g.standard_normal((B * S, 3 * H * Dh)).astype(np.float32), odt)
        qv, kv_, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
        ref = O.hp_attn(qv, kv_, vv, scale=1.0 / np.sqrt(Dh), dt=odt, **kw)
        dq = dev(qkv, tdt).view(B, S, 3, H, Dh)
        got = to_np(hero.hero_hp_attn(dq[:, :, 0], dq[:, :, 1], dq[:, :, 2], 1.0 / np.sqrt(Dh), **dkw))
        assert not ref[pad].any() and not got[pad].any()
        assert rel_err(O.hp_to_f32(got, odt), O.hp_to_f32(ref, odt)) <= 2e-2
    # the queries of a cross-attention (Sq != Skv) are all real
    Sq = 200
    ref = O.int8_attn(q[:, :Sq], k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=cs, **kw)
    got = to_np(hero.hero_int8_attn(dev(q[:, :Sq].copy()), dev(k), dev(v), qk_scale, sp, dev(cs), **dkw))
    assert_codes(got, ref, "X_attn cross")
    assert all(got[b * Sq + 150:(b + 1) * Sq].any() for b in range(B - 1)) and not got[(B - 1) * Sq:].any()


def test_probe_library_instruments():
    """The measuring instruments of the bench (libhero_probe, a library of its own): the copies copy (1 and 4 loads
    in flight, ragged tail, the runtime's copy), the write-only pass writes every element, the MFMA loops report
    their operation counts and leave the sink alone, bad sizes are refused before any launch."""
    from paper_2310_17723_amd.probe import Probe
    pr = Probe()
    n = (1 << 20) + 48
    src = torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda")
    for u in (1, 4):
        dst = torch.zeros_like(src)
        pr.copy(src, dst, u)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
    dst = torch.zeros_like(src)
    pr.memcpy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    dst = torch.full((n,), -1, dtype=torch.int8, device="cuda")
    pr.write(dst)
    torch.cuda.synchronize()
    w = dst.view(torch.int32).view(-1, 4)
    assert bool((w[:, 1] == 1).all() and (w[:, 2] == 2).all() and (w[:, 3] == 3).all())
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    pr.read(src, sink)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for rnd in (0, 1):
        ops = pr.mfma_i8(rnd, 8, sink)
        torch.cuda.synchronize()
        assert ops == cus * 8 * 8 * 16 * 65536.0 and int(sink.item()) == 0
    for mode, V in ((0, 0), (0, 4), (1, 8), (2, 4)):
        mo, vi = pr.coissue(mode, V, 4, sink)
        torch.cuda.synchronize()
        assert vi == cus * 8 * 4 * 8 * V and mo == (0 if mode == 1 else cus * 8 * 4 * 8 * 65536.0) and int(sink.item()) == 0
    with pytest.raises(RuntimeError):
        pr.mfma_i8(0, 0, sink)
    with pytest.raises(RuntimeError):
        pr.copy(src[:24], dst[:24])
    with pytest.raises(RuntimeError):
        pr.coissue(0, 5, 4, sink)
