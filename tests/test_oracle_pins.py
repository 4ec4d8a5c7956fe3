"""Pins for the CPU oracle: each check fixes the oracle to something other than itself
(exact rational arithmetic, closed forms, invariants, brute force, numpy / scipy / torch
library routines).  A dropped term, wrong sign, wrong index or transposed operand in the
oracle fails at least one of them.  No GPU needed."""
from fractions import Fraction
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle as O
from oracle import layer as OL
from paper_2310_17723_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- exact helpers (test-side)
def frac_to_f32(x: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 of an exact rational; normal range."""
    if x == 0:
        return np.float32(0.0)
    s = -1 if x < 0 else 1
    a = abs(x)
    e = math.floor(math.log2(float(a)))
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    assert -126 <= e <= 127
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return np.float32(s * float(fl * ulp))


def rne_int(x: Fraction) -> int:
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def F(x) -> Fraction:
    return Fraction(float(x))


# ---------------------------------------------------------------- 16-bit formats
def test_f16_matches_numpy():
    g = synth.rng(1)
    x = np.concatenate([g.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** g.integers(-9, 5, 20000),
                        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 6.1e-5, 6.0e-8, 2.98e-8, 2.9e-8,
                                  2 ** -14, 2 ** -24, 2 ** -25, 1.0009765625, 1.00048828125, 1.00146484375],
                                 np.float32)])
    with np.errstate(over="ignore"):
        assert np.array_equal(O.f32_to_f16(x), x.astype(np.float16).view(np.uint16))
    h = np.arange(0, 0x7c00, dtype=np.uint16)
    assert np.array_equal(O.f16_to_f32(h), h.view(np.float16).astype(np.float32))


def test_bf16_matches_torch():
    g = synth.rng(2)
    x = np.concatenate([g.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** g.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, 1.00390625, 1.01171875, 1.0078125, 3.3895314e38], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.f32_to_bf16(x), ref)
    assert np.array_equal(O.bf16_to_f32(ref), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


# ---------------------------------------------------------------- O1 quantization primitive
def test_twq_invariants():
    g = synth.rng(3)
    x = (g.standard_normal((64, 200)) * np.exp(g.standard_normal((64, 1)) * 3)).astype(np.float32)
    x[5] = 0.0
    q, s = O.quant_twq(x)
    assert q.min() >= -127 and q.max() <= 127
    amax = np.abs(x).max(axis=1)
    assert s[5] == 1.0 and not q[5].any()
    for i in range(64):
        if i == 5:
            continue
        j = int(np.abs(x[i]).argmax())
        assert abs(int(q[i, j])) == 127                      # the absmax element maps to +-127
        assert np.sign(q[i, j]) == np.sign(x[i, j])
        assert s[i] == np.float32(amax[i]) / np.float32(127.0)
        err = np.abs(x[i].astype(np.float64) - float(s[i]) * q[i].astype(np.float64))
        assert err.max() <= float(s[i]) / 2 * (1 + 1e-6)      # |x - s q| <= s/2
    # re-quantizing the reconstruction with the same scale is the identity
    xr = (s[:, None] * q.astype(np.float32)).astype(np.float32)
    assert np.array_equal(O.quant_static(xr[3:4], float(s[3])), q[3:4])
    # scaling by a power of two changes the scale, not the codes
    q2, s2 = O.quant_twq(x * np.float32(8.0))
    assert np.array_equal(q2, q) and np.array_equal(s2[np.arange(64) != 5], (s * 8)[np.arange(64) != 5])


def test_quant_code_is_rne_of_fp32_quotient_exact_rational():
    """code = rne(fl32(x / s)): the fp32 quotient is the correctly rounded exact quotient,
    then rounded half-to-even to an integer and saturated.  Checked with rationals."""
    g = synth.rng(4)
    xs = g.standard_normal(1500).astype(np.float32) * 3
    ss = np.float32([0.013, 1.0 / 127, 0.5, 0.0234375, 3.1e-3])
    # exact ties: x = (n + 0.5) * s with s a power of two
    ties = np.float32([(n + 0.5) * 0.5 for n in range(-6, 6)])
    for s in ss:
        x = np.concatenate([xs, ties]).astype(np.float32)
        got = O.quant_static(x[None, :], float(s))[0]
        for xv, c in zip(x, got):
            qf = frac_to_f32(F(xv) / F(s))
            exp = max(-127, min(127, rne_int(F(qf))))
            assert int(c) == exp, (xv, s, c, exp)
    assert list(O.quant_static(ties[None, :], 0.5)[0]) == [rne_int(Fraction(2 * n + 1, 2)) for n in range(-6, 6)]
    assert list(O.quant_static(np.float32([[1e6, -1e6, 127.4, -127.6]]), 1.0)[0]) == [127, -127, 127, -127]


def test_fwq_uses_column_scales_and_weight_quant_layout():
    g = synth.rng(5)
    x = g.standard_normal((7, 5)).astype(np.float32)
    cs = np.float32([0.01, 0.02, 0.04, 0.08, 0.16])
    q = O.quant_static(x, cs)
    for j in range(5):
        assert np.array_equal(q[:, j], O.quant_static(x[:, j:j + 1], float(cs[j]))[:, 0])
    # weights: W is [K, N]; codes come back [N, K]; each COLUMN of W has its own scale
    W = g.standard_normal((6, 4)).astype(np.float32) * np.float32([1, 10, 100, 1000])
    Wt, s = O.weight_quant(W)
    assert Wt.shape == (4, 6) and s.shape == (4,)
    for n in range(4):
        qn, sn = O.quant_twq(W[:, n][None, :])
        assert np.array_equal(Wt[n], qn[0]) and s[n] == sn[0]
        assert np.abs(Wt[n]).max() == 127
    assert np.allclose(Wt.T.astype(np.float64) * s, W, atol=float(s.max()) / 2 * 1.000001)


# ---------------------------------------------------------------- O3 integer GEMM
def test_weight_fold_quant_and_absmax_cols():
    """Fold + column-wise quantization (Sec. 2.2.2 / 2.2.3 folds, Sec. 2.1 column scales) and the calibration
    statistic.  Pins: power-of-two multipliers fold exactly, so the codes must equal those of the unfolded
    matrix and the scales shift by the same powers; an exact-rational re-derivation of every code on a small
    matrix; the half-step property codes * scale ~ folded W; brute-force column maxima."""
    g = synth.rng(13)
    K, N = 24, 10
    W = g.standard_normal((K, N)).astype(np.float32)
    q0, s0 = O.weight_quant(W)
    rm = np.float32(2.0) ** g.integers(-3, 4, K)
    cd = np.float32(2.0) ** g.integers(-3, 4, N)
    q1, s1 = O.weight_fold_quant(W, None, cd)
    assert np.array_equal(q1, q0) and np.array_equal(s1, s0 / cd)
    # general multipliers: exact rationals
    rm = g.uniform(0.01, 2.0, K).astype(np.float32)
    cd = g.uniform(0.01, 2.0, N).astype(np.float32)
    q, s = O.weight_fold_quant(W, rm, cd)
    assert q.shape == (N, K) and s.shape == (N,)
    fr = lambda v: Fraction(float(v))
    for n in range(N):
        col = []
        for k in range(K):
            t = float(np.float64(rm[k]) * np.float64(W[k, n]))             # fp64 product, then fp64 quotient, then fp32
            col.append(np.float32(np.float64(t) / np.float64(cd[n])))
        amax = max(abs(float(c)) for c in col)
        sc = np.float32(np.float32(amax) / np.float32(127))
        assert s[n] == sc
        for k in range(K):
            quo = np.float32(col[k]) / sc                                   # IEEE fp32 quotient
            exact = fr(quo)
            lo = math.floor(exact)
            code = lo if exact - lo < Fraction(1, 2) else lo + 1 if exact - lo > Fraction(1, 2) else lo + (lo % 2)
            assert q[n, k] == max(-127, min(127, code))
        exactW = [fr(rm[k]) * fr(W[k, n]) / fr(cd[n]) for k in range(K)]
        assert all(abs(Fraction(int(q[n, k])) * fr(s[n]) - exactW[k]) <= fr(s[n]) * Fraction(501, 1000) for k in range(K))
    # only the row multipliers / nothing at all
    q2, s2 = O.weight_fold_quant(W, rm, None)
    q3, s3 = O.weight_quant((rm[:, None].astype(np.float64) * W).astype(np.float32))
    assert np.array_equal(q2, q3) and np.array_equal(s2, s3)
    assert all(np.array_equal(a, b) for a, b in zip(O.weight_fold_quant(W), (q0, s0)))
    # calibration statistic: brute force, running maximum, sign-insensitive
    x = g.standard_normal((17, 6)).astype(np.float32)
    m = O.absmax_cols(x)
    assert all(m[j] == max(abs(float(x[i, j])) for i in range(17)) for j in range(6))
    run = np.float32([0, 10, 0, 0.5, 0, 0])
    assert np.array_equal(O.absmax_cols(x, run), np.maximum(m, run)) and np.array_equal(O.absmax_cols(-x), m)


def test_gemm_int_exact():
    g = synth.rng(6)
    A = g.integers(-127, 128, (37, 200), dtype=np.int8)
    Bt = g.integers(-127, 128, (29, 200), dtype=np.int8)
    ref = A.astype(np.int64) @ Bt.astype(np.int64).T
    assert np.array_equal(O.gemm_i64(A, Bt), ref)
    assert np.array_equal(O.gemm_i32(A, Bt).astype(np.int64), ref)
    # one-hot operands pick single entries: C[i][j] = Bt[j][k_i]
    A1 = np.zeros((5, 200), np.int8)
    ks = [0, 3, 64, 150, 199]
    for i, k in enumerate(ks):
        A1[i, k] = 1
    assert np.array_equal(O.gemm_i32(A1, Bt), Bt[:, ks].T.astype(np.int32))
    # the largest magnitude any config can reach stays inside int32
    K = 16384
    C = O.gemm_i32(np.full((1, K), 127, np.int8), np.full((2, K), -127, np.int8))
    assert C[0, 0] == -127 * 127 * K and abs(int(C[0, 0])) < 2 ** 31


# ---------------------------------------------------------------- O4 epilogues
def test_gelu_against_scipy():
    xs = np.linspace(-8, 8, 4001)
    ref = 0.5 * xs * (1 + scipy.special.erf(xs / math.sqrt(2)))
    got = np.array([O.gelu(v) for v in xs])
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-17)
    assert O.gelu(0.0) == 0.0
    for v in (0.3, 1.7, 5.0):
        assert abs(O.gelu(v) - O.gelu(-v) - v) < 1e-15


def test_epilogue_power_of_two_scales_are_integer_shifts():
    g = synth.rng(7)
    M, N, K = 9, 11, 64
    A = g.integers(-127, 128, (M, K), dtype=np.int8)
    Bt = g.integers(-127, 128, (N, K), dtype=np.int8)
    acc = A.astype(np.int64) @ Bt.astype(np.int64).T
    rs = np.float32(2.0) ** g.integers(-6, -2, M).astype(np.float32)
    cs = np.float32(2.0) ** g.integers(-8, -4, N).astype(np.float32)
    bias = g.integers(-40, 40, N).astype(np.float32) / 4
    got = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_REQUANT, c_dt=O.I8)
    for i in range(M):
        for j in range(N):
            y = Fraction(int(acc[i, j])) * F(rs[i]) * F(cs[j]) + F(bias[j])
            assert int(got[i, j]) == max(-127, min(127, rne_int(y)))
    # no row scale (FWQ folded into the weight): y = acc * cs + bias
    got = O.int8_gemm(A, Bt, b_col_scale=cs, bias=None, epi=O.EPI_REQUANT, c_dt=O.I8)
    for i in range(M):
        for j in range(N):
            assert int(got[i, j]) == max(-127, min(127, rne_int(Fraction(int(acc[i, j])) * F(cs[j]))))


def test_epilogue_general_scales_exact_rational_and_16bit_outputs():
    g = synth.rng(8)
    M, N, K = 6, 10, 4096
    c = synth.gemm_case(8, M, K, N)
    A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
    acc = A.astype(np.int64) @ Bt.astype(np.int64).T
    assert np.abs(acc).max() > 2 ** 17
    res = O.f32_to_bf16(g.standard_normal((M, N)).astype(np.float32))
    y = np.empty((M, N), np.float32)
    for i in range(M):
        for j in range(N):
            t = frac_to_f32(Fraction(int(acc[i, j])))                 # int32 -> fp32, RNE
            t = frac_to_f32(F(t) * F(rs[i]))
            y[i, j] = frac_to_f32(F(t) * F(cs[j]) + F(bias[j]))        # single-rounded fma
    f32 = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32)
    assert np.array_equal(f32, y)
    bf = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.BF16)
    assert np.array_equal(bf, torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    hf = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F16)
    assert np.array_equal(hf, y.astype(np.float16).view(np.uint16))
    # residual is added in fp32 after the fma, then one rounding to bf16
    yr = np.empty_like(y)
    rf = O.bf16_to_f32(res)
    for i in range(M):
        for j in range(N):
            yr[i, j] = frac_to_f32(F(y[i, j]) + F(rf[i, j]))
    bfr = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                      epi=O.EPI_DEQUANT, c_dt=O.BF16)
    assert np.array_equal(bfr, torch.from_numpy(yr).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    # GELU epilogues: fp64 erf GELU of the fp32 pre-activation (scipy as the library pin)
    gl = (0.5 * y.astype(np.float64) * (1 + scipy.special.erf(y.astype(np.float64) / math.sqrt(2)))).astype(np.float32)
    sa = (np.abs(gl).max(axis=0) / 127 + 1e-6).astype(np.float32)
    gq = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=sa, c_dt=O.I8)
    assert np.array_equal(gq, O.quant_static(gl, sa))
    gb = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
    assert np.array_equal(gb, gl)
    with pytest.raises(ValueError):
        O.int8_gemm(A, Bt, b_col_scale=cs, epi=O.EPI_REQUANT, c_dt=O.BF16)


# ---------------------------------------------------------------- O4f FP8 variant
def test_fp8_e4m3_format_quantizer_and_gemm():
    """Pins for the FP8 (OCP E4M3) variant: the format against torch's float8_e4m3fn (all 256 codes decoded, a dense
    sweep encoded; torch has no saturation, so values beyond 448 are checked against the rule), the token-wise
    quantizer against its defining properties, the GEMM against a float64 matmul of the decoded operands and an
    exact-rational epilogue."""
    codes = np.arange(256, dtype=np.uint8)
    dec = O.e4m3_to_f32(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    assert np.array_equal(np.isnan(dec), np.isnan(ref)) and np.array_equal(dec[~np.isnan(dec)], ref[~np.isnan(ref)])
    assert dec[0x7E] == 448 and dec[0x01] == 2.0 ** -9 and dec[0x08] == 2.0 ** -6 and np.isnan(dec[0x7F])
    fin = ~np.isnan(dec)
    assert np.array_equal(O.f32_to_e4m3(dec[fin]) & 0x7F, codes[fin] & 0x7F)          # every finite code round-trips
    g = synth.rng(14)
    x = np.concatenate([g.standard_normal(20000) * np.exp(g.uniform(-8, 6, 20000)), dec[fin],
                        (dec[fin][:-1] + dec[fin][1:]) / 2]).astype(np.float32)        # incl. exact ties
    x = x[np.abs(x) <= 448]
    enc = O.f32_to_e4m3(x)
    tref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    nz = x != 0
    assert np.array_equal(enc[nz], tref[nz]) and np.array_equal(enc[~nz] & 0x7F, tref[~nz] & 0x7F)
    big = np.float32([449, 463.9, 464, 1e9, np.inf, -470, -np.inf])
    assert np.array_equal(O.f32_to_e4m3(big), np.uint8([0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE]))
    assert O.f32_to_e4m3(np.float32([np.nan]))[0] & 0x7F == 0x7F
    # token-wise quantizer: scale = absmax / 448, the absmax element maps to +-448, error within half a step
    X = (g.standard_normal((9, 64)) * g.uniform(0.1, 30, (9, 1))).astype(np.float32)
    X[3] = 0
    q, s = O.quant_twq_fp8(X)
    amax = np.abs(X).max(axis=1)
    assert np.array_equal(s, np.where(amax == 0, np.float32(1), amax / np.float32(448)).astype(np.float32))
    dq = O.e4m3_to_f32(q)
    assert (np.abs(dq).max(axis=1)[amax > 0] == 448).all() and (dq[3] == 0).all()
    for i in range(9):
        for j in range(64):
            t = np.float32(X[i, j]) / s[i]
            assert q[i, j] == O.f32_to_e4m3(np.float32([t]))[0]
            step = max(2.0 ** (math.floor(math.log2(max(abs(float(t)), 2.0 ** -6))) - 3), 2.0 ** -9)
            assert abs(float(dq[i, j]) - float(t)) <= step / 2 * (1 + 1e-6)
    # GEMM: float64 matmul of the decoded operands (products of two E4M3 values are exact in fp64, so is their sum here)
    M, N, K = 5, 7, 256
    A = O.f32_to_e4m3(g.standard_normal((M, K)).astype(np.float32) * 3)
    Bt = O.f32_to_e4m3(g.standard_normal((N, K)).astype(np.float32) * 3)
    acc = O.e4m3_to_f32(A).astype(np.float64) @ O.e4m3_to_f32(Bt).astype(np.float64).T
    rs = g.uniform(0.01, 0.1, M).astype(np.float32)
    cs = g.uniform(0.01, 0.1, N).astype(np.float32)
    bias = g.standard_normal(N).astype(np.float32)
    y = np.empty((M, N), np.float32)
    for i in range(M):
        for j in range(N):
            t = frac_to_f32(Fraction(float(acc[i, j])))
            t = frac_to_f32(F(t) * F(rs[i]))
            y[i, j] = frac_to_f32(F(t) * F(cs[j]) + F(bias[j]))
    assert np.array_equal(O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.F32), y)
    assert np.array_equal(O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_REQUANT, c_dt=O.F8),
                          O.f32_to_e4m3(y))
    bf = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_DEQUANT, c_dt=O.BF16)
    assert np.array_equal(bf, torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    gl = (0.5 * y.astype(np.float64) * (1 + scipy.special.erf(y.astype(np.float64) / math.sqrt(2)))).astype(np.float32)
    sa = (np.abs(gl).max(axis=0) / 448 + 1e-6).astype(np.float32)
    gq = O.fp8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=sa, c_dt=O.F8)
    assert np.array_equal(gq, O.f32_to_e4m3((gl / sa[None, :]).astype(np.float32)))
    # one-hot rows pick single weights: operand layout
    A1 = np.zeros((3, K), np.uint8); ks = [5, 100, 255]
    for i, k in enumerate(ks):
        A1[i, k] = 0x38                                                               # 1.0
    one = np.ones(N, np.float32)
    assert np.array_equal(O.fp8_gemm(A1, Bt, b_col_scale=one, epi=O.EPI_DEQUANT, c_dt=O.F32), O.e4m3_to_f32(Bt)[:, ks].T)
    with pytest.raises(ValueError):
        O.fp8_gemm(A, Bt, b_col_scale=cs, epi=O.EPI_REQUANT, c_dt=O.BF16)


# ---------------------------------------------------------------- O5 LN^quant
def test_ln_quant_fp8_output_against_torch_and_the_fp8_quantizer():
    """LN^quant with a token-wise E4M3 output: without a LayerNorm it is the (pinned) FP8 token-wise quantizer;
    with one, torch's fp64 layer_norm followed by torch's own float8_e4m3fn rounding of y / (max|y| / 448)."""
    g = synth.rng(40)
    M, D = 11, 96
    X = (g.standard_normal((M, D)) * g.uniform(0.2, 5, (M, 1))).astype(np.float32)
    q0, s0 = O.quant_twq_fp8(X)
    q1, s1, _ = O.ln_quant(X, O.F32, None, None, 0, None, None, None, 0.0, fp8=True)
    assert np.array_equal(q0, q1) and np.array_equal(s0, s1)
    xq = g.integers(-127, 128, (M, D), dtype=np.int8)
    rq = g.integers(-127, 128, (M, D), dtype=np.int8)
    xs = g.uniform(0.005, 0.05, M).astype(np.float32)
    rc = g.uniform(0.001, 0.02, D).astype(np.float32)
    gam = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
    bet = (0.02 * g.standard_normal(D)).astype(np.float32)
    q, sc, hp = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, 1e-5, y_hp_dt=O.BF16, fp8=True)
    ssum = torch.from_numpy(xq.astype(np.float64) * xs[:, None].astype(np.float64) + rq.astype(np.float64) * rc[None, :].astype(np.float64))
    y = torch.nn.functional.layer_norm(ssum, (D,), torch.from_numpy(gam).double(), torch.from_numpy(bet).double(), 1e-5).float()
    s_ref = (y.abs().amax(dim=1) / 448).numpy()
    np.testing.assert_allclose(sc, s_ref, rtol=2e-7)
    c_ref = (y / torch.from_numpy(sc)[:, None]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.count_nonzero(q != c_ref) <= 2                      # a last-bit difference of y next to a rounding boundary
    dq = O.e4m3_to_f32(q)
    assert (np.abs(dq).max(axis=1) == 448).all()
    assert np.array_equal(hp, torch.from_numpy(O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, 1e-5, y_hp_dt=O.BF16)[2].astype(np.int16)).numpy().view(np.uint16))


def test_ln_quant_closed_forms_and_torch():
    g = synth.rng(9)
    M, D = 12, 96
    xq = g.integers(-127, 128, (M, D), dtype=np.int8)
    rq = g.integers(-127, 128, (M, D), dtype=np.int8)
    xs = g.uniform(0.01, 0.05, M).astype(np.float32)          # per ROW
    rc = g.uniform(0.001, 0.2, D).astype(np.float32)          # per COLUMN
    one, zero = np.ones(D, np.float32), np.zeros(D, np.float32)
    eps = 1e-3
    q, s, y = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, one, zero, eps, y_hp_dt=O.F32)
    r = xs[:, None].astype(np.float64) * xq + rc[None, :].astype(np.float64) * rq
    var = r.var(axis=1)
    assert np.allclose(y.astype(np.float64).mean(axis=1), 0, atol=1e-7)
    assert np.allclose(y.astype(np.float64).var(axis=1), var / (var + eps), rtol=1e-6)
    # library pin: torch fp64 layer_norm of the dequantized sum, with gain and bias
    gam = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
    bet = (0.02 * g.standard_normal(D)).astype(np.float32)
    q, s, y = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, eps, y_hp_dt=O.F32)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(r), (D,), torch.from_numpy(gam).double(),
                                         torch.from_numpy(bet).double(), eps).numpy()
    assert np.allclose(y, ref.astype(np.float32), rtol=0, atol=2e-7 * np.abs(ref).max())
    assert np.abs(y.astype(np.float64) - ref).max() <= 2.0 ** -24 * np.abs(ref).max() * 1.01
    # the codes are the TWQ primitive applied to y
    q2, s2 = O.quant_twq(y)
    assert np.array_equal(q, q2) and np.array_equal(s, s2)
    # two-element rows: y = +-1/sqrt(1 + eps/sigma^2)
    x2 = np.float32([[3.0, 1.0], [-2.0, 6.0]])
    _, _, y2 = O.ln_quant(x2, O.F32, None, None, 0, None, np.ones(2, np.float32), np.zeros(2, np.float32), 0.25,
                          y_hp_dt=O.F32)
    for row, (a, b) in zip(y2, x2):
        sig2 = ((a - b) / 2) ** 2
        v = 1 / math.sqrt(1 + 0.25 / sig2)
        assert np.allclose(row, [math.copysign(v, a - b), math.copysign(v, b - a)], rtol=1e-7)
    # gamma = None: pure per-token quantization of the (bf16) input
    hb = O.f32_to_bf16(g.standard_normal((4, 32)).astype(np.float32))
    q3, s3, _ = O.ln_quant(hb, O.BF16, None, None, 0, None, None, None, 0.0)
    q4, s4 = O.quant_twq(O.bf16_to_f32(hb))
    assert np.array_equal(q3, q4) and np.array_equal(s3, s4)
    # bf16 second addend and bf16 copy of y
    rb = O.f32_to_bf16(g.standard_normal((M, D)).astype(np.float32))
    q5, s5, y5 = O.ln_quant(xq, O.I8, xs, rb, O.BF16, None, gam, bet, eps, y_hp_dt=O.BF16)
    r5 = xs[:, None].astype(np.float64) * xq + O.bf16_to_f32(rb).astype(np.float64)
    ref5 = torch.nn.functional.layer_norm(torch.from_numpy(r5), (D,), torch.from_numpy(gam).double(),
                                          torch.from_numpy(bet).double(), eps).float()
    assert np.array_equal(y5, ref5.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)) or \
        np.mean(y5 != ref5.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)) < 2e-3


# ---------------------------------------------------------------- O5b embedding LN^quant
def test_embed_ln_quant_against_torch_and_invariants():
    """Sec. 2.2.1.  Pins that do not go through the oracle's own arithmetic: torch's embedding lookups and
    fp64 layer_norm for the value that is quantized; the half-step property of a round-to-nearest code
    (|y_q s - y| <= s/2) and s = max|y| / 127 for the quantization; a permutation of the tokens permutes the
    outputs; dropping any of the three addends changes the result (each term is really there)."""
    d, V, P, NT, B, S = 96, 500, 40, 2, 3, 40
    tb = synth.embedding_tables(3, d, V, P, NT)
    ids = synth.embedding_ids(4, B, S, V, NT)
    tq, ts = O.quant_twq(tb["tok"])                                   # INT8 token table, one scale per row
    pos16, typ16 = O.f32_to_bf16(tb["pos"]), O.f32_to_bf16(tb["type"])
    g = synth.rng(5)
    gam = (1 + 0.1 * g.standard_normal(d)).astype(np.float32)
    bet = (0.02 * g.standard_normal(d)).astype(np.float32)
    eps = 1e-6
    q, s = O.embed_ln_quant(ids["tok"], ids["pos"], ids["type"], tq, ts, pos16, typ16, O.BF16, gam, bet, eps)
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    tok64 = t(ts.astype(np.float64)[:, None] * tq.astype(np.float64))
    h = F.embedding(t(ids["tok"]).long(), tok64) + F.embedding(t(ids["pos"]).long(), t(O.bf16_to_f32(pos16)).double()) \
        + F.embedding(t(ids["type"]).long(), t(O.bf16_to_f32(typ16)).double())
    y = F.layer_norm(h, (d,), t(gam).double(), t(bet).double(), eps).numpy()
    amax = np.abs(y).max(axis=1)
    assert np.allclose(s, amax / 127, rtol=3e-7, atol=0)
    assert (np.abs(q) <= 127).all() and (np.abs(q).max(axis=1) == 127).all()
    err = np.abs(q.astype(np.float64) * s[:, None].astype(np.float64) - y)
    assert (err <= 0.5 * s[:, None] * (1 + 1e-5) + 1e-7 * amax[:, None]).all()
    # f32 tables, no type table
    q2, s2 = O.embed_ln_quant(ids["tok"], ids["pos"], None, tq, ts, tb["pos"], None, O.F32, gam, None, eps)
    h2 = F.embedding(t(ids["tok"]).long(), tok64) + F.embedding(t(ids["pos"]).long(), t(tb["pos"]).double())
    y2 = F.layer_norm(h2, (d,), t(gam).double(), None, eps).numpy()
    assert np.allclose(s2, np.abs(y2).max(axis=1) / 127, rtol=3e-7, atol=0)
    assert (np.abs(q2.astype(np.float64) * s2[:, None] - y2) <= 0.5 * s2[:, None] * (1 + 1e-5) + 1e-7).all()
    assert not np.array_equal(q, q2)                                  # the type rows matter
    qz, _ = O.embed_ln_quant(ids["tok"], np.zeros_like(ids["pos"]), ids["type"], tq, ts, pos16, typ16, O.BF16, gam, bet, eps)
    assert not np.array_equal(q, qz)                                  # ... and so do the position rows
    # permuting the tokens permutes the rows of the output
    perm = g.permutation(B * S)
    qp, sp = O.embed_ln_quant(ids["tok"][perm], ids["pos"][perm], ids["type"][perm], tq, ts, pos16, typ16, O.BF16, gam, bet, eps)
    assert np.array_equal(qp, q[perm]) and np.array_equal(sp, s[perm])
    bad = ids["tok"].copy(); bad[7] = V
    with pytest.raises(ValueError):
        O.embed_ln_quant(bad, ids["pos"], ids["type"], tq, ts, pos16, typ16, O.BF16, gam, bet, eps)
    with pytest.raises(ValueError):
        O.embed_ln_quant(ids["tok"], ids["pos"], None, tq, ts, pos16, typ16, O.BF16, gam, bet, eps)


# ---------------------------------------------------------------- O6 attention
def _attn_inputs(seed, B, Sq, Skv, H, Dh):
    g = synth.rng(seed)
    q = g.integers(-127, 128, (B, Sq, H, Dh), dtype=np.int8)
    k = g.integers(-127, 128, (B, Skv, H, Dh), dtype=np.int8)
    v = g.integers(-127, 128, (B, Skv, H, Dh), dtype=np.int8)
    return q, k, v


def test_attention_closed_forms():
    B, S, H, Dh = 1, 7, 2, 8
    q, k, v = _attn_inputs(10, B, S, S, H, Dh)
    one = np.ones(H * Dh, np.float32)
    # equal scores -> p = 1/n -> every code rne(255/n)
    out, P = O.int8_attn(np.zeros_like(q), k, v, qk_scale=0.01, p_scale=float(OL.S_P), out_col_scale=one,
                         mask=O.MASK_CAUSAL, out_dt=O.F32, out_scale_is_scalar=True, dump_p=True)
    for i in range(S):
        n = i + 1
        code = int(np.float32(np.float32(1.0 / n) / OL.S_P).round())
        assert (P[0, :, i, :n] == code).all() and (P[0, :, i, n:] == 0).all()
        for h in range(H):       # causal = attention over the prefix, by brute force
            exp = code * v[0, :n, h, :].astype(np.int64).sum(axis=0)
            assert np.array_equal(out[i, h * Dh:(h + 1) * Dh], exp.astype(np.float32))
    # one dominant score -> 255 at the argmax, 0 elsewhere -> output = 255 * that V row
    qd = np.zeros_like(q)
    kd = np.zeros_like(k)
    qd[..., 0] = 127
    kd[0, 4, :, 0] = 127
    out, P = O.int8_attn(qd, kd, v, qk_scale=0.01, p_scale=float(OL.S_P), out_col_scale=one, out_dt=O.F32,
                         out_scale_is_scalar=True, dump_p=True)
    assert (P[..., 4] == 255).all() and P.sum() == 255 * H * S
    assert np.array_equal(out[:, :Dh], np.repeat(255.0 * v[0, 4:5, 0, :], S, axis=0).astype(np.float32))
    # constant V columns -> output = v_e * sum_k P  (INT8 output with a per-column scale)
    vc = np.repeat(np.repeat(np.arange(1, Dh + 1, dtype=np.int8)[None, None, None, :], S, 1), H, 2)
    cs = np.linspace(0.001, 0.004, H * Dh).astype(np.float32)
    out, P = O.int8_attn(q, k, vc, qk_scale=3e-4, p_scale=float(OL.S_P), out_col_scale=cs, out_dt=O.I8, dump_p=True)
    ps = P.astype(np.int64).sum(axis=-1)
    assert (np.abs(ps - 255) <= S / 2).all()                       # sum of codes = 255 +- n/2
    for i in range(S):
        for h in range(H):
            for e in range(Dh):
                y = frac_to_f32(F(frac_to_f32(Fraction(int(ps[0, h, i]) * (e + 1)))) * F(cs[h * Dh + e]))
                assert int(out[i, h * Dh + e]) == max(-127, min(127, rne_int(F(y))))


@pytest.mark.parametrize("mask,Sq", [(O.MASK_NONE, 9), (O.MASK_PADDING, 9), (O.MASK_PADDING, 7), (O.MASK_CAUSAL, 9)])
def test_attention_against_scipy_softmax(mask, Sq):
    """The mask rules written out independently: key k < kv_len[b]; causal k <= i + (len - Sq); with the padding
    mask in self-attention (Sq == Skv) a position i >= kv_len[b] is padding as a query too and sees no key, while
    with Sq != Skv (the queries are not the padded positions) every query sees the valid keys."""
    B, Skv, H, Dh = 3, 9, 2, 16
    q, k, v = _attn_inputs(11, B, Sq, Skv, H, Dh)
    kv_len = np.int32([9, 5, 0]) if mask == O.MASK_PADDING else (np.int32([9, 6, 3]) if mask == O.MASK_CAUSAL else None)
    d_t, sp = np.float32(2.5e-4), OL.S_P
    cs = synth.rng(12).uniform(2e-5, 6e-5, H * Dh).astype(np.float32)
    out, P = O.int8_attn(q, k, v, qk_scale=float(d_t), p_scale=float(sp), out_col_scale=cs, mask=mask,
                         kv_len=kv_len, out_dt=O.I8, dump_p=True)
    for b in range(B):
        L = Skv if kv_len is None else int(kv_len[b])
        for h in range(H):
            acc = q[b, :, h].astype(np.int64) @ k[b, :, h].astype(np.int64).T
            a = acc.astype(np.float32) * d_t
            for i in range(Sq):
                n = L if mask != O.MASK_CAUSAL else min(L, i + (L - Sq) + 1)
                n = max(n, 0)
                if mask == O.MASK_PADDING and Sq == Skv and i >= L:
                    n = 0
                codes = np.zeros(Skv, np.int64)
                if n > 0:
                    p = scipy.special.softmax(a[i, :n].astype(np.float64)).astype(np.float32)
                    codes[:n] = np.clip(np.rint(p / sp), 0, 255).astype(np.int64)
                assert np.array_equal(P[b, h, i], codes.astype(np.uint8))
                pv = codes @ v[b, :, h].astype(np.int64)
                y = pv.astype(np.float32) * cs[h * Dh:(h + 1) * Dh]
                exp = np.clip(np.rint(y), -127, 127).astype(np.int8)
                assert np.array_equal(out[b * Sq + i, h * Dh:(h + 1) * Dh], exp)
    if mask == O.MASK_PADDING:
        assert not out[2 * Sq:].any()            # a batch row with no visible key outputs 0
        assert out[Sq:Sq + 5].any()
        assert out[Sq + 5:2 * Sq].any() == (Sq != Skv)     # positions 5.. of the length-5 row: padding only in self-attention


def test_attention_strided_views_and_offset_identity():
    """q/k/v as views into a fused [T, 3d] buffer and k/v from a [B,H,Smax,Dh] cache give
    the same result as contiguous copies; P_u8 V = (P_u8 - 128) V + 128 colsum(V)."""
    B, S, H, Dh = 2, 6, 3, 8
    g = synth.rng(13)
    qkv = g.integers(-127, 128, (B * S, 3 * H * Dh), dtype=np.int8)
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    cs = np.full(H * Dh, 4e-5, np.float32)
    kw = dict(qk_scale=3e-4, p_scale=float(OL.S_P), out_col_scale=cs, mask=O.MASK_CAUSAL)
    a = O.int8_attn(qv, kv, vv, **kw)
    b = O.int8_attn(qv.copy(), kv.copy(), vv.copy(), **kw)
    assert np.array_equal(a, b)
    cache_k = np.zeros((B, H, S + 3, Dh), np.int8)
    cache_v = np.zeros((B, H, S + 3, Dh), np.int8)
    cache_k[:, :, :S] = kv.transpose(0, 2, 1, 3)
    cache_v[:, :, :S] = vv.transpose(0, 2, 1, 3)
    c = O.int8_attn(qv, cache_k.transpose(0, 2, 1, 3), cache_v.transpose(0, 2, 1, 3), kv_len=np.int32([S, S]), **kw)
    assert np.array_equal(a, c)
    _, P = O.int8_attn(qv, kv, vv, dump_p=True, **kw)
    Pi = P.astype(np.int64)
    V = vv.transpose(0, 2, 1, 3).astype(np.int64)
    assert np.array_equal(Pi @ V, (Pi - 128) @ V + 128 * V.sum(axis=2, keepdims=True))


def _f8(x):
    """torch's own E4M3 rounding (independent of the oracle's codec), as bytes."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def _f8_dec(c):
    return torch.from_numpy(np.ascontiguousarray(c, np.uint8)).view(torch.float8_e4m3fn).float().numpy()


def test_fp8_attention_closed_forms():
    """Sec. 2.2.2 with E4M3 codes: one visible key -> code 448 -> the V row itself; equal scores over n = 2^j keys
    -> every code 448 / n exactly -> the mean of the V rows; masks by truncation."""
    B, S, H, Dh = 1, 8, 2, 16
    g = synth.rng(70)
    q = _f8(g.standard_normal((B, S, H, Dh)) * 2)
    k = _f8(g.standard_normal((B, S, H, Dh)) * 2)
    v = _f8(g.integers(-8, 9, (B, S, H, Dh)).astype(np.float32))          # small integers: sums are exact
    sp = np.float32(1.0 / 448.0)
    vf = _f8_dec(v)
    # causal, zero queries: query i averages the first i + 1 rows of V; 448 / n is a code for n = 1, 2, 4, 8
    out, P = O.fp8_attn(np.zeros_like(q), k, v, qk_scale=0.05, p_scale=float(sp), out_col_scale=np.float32([sp]),
                        out_scale_is_scalar=True, mask=O.MASK_CAUSAL, out_dt=O.F32, dump_p=True)
    for i in (0, 1, 3, 7):
        n = i + 1
        assert (_f8_dec(P[0, :, i, :n]) == 448.0 / n).all() and (P[0, :, i, n:] == 0).all()
        for h in range(H):
            acc = (448.0 / n * vf[0, :n, h, :].astype(np.float64).sum(axis=0)).astype(np.float32)     # exact
            np.testing.assert_array_equal(out[i, h * Dh:(h + 1) * Dh], acc * sp)                       # ~ the mean (S_p is not 2^-j)
            np.testing.assert_allclose(out[i, h * Dh:(h + 1) * Dh], vf[0, :n, h, :].mean(axis=0), rtol=2e-7, atol=0)
    # n = 3: 448 / 3 = 149.33 rounds to the code 144 (step 16 between 128 and 256)
    assert (_f8_dec(P[0, :, 2, :3]) == 144.0).all()
    # a dominant score: code 448 at the argmax, 0 elsewhere (exp(-huge) / S_p underflows the smallest subnormal 2^-9)
    qd = np.zeros((B, S, H, Dh), np.float32); kd = np.zeros((B, S, H, Dh), np.float32)
    qd[..., 0] = 16.0; kd[0, 5, :, 0] = 16.0
    out, P = O.fp8_attn(_f8(qd), _f8(kd), v, qk_scale=1.0, p_scale=float(sp), out_col_scale=np.float32([sp]),
                        out_scale_is_scalar=True, out_dt=O.F32, dump_p=True)
    assert (_f8_dec(P[..., 5]) == 448.0).all() and np.count_nonzero(P) == H * S
    np.testing.assert_array_equal(out[:, :Dh], np.repeat((448.0 * vf[0, 5:6, 0, :]).astype(np.float32) * sp, S, axis=0))
    # padding: kv_len = 0 -> zeros; E4M3 output with per-column scales = torch's rounding of acc * c[j]
    cs = g.uniform(0.5, 2.0, H * Dh).astype(np.float32) * sp
    o8 = O.fp8_attn(q, k, v, qk_scale=0.05, p_scale=float(sp), out_col_scale=cs, mask=O.MASK_PADDING, kv_len=np.int32([0]))
    assert not o8.any()
    o8, P = O.fp8_attn(q, k, v, qk_scale=0.05, p_scale=float(sp), out_col_scale=cs, dump_p=True)
    acc = np.einsum("bhik,bkhe->bihe", _f8_dec(P).astype(np.float64), vf.astype(np.float64)).reshape(B * S, H * Dh)
    np.testing.assert_array_equal(o8, _f8(acc.astype(np.float32) * cs[None, :]))


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
def test_fp8_attention_against_scipy_softmax_and_torch_rounding(mask):
    """Every step re-done with numpy / scipy / torch: decoded operands, fp64 scores rounded once, scipy softmax,
    torch's E4M3 rounding of p / S_p, fp64 PV rounded once, torch's rounding of the scaled output."""
    B, Sq, Skv, H, Dh = 3, 9, 9, 2, 32
    g = synth.rng(71)
    q = _f8(g.standard_normal((B, Sq, H, Dh)) * 3); k = _f8(g.standard_normal((B, Skv, H, Dh)) * 3)
    v = _f8(g.standard_normal((B, Skv, H, Dh)) * 5)
    kv_len = np.int32([9, 5, 0]) if mask == O.MASK_PADDING else (np.int32([9, 6, 3]) if mask == O.MASK_CAUSAL else None)
    d_t, sp = np.float32(0.02), np.float32(1.0 / 448.0)
    cs = g.uniform(0.5, 2.0, H * Dh).astype(np.float32) * sp * np.float32(20.0)
    out, P = O.fp8_attn(q, k, v, qk_scale=float(d_t), p_scale=float(sp), out_col_scale=cs, mask=mask, kv_len=kv_len, dump_p=True)
    qf, kf, vf = (_f8_dec(t).astype(np.float64) for t in (q, k, v))
    flips = 0
    for b in range(B):
        L = Skv if kv_len is None else int(kv_len[b])
        for h in range(H):
            a = (qf[b, :, h] @ kf[b, :, h].T).astype(np.float32) * d_t
            for i in range(Sq):
                n = max(L if mask != O.MASK_CAUSAL else min(L, i + (L - Sq) + 1), 0)
                if mask == O.MASK_PADDING and Sq == Skv and i >= L:
                    n = 0                            # self-attention: a padded position asks nothing
                codes = np.zeros(Skv, np.uint8)
                if n > 0:
                    p = scipy.special.softmax(a[i, :n].astype(np.float64)).astype(np.float32)
                    codes[:n] = _f8(p / sp)
                # scipy's softmax and the oracle's may differ in the last bit of p next to a rounding boundary
                flips += np.count_nonzero(P[b, h, i] != codes)
                pv = (_f8_dec(P[b, h, i]).astype(np.float64) @ vf[b, :, h]).astype(np.float32)
                np.testing.assert_array_equal(out[b * Sq + i, h * Dh:(h + 1) * Dh], _f8(pv * cs[h * Dh:(h + 1) * Dh]))
    assert flips <= 2
    if mask == O.MASK_PADDING:
        assert not out[2 * Sq:].any()


def test_fp8_attention_accuracy_and_views():
    """Dequantized, the FP8 flow follows the exact softmax attention of the decoded operands within the E4M3
    rounding of P and of the output (3 mantissa bits: relative step 2^-3 .. 2^-4); strided views of a fused QKV
    buffer give the same bytes as contiguous copies."""
    B, S, H, Dh = 2, 40, 2, 64
    g = synth.rng(72)
    qkv = _f8(g.standard_normal((B * S, 3 * H * Dh)) * 2)
    qv, kv, vv = (OL._heads(qkv, B, S, H, Dh, i) for i in range(3))
    sp = np.float32(1.0 / 448.0)
    kw = dict(qk_scale=0.03, p_scale=float(sp), out_col_scale=np.float32([sp]), out_scale_is_scalar=True, out_dt=O.F32)
    a = O.fp8_attn(qv, kv, vv, **kw)
    assert np.array_equal(a, O.fp8_attn(qv.copy(), kv.copy(), vv.copy(), **kw))
    qf, kf, vf = (_f8_dec(t).astype(np.float64) for t in (qv, kv, vv))
    ref = OL.fp64_attention(qf.reshape(B * S, -1) * 0.03 * np.sqrt(Dh), kf.reshape(B * S, -1), vf.reshape(B * S, -1),
                            B, S, S, H, Dh, O.MASK_NONE, None)
    err = a.astype(np.float64) - ref
    snr = 10 * np.log10((ref ** 2).sum() / (err ** 2).sum())
    assert 25.0 < snr < 45.0, snr          # E4M3 rounding of P: relative error <= 2^-4 per term, averaged over the keys


def test_attention_online_closed_forms():
    """The online Softmax^quant variant (codes against the running block maximum, normalised at the end):
    closed forms that a dropped rescale, a wrong exponent sign or a wrong block boundary would break."""
    B, S, H, Dh = 1, 12, 2, 8
    q, k, v = _attn_inputs(30, B, S, S, H, Dh)
    sp = float(OL.S_P)
    unit = np.full(H * Dh, sp, np.float32)              # c[j] = S_p  ->  the output is O / L itself
    kw = dict(p_scale=sp, out_col_scale=unit, out_dt=O.F32, out_scale_is_scalar=True)
    # (1) equal scores, causal: every visible code is 255, the output is the mean of the visible V rows
    out, Cd = O.int8_attn_online(np.zeros_like(q), k, v, qk_scale_h=[0.01, 0.02], mask=O.MASK_CAUSAL, kv_block=5,
                                 dump_c=True, **kw)
    for i in range(S):
        assert (Cd[0, :, i, :i + 1] == 255).all() and (Cd[0, :, i, i + 1:] == 0).all()
        for h in range(H):
            mean = v[0, :i + 1, h, :].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(out[i, h * Dh:(h + 1) * Dh], mean, rtol=1e-6, atol=1e-6)
    # (2) three blocks of 4 keys with one score level each: s0 < s2 < s1.  Blocks 0 and 1 are all 255 (each is
    # the running maximum when it arrives), block 2 gets c2 = rne(255 exp(s2 - s1)), block 0 is rescaled by
    # exp(s0 - s1) at the end.
    qd = np.zeros_like(q)
    qd[..., 0] = 100
    kd = np.zeros_like(k)
    lev = [-30, 50, 20]
    for t in range(3):
        kd[0, 4 * t:4 * t + 4, :, 0] = lev[t]
    dts = np.float32([3e-4, 5e-4])
    out, Cd = O.int8_attn_online(qd, kd, v, qk_scale_h=dts, kv_block=4, dump_c=True, **kw)
    for h in range(H):
        s0, s1, s2 = (float(np.float32(100 * l) * dts[h]) for l in lev)
        c2 = round(float(np.float32(255.0 * math.exp(s2 - s1))))
        assert (Cd[0, h, :, :8] == 255).all() and (Cd[0, h, :, 8:] == c2).all() and 0 < c2 < 255
        V = v[0, :, h, :].astype(np.float64)
        r0 = math.exp(s0 - s1)
        num = r0 * 255 * V[0:4].sum(0) + 255 * V[4:8].sum(0) + c2 * V[8:12].sum(0)
        den = r0 * 255 * 4 + 255 * 4 + c2 * 4
        for i in range(S):
            np.testing.assert_allclose(out[i, h * Dh:(h + 1) * Dh], num / den, rtol=1e-6, atol=1e-6)
    # with the levels in ascending block order the last block is the maximum and c2 never appears
    # (3) one dominant key -> its V row, whatever block it sits in
    kd = np.zeros_like(k)
    kd[0, 9, :, 0] = 127
    qd[..., 0] = 127
    out = O.int8_attn_online(qd, kd, v, qk_scale_h=0.01, kv_block=4, **kw)
    for h in range(H):
        np.testing.assert_allclose(out[:, h * Dh:(h + 1) * Dh], np.repeat(v[0, 9:10, h, :], S, 0).astype(np.float32), rtol=1e-6)
    # (4) keys permuted inside their blocks: the same integers, the same output, bit for bit
    g = synth.rng(31)
    perm = np.concatenate([4 * t + g.permutation(4) for t in range(3)])
    cs = g.uniform(2e-5, 6e-5, H * Dh).astype(np.float32)
    a1 = O.int8_attn_online(q, k, v, qk_scale_h=3e-4, p_scale=sp, out_col_scale=cs, kv_block=4)
    a2 = O.int8_attn_online(q, k[:, perm], v[:, perm], qk_scale_h=3e-4, p_scale=sp, out_col_scale=cs, kv_block=4)
    assert np.array_equal(a1, a2)


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
def test_attention_online_single_block_against_numpy_and_masks_by_truncation(mask):
    """One block covering all keys: the codes are rne(255 exp(a - max)) and the output their normalised
    combination, written out with numpy / scipy; the masks are checked by truncating the inputs instead."""
    B, Sq, Skv, H, Dh = 3, 9, 9, 2, 16
    q, k, v = _attn_inputs(32, B, Sq, Skv, H, Dh)
    kv_len = np.int32([9, 5, 0]) if mask == O.MASK_PADDING else (np.int32([9, 6, 3]) if mask == O.MASK_CAUSAL else None)
    dts, sp = np.float32([2.5e-4, 4e-4]), float(OL.S_P)
    cs = synth.rng(33).uniform(0.5, 1.5, H * Dh).astype(np.float32) * np.float32(sp)
    out, Cd = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len,
                                 out_dt=O.I8, kv_block=64, dump_c=True)
    for b in range(B):
        L = Skv if kv_len is None else int(kv_len[b])
        for h in range(H):
            a = (q[b, :, h].astype(np.int64) @ k[b, :, h].astype(np.int64).T).astype(np.float32) * dts[h]
            for i in range(Sq):
                n = max(L if mask != O.MASK_CAUSAL else min(L, i + (L - Sq) + 1), 0)
                if mask == O.MASK_PADDING and Sq == Skv and i >= L:
                    n = 0                            # self-attention: a padded position asks nothing
                codes = np.zeros(Skv, np.int64)
                exp = np.zeros(Dh, np.int8)
                if n > 0:
                    w = scipy.special.softmax(a[i, :n].astype(np.float64))
                    codes[:n] = np.rint((255.0 * w / w.max()).astype(np.float32)).astype(np.int64)
                    y = (codes @ v[b, :, h].astype(np.int64)) / codes.sum() * cs[h * Dh:(h + 1) * Dh].astype(np.float64) / sp
                    exp = np.clip(np.rint(y.astype(np.float32)), -127, 127).astype(np.int8)
                assert np.array_equal(Cd[b, h, i], codes.astype(np.uint8))
                assert np.array_equal(out[b * Sq + i, h * Dh:(h + 1) * Dh], exp)
                if n > 0 and mask != O.MASK_NONE and i % 4 == 0:    # a masked row = an unmasked call on the visible prefix
                    sub = O.int8_attn_online(q[b:b + 1, i:i + 1], k[b:b + 1, :n], v[b:b + 1, :n], qk_scale_h=dts, p_scale=sp,
                                             out_col_scale=cs, out_dt=O.I8, kv_block=4)
                    ref = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len,
                                             out_dt=O.I8, kv_block=4)
                    assert np.array_equal(sub[0, h * Dh:(h + 1) * Dh], ref[b * Sq + i, h * Dh:(h + 1) * Dh])


def test_attention_online_accuracy_against_exact_softmax_and_two_pass():
    """Accuracy of the variant against the exact (unquantized-P) attention on the same INT8 operands: every
    weight is off by at most half a code of ITS block's scale, which bounds the output error; and on long,
    diffuse rows (where the normalised probabilities of the two-pass form use only a few codes) it is the more
    accurate of the two."""
    B, Sq, Skv, H, Dh = 1, 16, 256, 2, 16
    q, k, v = _attn_inputs(34, B, Sq, Skv, H, Dh)
    sp, dt = float(OL.S_P), np.float32(1.2e-4)
    unit = np.full(H * Dh, sp, np.float32)
    on = O.int8_attn_online(q, k, v, qk_scale_h=dt, p_scale=sp, out_col_scale=unit, out_dt=O.F32, out_scale_is_scalar=True, kv_block=64)
    tp, P = O.int8_attn(q, k, v, qk_scale=float(dt), p_scale=sp, out_col_scale=unit, out_dt=O.F32, out_scale_is_scalar=True, dump_p=True)
    exact = np.empty_like(on, dtype=np.float64)
    for h in range(H):
        a = (q[0, :, h].astype(np.int64) @ k[0, :, h].astype(np.int64).T).astype(np.float32) * dt
        w = scipy.special.softmax(a.astype(np.float64), axis=1)
        exact[:, h * Dh:(h + 1) * Dh] = w @ v[0, :, h].astype(np.float64)
        # hard bound: |w~ - w| <= 0.5/255 per key relative to the row maximum (rescale factors are <= 1)
        bound = 2 * 127 * Skv * (0.5 / 255) / (w / w.max(axis=1, keepdims=True)).sum(axis=1)
        assert (np.abs(on[:, h * Dh:(h + 1) * Dh] - exact[:, h * Dh:(h + 1) * Dh]).max(axis=1) <= bound).all()
    snr = lambda x: 10 * math.log10(float((exact ** 2).sum() / ((x - exact) ** 2).sum()))
    print("SNR online %.1f dB, two-pass %.1f dB" % (snr(on), snr(tp)))     # O6 with c[0] = S_p returns sum_k P v S_p
    assert snr(on) > 35 and snr(on) > snr(tp) + 6, (snr(on), snr(tp))


# ---------------------------------------------------------------- 16-bit side (BF16 / FP16)
@pytest.mark.parametrize("dt", [O.BF16, O.F16])
def test_16bit_ops_against_torch_fp64(dt):
    g = synth.rng(14)
    tdt = torch.bfloat16 if dt == O.BF16 else torch.float16
    enc = lambda a: O.f32_to_hp(a.astype(np.float32), dt)
    tb = lambda u: torch.from_numpy(O.hp_to_f32(u, dt)).double()
    bits = lambda t: t.float().to(tdt).view(torch.int16).numpy().view(np.uint16)
    M, K, N = 5, 48, 7
    A, Wt, res = enc(g.standard_normal((M, K))), enc(g.standard_normal((N, K))), enc(g.standard_normal((M, N)))
    bias = g.standard_normal(N).astype(np.float32)
    ref = torch.nn.functional.gelu(tb(A) @ tb(Wt).T + torch.from_numpy(bias).double()) + tb(res)
    got = O.hp_gemm(A, Wt, bias=bias, residual=res, gelu=True, dt=dt)
    assert np.array_equal(got, bits(ref))
    if dt == O.BF16:
        assert np.array_equal(got, O.bf16_gemm(A, Wt, bias=bias, residual=res, gelu=True))
    B, S, H, Dh = 2, 5, 2, 8
    q, k, v = (enc(g.standard_normal((B, S, H, Dh))) for _ in range(3))
    out = O.hp_attn(q, k, v, scale=0.35, mask=O.MASK_CAUSAL, dt=dt)
    tq, tk, tv = (tb(u).permute(0, 2, 1, 3) for u in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.35)
    ref = ref.permute(0, 2, 1, 3).reshape(B * S, H * Dh)
    assert np.array_equal(out, bits(ref))
    with pytest.raises(ValueError):
        O.hp_gemm(A, Wt, dt=O.F32)


# ---------------------------------------------------------------- layer: folds, modes, sanity
def test_table1_mode_masks():
    bits = [OL.M_QKV, OL.M_ATTN, OL.M_ATTN_OUT, OL.M_FC1, OL.M_FC2]
    want = {}
    for line in open(os.path.join(GOLDEN, "table1_modes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, emb, *flags = line.split()
        want[name] = sum(b for b, f in zip(bits, flags) if f == "1")
    assert want == {"M1": OL.MODE_M1, "M2": OL.MODE_M2, "M3": OL.MODE_M3}


def _tiny_shape(arch=synth.POST_LN, mask=synth.MASK_NONE):
    return synth.small(synth.CONFIGS[0], name="tiny", arch=arch, d=64, H=4, Dh=16, f=128, B=2, S=12, mask=mask,
                       eps=1e-5, w_std=0.08)


def _setup(shape, seed=20, mode=OL.MODE_M3, fp8=False):
    p = synth.layer_params(seed, shape)
    T = shape.B * shape.S
    emb = synth.embedding_ln_params(seed, shape)
    ln = lambda h: OL._ln64(h.astype(np.float64), emb["g"].astype(np.float64), emb["b"].astype(np.float64), shape.eps)
    hc = synth.activations(seed, shape, 4 * T, stream=1)
    h0 = synth.activations(seed, shape, T, stream=0)
    xc = ln(hc) if shape.arch == synth.POST_LN else hc.astype(np.float64)
    sc, _ = OL.calibrate(p, xc, shape, 4 * shape.B, shape.S, fp8=fp8)
    w = OL.prepare(p, sc, shape, mode, fp8=fp8)
    return p, sc, w, h0, emb


def test_fold_identities():
    """Folding S into the weights (Sec. 2.2.2 / 2.2.3) is exact in real arithmetic:
    X (W / S) = (X W) / S, (X_attn S_attn) W_o / S_o = X_attn (S_attn W_o / S_o), and the
    same for W_2.  Checked on the fp64 folded weights before they are quantized, and on the
    quantized route up to the weight-quantization error."""
    shape = _tiny_shape()
    p, sc, w, h0, emb = _setup(shape)
    g = synth.rng(21)
    d, f = shape.d, shape.f
    X = g.standard_normal((10, d))
    Wq = p["w_qkv"][:, :d].astype(np.float64)
    assert np.allclose(X @ (Wq / float(sc["S_q"])), (X @ Wq) / float(sc["S_q"]), rtol=1e-12)
    Xa = g.integers(-127, 128, (10, d)).astype(np.float64)
    Wo = p["w_o"].astype(np.float64)
    lhs = (Xa * sc["S_attn"].astype(np.float64)) @ Wo / sc["S_o"].astype(np.float64)
    Wt = sc["S_attn"].astype(np.float64)[:, None] * Wo / sc["S_o"].astype(np.float64)[None, :]
    assert np.allclose(lhs, Xa @ Wt, rtol=1e-10, atol=1e-9)
    # prepare() stores exactly the column-quantized folded weight, transposed to [N][K]
    wq, s = O.weight_quant(Wt.astype(np.float32))
    assert np.array_equal(wq, w["wq_o"]) and np.array_equal(s, w["s_o_w"])
    assert np.allclose(w["b_o"], p["b_o"] / sc["S_o"], rtol=1e-6)
    W2t = sc["S_a"].astype(np.float64)[:, None] * p["w_2"].astype(np.float64) / sc["S_x2"].astype(np.float64)[None, :]
    wq, s = O.weight_quant(W2t.astype(np.float32))
    assert np.array_equal(wq, w["wq_2"]) and np.array_equal(s, w["s_2_w"])
    assert w["wq_2"].shape == (d, f) and w["wq_1"].shape == (f, d) and w["wq_qkv"].shape == (3 * d, d)
    assert np.isclose(float(w["qk_scale"]), float(sc["S_q"]) * float(sc["S_k"]) / math.sqrt(shape.Dh), rtol=1e-6)
    # folded REQUANT route == explicit "dequantize, divide by S_q, round" route except near ties
    xq, xs = O.quant_twq(X.astype(np.float32))
    codes = O.int8_gemm(xq, w["wq_qkv"], a_row_scale=xs, b_col_scale=w["s_qkv"], bias=w["b_qkv"],
                        epi=O.EPI_REQUANT, c_dt=O.I8)
    acc = xq.astype(np.float64) @ w["wq_qkv"].astype(np.float64).T
    val = acc * xs[:, None] * w["s_qkv"][None, :] + w["b_qkv"][None, :]      # already in units of S_q|k|v
    near_tie = np.abs(val - np.floor(val) - 0.5) < 1e-4
    exp = np.clip(np.rint(val), -127, 127)
    assert np.array_equal(codes[~near_tie], exp[~near_tie].astype(np.int8))
    # ... and those codes times S_q approximate the unquantized X_q
    xq_true = (X @ p["w_qkv"].astype(np.float64) + p["b_qkv"])[:, :d]
    err = np.abs(codes[:, :d] * float(sc["S_q"]) - xq_true)
    assert np.median(err) < 2 * float(sc["S_q"])


@pytest.mark.parametrize("arch", [synth.POST_LN, synth.PRE_LN])
def test_layer_modes_track_fp64_model(arch):
    """Sanity (not pass/fail on accuracy): every mode of Table 1 stays close to the
    unquantized layer, and the layer chain is wired correctly (a wrong scale, a swapped
    q/k/v block or a missing residual drops the SNR to ~0 dB)."""
    mask = synth.MASK_NONE if arch == synth.POST_LN else synth.MASK_CAUSAL
    shape = _tiny_shape(arch, mask)
    B, S, T = shape.B, shape.S, shape.B * shape.S
    snr = {}
    for name, mode in (("M1", OL.MODE_M1), ("M2", OL.MODE_M2), ("M3", OL.MODE_M3)):
        p, sc, w, h0, emb = _setup(shape, mode=mode)
        if arch == synth.POST_LN:
            xq, xs, xf = O.ln_quant(h0, O.F32, None, None, 0, None, emb["g"], emb["b"], shape.eps, y_hp_dt=O.F32)
            ref = OL.fp64_layer(p, xf.astype(np.float64), shape, B, S)["out"]
            oq, os_ = OL.layer_fwd(w, shape, B, S, x_q=xq, x_s=xs)
            got = oq.astype(np.float64) * os_[:, None]
        else:
            hb = O.f32_to_bf16(h0)
            ref = OL.fp64_layer(p, O.bf16_to_f32(hb).astype(np.float64), shape, B, S)["out"]
            got = O.bf16_to_f32(OL.layer_fwd(w, shape, B, S, h=hb)).astype(np.float64)
        snr[name] = 10 * math.log10((ref ** 2).sum() / ((ref - got) ** 2).sum())
    assert all(v > 15.0 for v in snr.values()), snr


@pytest.mark.parametrize("hp", [O.BF16, O.F16])
@pytest.mark.parametrize("arch", [synth.POST_LN, synth.PRE_LN])
def test_module_switch_all_subsets_ordered_against_fp64_model(arch, hp):
    """Sec. 2.3: every module has an INT8 / 16-bit switch.  The all-16-bit layer (Table 2's FP16 row; mode 0) is
    the unquantized layer up to 16-bit rounding; switching modules to INT8 one group at a time (M1, M2, M3 of
    Table 1, and the two subsets in between that keep a whole sub-block 16-bit) can only add quantization
    noise.  Pinned against the fp64 layer: SNR(M0) is at the level of the 16-bit format (bf16: 8 bits of
    significand, fp16: 11), and SNR(M0) >= SNR(M1) >= SNR(M2) >= SNR(M3) up to half a dB of luck.  A mis-wired
    16-bit module (wrong weight, missing bias or residual, GELU left out) drops its mode to ~0-10 dB and breaks
    the order.  Subsets that would need a stand-alone quantization kernel are refused."""
    mask = synth.MASK_NONE if arch == synth.POST_LN else synth.MASK_CAUSAL
    shape = _tiny_shape(arch, mask)
    B, S = shape.B, shape.S
    p, sc, _, h0, emb = _setup(shape)
    enc = lambda a: O.f32_to_hp(np.asarray(a, np.float32), hp)
    dec = lambda u: O.hp_to_f32(u, hp).astype(np.float64)
    if arch == synth.POST_LN:
        xq, xs, xf = O.ln_quant(h0, O.F32, None, None, 0, None, emb["g"], emb["b"], shape.eps, y_hp_dt=O.F32)
        ref = OL.fp64_layer(p, xf.astype(np.float64), shape, B, S)["out"]
    else:
        hb = enc(h0)
        ref = OL.fp64_layer(p, dec(hb), shape, B, S)["out"]
    A_ONLY = OL.M_QKV | OL.M_ATTN | OL.M_ATTN_OUT                      # attention block INT8, MLP block 16-bit
    F_ONLY = OL.M_FC1 | OL.M_FC2                                        # the other way round
    snr = {}
    for name, mode in (("M0", OL.MODE_M0), ("M1", OL.MODE_M1), ("M2", OL.MODE_M2), ("M3", OL.MODE_M3),
                       ("attn-block", A_ONLY), ("mlp-block", F_ONLY), ("qkv", OL.M_QKV), ("fc1", OL.M_FC1)):
        w = OL.prepare(p, sc, shape, mode, hp_dt=hp)
        tr = {}
        if arch == synth.POST_LN:
            kw = dict(x_q=xq, x_s=xs) if mode & OL.M_QKV else dict(x_hp=enc(xf))
            OL.layer_fwd(w, shape, B, S, trace=tr, **kw)
            got = dec(tr["out_hp"])
        else:
            got = dec(OL.layer_fwd(w, shape, B, S, h=hb, trace=tr))
        snr[name] = 10 * math.log10((ref ** 2).sum() / ((ref - got) ** 2).sum())
        # a 16-bit module reads and writes 16-bit tensors, an INT8 module INT8 ones
        assert (tr["qkv"].dtype == np.int8) == bool(mode & OL.M_ATTN)
        assert (tr["a"].dtype == np.int8) == bool(mode & OL.M_FC2)
    print({k: round(v, 1) for k, v in snr.items()})
    assert snr["M0"] > (38.0 if hp == O.BF16 else 55.0), snr
    assert snr["M0"] + 0.5 >= snr["M1"] and snr["M1"] + 0.5 >= snr["M2"] and snr["M2"] + 0.5 >= snr["M3"], snr
    for k in ("attn-block", "mlp-block", "qkv", "fc1"):
        assert snr["M0"] + 0.5 >= snr[k] >= snr["M3"] - 0.5, (k, snr)
    assert snr["M3"] > 15.0
    for bad in (OL.M_ATTN, OL.M_QKV | OL.M_ATTN_OUT, OL.M_FC2, OL.M_QKV | OL.M_FC2):
        with pytest.raises(ValueError):
            OL.prepare(p, sc, shape, bad, hp_dt=hp)
    with pytest.raises(ValueError):
        OL.prepare(p, sc, shape, OL.MODE_M1, hp_dt=O.F32)


@pytest.mark.parametrize("arch", [synth.POST_LN, synth.PRE_LN])
def test_fp8_layer_tracks_fp64_model_and_ln_reads_e4m3_inputs(arch):
    """The FP8 variant of the layer (Sec. 2.1): every module with E4M3 codes, the scale granularities and folds of
    the INT8 layer.  It stays close to the unquantized layer (E4M3 has 3 mantissa bits: the relative error per
    value is up to 2^-4 where INT8's is absolute, so the SNR sits below the INT8 layer's), a mis-wired scale drops
    it to ~0 dB; the weights are E4M3 codes with max 448 per column; LN^quant with E4M3 addends equals LN^quant of
    the decoded addends."""
    mask = synth.MASK_NONE if arch == synth.POST_LN else synth.MASK_CAUSAL
    shape = _tiny_shape(arch, mask)
    B, S = shape.B, shape.S
    p, sc, w, h0, emb = _setup(shape, fp8=True)
    assert w["fp8"] and w["wq_qkv"].dtype == np.uint8 and float(w["S_p"]) == float(OL.S_P_FP8)
    for k_ in ("wq_qkv", "wq_o", "wq_1", "wq_2"):
        assert (np.abs(O.e4m3_to_f32(w[k_])).max(axis=1) == 448.0).all()
    tr = {}
    if arch == synth.POST_LN:
        xq, xs, xf = O.ln_quant(h0, O.F32, None, None, 0, None, emb["g"], emb["b"], shape.eps, y_hp_dt=O.F32, fp8=True)
        ref = OL.fp64_layer(p, xf.astype(np.float64), shape, B, S)["out"]
        oq, os_ = OL.layer_fwd(w, shape, B, S, x_q=xq, x_s=xs, trace=tr)
        got = O.e4m3_to_f32(oq).astype(np.float64) * os_[:, None]
        # LN^quant(S_in X_in,f8, X_o,f8 S_o) = LN^quant of the decoded sum handed over in fp32
        ssum = (O.e4m3_to_f32(xq).astype(np.float64) * xs[:, None] + O.e4m3_to_f32(tr["xo"]).astype(np.float64) * w["S_o"][None, :])
        q2, s2, _ = O.ln_quant(ssum.astype(np.float32), O.F32, None, None, 0, None, w["ln1_g"], w["ln1_b"], shape.eps, fp8=True)
        assert np.count_nonzero(q2 != tr["mid_q"]) <= 0.01 * q2.size and np.allclose(s2, tr["mid_s"], rtol=1e-5)
    else:
        hb = O.f32_to_bf16(h0)
        ref = OL.fp64_layer(p, O.bf16_to_f32(hb).astype(np.float64), shape, B, S)["out"]
        got = O.bf16_to_f32(OL.layer_fwd(w, shape, B, S, h=hb, trace=tr)).astype(np.float64)
    snr = 10 * math.log10((ref ** 2).sum() / ((ref - got) ** 2).sum())
    assert snr > 22.0, snr                  # measured 27.9 dB (post-LN) and 37.3 dB (pre-LN); the INT8 layer: 28.5 and 38.4
    with pytest.raises(ValueError):
        OL.prepare(p, sc, shape, OL.MODE_M2, fp8=True)


def test_decode_with_cache_equals_prefill():
    """Pre-LN layer: feeding a sequence token by token through the INT8 KV cache gives the
    same INT8 attention inputs/outputs as one causal prefill call (the cache holds exactly
    the K/V codes the prefill computes)."""
    shape = _tiny_shape(synth.PRE_LN, synth.MASK_CAUSAL)
    B, S = shape.B, shape.S
    p, sc, w, h0, emb = _setup(shape)
    hb = O.f32_to_bf16(h0)
    full = OL.layer_fwd(w, shape, B, S, h=hb)
    cache = {"k": np.zeros((B, shape.H, S + 2, shape.Dh), np.int8), "v": np.zeros((B, shape.H, S + 2, shape.Dh), np.int8)}
    hb3 = hb.reshape(B, S, shape.d)
    outs = []
    for t in range(S):
        step = OL.layer_fwd(w, shape, B, 1, h=np.ascontiguousarray(hb3[:, t]), kv_len=np.full(B, t + 1, np.int32),
                            cache=cache)
        outs.append(step.reshape(B, 1, shape.d))
    assert np.array_equal(np.concatenate(outs, axis=1).reshape(B * S, shape.d), full)
