"""GPU parity on a seeded sweep of random shapes: many small problems whose sizes are drawn so that every tile
shape, ragged tail, K-slab count (odd and even), head width, mask and epilogue of the kernels is hit by some
case.  Each case is compared with the oracle in the tolerance class of its operator."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import layer as OL
from paper_2310_17723_amd import binding as HB
from paper_2310_17723_amd import synth
from parity import assert_codes, assert_exact, assert_scales, dev, rel_err, to_np

pytestmark = pytest.mark.gpu


def test_gemm_random_shapes(hero):
    g = synth.rng(4000)
    for case in range(36):
        big = case % 9 == 8                                      # a many-tile case now and then (persistent kernel)
        M = int(g.integers(1, 3000)) if big else int(g.integers(1, 520))
        N = 4 * int(g.integers(1, 700)) if big else 4 * int(g.integers(1, 200))
        K = 64 * int(g.integers(1, 7 if big else 20))
        c = synth.gemm_case(4001 + case, M, K, N, outlier_rows=bool(case & 1))
        A, Bt, rs, cs, bias = c["A"], c["Bt"], c["a_row_scale"], c["b_col_scale"], c["bias"]
        dA, dB = dev(A), dev(Bt)
        what = f"case {case}: M={M} N={N} K={K}"
        assert_exact(to_np(hero.hero_int8_gemm(dA, dB)), O.gemm_i32(A, Bt), what + " raw")
        cs2 = (cs * np.float32(3000.0 / np.sqrt(K))).astype(np.float32)
        epi = case % 3
        if epi == 0:
            ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs2, bias=bias, epi=O.EPI_REQUANT, c_dt=O.I8)
            got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs2), dev(bias), epi=HB.EPI_REQUANT, out_dtype=torch.int8)
            assert_exact(to_np(got), ref, what + " requant")
        elif epi == 1:
            res = O.f32_to_bf16(g.standard_normal((M, N)).astype(np.float32))
            ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=cs, bias=bias, residual=res, res_dt=O.BF16,
                              epi=O.EPI_DEQUANT, c_dt=O.BF16)
            got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(cs), dev(bias), residual=dev(res), epi=HB.EPI_DEQUANT,
                                      out_dtype=torch.bfloat16)
            assert_exact(to_np(got), ref, what + " dequant + residual")
        else:
            csg = (cs * np.float32(30.0 / np.sqrt(K))).astype(np.float32)
            gl = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_DEQUANT_GELU, c_dt=O.F32)
            s_a = (np.abs(gl).max(axis=0) / 127 + 1e-6).astype(np.float32)
            ref = O.int8_gemm(A, Bt, a_row_scale=rs, b_col_scale=csg, bias=bias, epi=O.EPI_GELU_REQUANT, out_col_scale=s_a, c_dt=O.I8)
            got = hero.hero_int8_gemm(dA, dB, dev(rs), dev(csg), dev(bias), epi=HB.EPI_GELU_REQUANT, out_col_scale=dev(s_a),
                                      out_dtype=torch.int8)
            assert_codes(to_np(got), ref, what + " gelu requant", max_frac=max(1e-3, 2.5 / ref.size))


def test_ln_quant_random_shapes(hero):
    g = synth.rng(4100)
    for case in range(24):
        M = int(g.integers(1, 400))
        D = 16 * int(g.integers(1, 513 if case % 2 == 0 else 257))   # 16 .. 8192 (INT8 rows), .. 4096 (16-bit rows)
        xq = g.integers(-127, 128, (M, D), dtype=np.int8)
        rq = g.integers(-127, 128, (M, D), dtype=np.int8)
        xs = g.uniform(0.005, 0.05, M).astype(np.float32)
        rc = g.uniform(0.001, 0.02, D).astype(np.float32)
        gam = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
        bet = (0.02 * g.standard_normal(D)).astype(np.float32)
        what = f"case {case}: M={M} D={D}"
        if case % 2 == 0:
            q_o, s_o, _ = O.ln_quant(xq, O.I8, xs, rq, O.I8, rc, gam, bet, 1e-12)
            q, s, _ = hero.hero_ln_quant(dev(xq), dev(xs), dev(rq), dev(rc), dev(gam), dev(bet), 1e-12)
        else:
            hb = O.f32_to_bf16((g.standard_normal((M, D)) * g.uniform(0.5, 3, (M, 1))).astype(np.float32))
            q_o, s_o, _ = O.ln_quant(hb, O.BF16, None, None, 0, None, gam, bet, 1e-5)
            q, s, _ = hero.hero_ln_quant(dev(hb), None, None, None, dev(gam), dev(bet), 1e-5)
        assert_scales(to_np(s), s_o, what)
        assert_codes(to_np(q), q_o, what, max_frac=max(1e-3, 2.5 / q_o.size))


def test_attention_random_shapes(hero):
    g = synth.rng(4200)
    sp = float(OL.S_P)
    for case in range(16):
        Dh = 64 if case % 2 == 0 else 128
        B, H = int(g.integers(1, 3)), int(g.integers(1, 4))
        Sq = int(g.integers(1, 300))
        mask = case % 3
        Skv = Sq if mask == O.MASK_CAUSAL and case % 4 else int(g.integers(Sq, Sq + 200))
        mk = lambda s: np.clip(np.rint(g.standard_normal(s) * 30), -127, 127).astype(np.int8)
        q, k, v = mk((B, Sq, H, Dh)), mk((B, Skv, H, Dh)), mk((B, Skv, H, Dh))
        qk_scale = float(np.float32(24.0 / (900 * Dh)))
        cs = g.uniform(0.8, 1.2, H * Dh).astype(np.float32) * np.float32(1.0 / (255 * 30) * 127 / 2.5)
        kv_len = None
        if mask == O.MASK_PADDING:
            kv_len = g.integers(1, Skv + 1, B).astype(np.int32)
        elif mask == O.MASK_CAUSAL:
            kv_len = g.integers(Sq, Skv + 1, B).astype(np.int32)
        what = f"case {case}: B={B} H={H} Sq={Sq} Skv={Skv} Dh={Dh} mask={mask}"
        ref = O.int8_attn(q, k, v, qk_scale=qk_scale, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len)
        got = hero.hero_int8_attn(dev(q), dev(k), dev(v), qk_scale, sp, dev(cs), mask=mask, kv_len=dev(kv_len))
        assert_codes(to_np(got), ref, what + " two-pass", max_frac=max(1e-3, 2.5 / ref.size))
        dts = (np.float32(qk_scale) * g.uniform(0.7, 1.5, H)).astype(np.float32)
        ref = O.int8_attn_online(q, k, v, qk_scale_h=dts, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len, kv_block=64)
        got = hero.hero_int8_attn_online(dev(q), dev(k), dev(v), dev(dts), sp, dev(cs), mask=mask, kv_len=dev(kv_len))
        assert_codes(to_np(got), ref, what + " online", max_frac=max(1e-3, 2.5 / ref.size))
