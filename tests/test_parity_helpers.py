"""The FP8 attention tolerance (parity.fp8_attn_flip_bound / assert_fp8_attn_codes) on the CPU: it admits an oracle
whose scores are perturbed the way a kernel's are, and rejects an output that is off where no flip is possible."""
import numpy as np
import pytest

import oracle as O
from paper_2310_17723_amd import synth
from parity import assert_fp8_attn_codes, fp8_attn_flip_bound


def _case(seed, B, S, H, Dh):
    g = synth.rng(seed)
    mk = lambda s: O.f32_to_e4m3((g.standard_normal(s) * 40).astype(np.float32))
    q, k, v = mk((B, S, H, Dh)), mk((B, S, H, Dh)), mk((B, S, H, Dh))
    sp = np.float32(1.0 / 448.0)
    cs = g.uniform(0.8, 1.2, H * Dh).astype(np.float32) * sp * np.float32(4.0)
    return q, k, v, float(np.float32(1.5 / (40 * 40 * np.sqrt(Dh)))), float(sp), cs


@pytest.mark.parametrize("mask", [O.MASK_NONE, O.MASK_PADDING, O.MASK_CAUSAL])
def test_flip_bound_admits_perturbed_scores_and_rejects_real_errors(mask):
    B, S, H, Dh = 2, 96, 2, 32
    q, k, v, qk, sp, cs = _case(91, B, S, H, Dh)
    kv_len = np.int32([S - 5, 40]) if mask == O.MASK_PADDING else None
    ref = O.fp8_attn(q, k, v, qk_scale=qk, p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len)
    D = fp8_attn_flip_bound(q, k, v, qk, sp, cs, mask=mask, kv_len=kv_len)
    assert D.shape == ref.shape and (D >= 0).all() and (D == 0).mean() > 0.05       # some rows have no flip candidate at all
    flips = 0
    for rel in (2e-5, -3e-5, 5e-5):                    # scores off by a few 1e-5 relative: the kernel's kind of error
        per = O.fp8_attn(q, k, v, qk_scale=qk * (1 + rel), p_scale=sp, out_col_scale=cs, mask=mask, kv_len=kv_len)
        clean, diff = assert_fp8_attn_codes(per, ref, O.e4m3_to_f32, f"perturbed {rel}", flip_bound=D)
        flips += np.count_nonzero(per != ref)
    assert flips > 0                                   # the perturbation did flip codes: the bound was exercised
    # an output that is wrong by two grid steps in a row without flip candidates is caught
    rows = np.flatnonzero((D == 0).all(axis=1) & (ref != 0).all(axis=1))
    assert rows.size > 0
    bad = ref.copy()
    bad[rows[0], 3] = (bad[rows[0], 3] & 0x80) | min((bad[rows[0], 3] & 0x7f) + 2, 0x7e)
    with pytest.raises(AssertionError):
        assert_fp8_attn_codes(bad, ref, O.e4m3_to_f32, "planted", flip_bound=D)
    # and so are too many one-step differences where no flip is possible
    bad = ref.copy()
    cl = np.argwhere((D == 0) & ((ref & 0x7f) > 8) & ((ref & 0x7f) < 0x70))[:200]
    bad[cl[:, 0], cl[:, 1]] += 1
    with pytest.raises(AssertionError):
        assert_fp8_attn_codes(bad, ref, O.e4m3_to_f32, "planted one-step", flip_bound=D)
