"""Comparison helpers for the GPU-vs-oracle parity tests (tolerance classes of the
benchmark contract: bit-exact integers, +-1 LSB on <= 0.1 % for LayerNorm / softmax / GELU
fused paths, 2e-2 relative for 16-bit float outputs)."""
import numpy as np
import torch


def to_np(t):
    """Device tensor -> numpy; 16-bit floats come back as uint16 bit patterns."""
    t = t.detach().cpu()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()


def dev(a, dtype=None):
    """numpy -> cuda tensor; uint16 arrays are reinterpreted as `dtype` (bf16/f16)."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(dtype or torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def assert_exact(got, ref, what=""):
    got, ref = np.asarray(got), np.asarray(ref)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    bad = np.flatnonzero(got.ravel() != ref.ravel())
    assert bad.size == 0, f"{what}: {bad.size} of {got.size} differ, first at {bad[:5]}: " \
                          f"{got.ravel()[bad[:5]]} vs {ref.ravel()[bad[:5]]}"


def assert_codes(got, ref, what="", max_frac=1e-3):
    """INT8 codes: |diff| <= 1 everywhere, differing on at most max_frac of the elements."""
    d = np.abs(got.astype(np.int32) - ref.astype(np.int32))
    assert d.max() <= 1, f"{what}: max code difference {d.max()} at {np.unravel_index(d.argmax(), d.shape)}"
    frac = np.count_nonzero(d) / d.size
    assert frac <= max_frac, f"{what}: {frac:.2e} of the codes differ by 1 LSB (limit {max_frac:.0e})"
    return frac


def assert_scales(got, ref, what="", rtol=1e-5):
    assert np.allclose(got, ref, rtol=rtol, atol=0), f"{what}: scales differ, max rel " \
        f"{np.max(np.abs(got - ref) / np.abs(ref)):.2e}"


def rel_err(got_f32, ref_f32):
    """max_i |g - o| / max(|o_i|, rms(o)): the 16-bit float output tolerance."""
    g, o = got_f32.astype(np.float64), ref_f32.astype(np.float64)
    rms = np.sqrt(np.mean(o * o)) + 1e-30
    return float(np.max(np.abs(g - o) / np.maximum(np.abs(o), rms)))


def upload_weights(hero, w):
    """Oracle-prepared layer parameters (oracle.layer.prepare) -> device hero_layer_weights.
    Returns (struct, keepalive dict of device tensors)."""
    from paper_2310_17723_amd import binding as HB
    mode = w["mode"]
    names = {"w_qkv": "wq_qkv", "w_qkv_s": "s_qkv", "b_qkv": "b_qkv", "w_o": "wq_o", "w_o_s": "s_o_w", "b_o": "b_o",
             "w_1": "wq_1", "w_1_s": "s_1", "b_1": "b_1", "w_2": "wq_2", "w_2_s": "s_2_w", "b_2": "b_2",
             "w_o_bf16": "wb_o", "w_2_bf16": "wb_2", "w_qkv_hp": "wb_qkv", "w_1_hp": "wb_1", "ln1_g": "ln1_g", "ln1_b": "ln1_b", "ln2_g": "ln2_g",
             "ln2_b": "ln2_b", "S_o": "S_o", "S_x2": "S_x2", "S_a": "S_a"}
    t = {k: dev(w[v]) for k, v in names.items() if v in w}
    t["attn_out_scale"] = dev(w["attn_out_scale"] if mode & HB.M_ATTN_OUT else w["attn_out_scalar"])
    qk = float(w["qk_scale"] if mode & HB.M_ATTN else w["bf16_qk_scale"])
    return hero.layer_weights(t, qk, float(w["S_p"])), t


def assert_fp8_codes(got, ref, decode, what="", max_frac=1e-3, acc_rel=0.0):
    """E4M3 codes: equal on all but max_frac of the elements, and where they differ the decoded values are
    within one E4M3 step plus acc_rel x rms(ref): the matrix cores' accumulation carries an error that is a
    fraction of the TYPICAL dot product, not of the individual one, so an output much smaller than typical may
    move by more than its own (fine) grid step.  The caller derives max_frac and acc_rel."""
    g, o = decode(got).astype(np.float64), decode(ref).astype(np.float64)
    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(o), 2.0 ** -6))) - 3), 2.0 ** -9)
    slack = acc_rel * np.sqrt(np.mean(o * o))
    bad = np.abs(g - o) > step * 1.0001 + slack
    assert not bad.any(), f"{what}: {np.count_nonzero(bad)} codes are further away than one step + {slack:.3g}"
    frac = np.count_nonzero(got != ref) / got.size
    assert frac <= max_frac, f"{what}: {frac:.2e} of the codes differ (limit {max_frac:.0e})"
    return frac


def assert_fp8_attn_codes(got, ref, decode, what="", max_frac=2e-2, rel_l2=2e-2, flip_rel=0.25):
    """E4M3 outputs of the FP8 attention.  The probabilities are E4M3 codes themselves (relative step 2^-3 .. 2^-4),
    and the matrix cores' scores differ from the exactly accumulated ones by ~1e-3 relative, so about one
    probability in a hundred lands on the neighbouring code; when that happens to a dominant key (p ~ 0.5) the
    whole output row moves by up to 2^-3 p |v| ~ a quarter of the typical output.  Hence: the decoded outputs
    agree in relative L2 (the bar of the 16-bit outputs), the codes differ on at most max_frac of the elements,
    and no element is further away than one output step plus flip_rel x rms(ref)."""
    g, o = decode(got).astype(np.float64), decode(ref).astype(np.float64)
    rms = np.sqrt(np.mean(o * o))
    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(o), 2.0 ** -6))) - 3), 2.0 ** -9)
    bad = np.abs(g - o) > step * 1.0001 + flip_rel * rms
    assert not bad.any(), f"{what}: {np.count_nonzero(bad)} outputs are further away than one step + {flip_rel} rms"
    l2 = np.sqrt(((g - o) ** 2).sum() / max((o * o).sum(), 1e-30))
    assert l2 <= rel_l2, f"{what}: relative L2 distance {l2:.2e} (limit {rel_l2:.0e})"
    frac = np.count_nonzero(got != ref) / got.size
    assert frac <= max_frac, f"{what}: {frac:.2e} of the codes differ (limit {max_frac:.0e})"
    return frac


def assert_fp8_attn_values(got_f32, ref_f32, what="", rel_l2=2e-2, flip_rel=0.25):
    """16-bit outputs of the FP8 attention: the same class as assert_fp8_attn_codes without the output grid: relative
    L2 within rel_l2, every element within flip_rel x rms(ref) (one flipped probability code of a dominant key)
    plus the 16-bit rounding of its own value."""
    g, o = got_f32.astype(np.float64), ref_f32.astype(np.float64)
    rms = np.sqrt(np.mean(o * o))
    bad = np.abs(g - o) > flip_rel * rms + 2e-2 * np.abs(o)
    assert not bad.any(), f"{what}: {np.count_nonzero(bad)} outputs are further away than {flip_rel} rms"
    l2 = np.sqrt(((g - o) ** 2).sum() / max((o * o).sum(), 1e-30))
    assert l2 <= rel_l2, f"{what}: relative L2 distance {l2:.2e} (limit {rel_l2:.0e})"
    return l2
