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


def fp8_attn_flip_bound(q8, k8, v8, qk_scale, p_scale, out_col_scale, mask=0, kv_len=None, tau=5e-4):
    """Where, and by how much, the FP8 attention's output MAY differ from the oracle's because a probability code
    landed on the neighbouring E4M3 value.  The codes are e4m3(p / S_p); the kernel's p differs from the oracle's by
    a small relative error (the matrix cores' accumulation of the E4M3 products, exp2 / log2 approximations), so a
    code can differ only where p / S_p lies within a relative distance tau of a rounding boundary of the E4M3 grid,
    and then by one grid step.  tau is measured: on the four shapes of the kernel tests every deviation of more than
    one output step is explained from tau = 2e-4 on (one is not at 1e-4); the default leaves a factor 2.5.  From the oracle's side of the computation alone (decoded operands, fp64 softmax) this
    returns D[row, column] = sum over the keys flagged that way of step_k |v_k[column]| c[column]: the largest
    output deviation those flips can cause.  D is 0 wherever no key of the row is near a boundary.
    q8 [B,Sq,H,Dh], k8 / v8 [B,Skv,H,Dh] E4M3 codes (any strides); returns float64 [B*Sq, H*Dh]."""
    import oracle as O
    qf, kf, vf = (O.e4m3_to_f32(np.ascontiguousarray(t)).astype(np.float64) for t in (q8, k8, v8))
    B, Sq, H, Dh = qf.shape
    Skv = kf.shape[1]
    cs = np.broadcast_to(np.asarray(out_col_scale, np.float64).ravel(), (H * Dh,)) if np.size(out_col_scale) > 1 \
        else np.full(H * Dh, float(np.asarray(out_col_scale).ravel()[0]))
    D = np.zeros((B * Sq, H * Dh))
    ki, qi = np.arange(Skv)[None, :], np.arange(Sq)[:, None]
    for b in range(B):
        L = Skv if kv_len is None else int(min(max(kv_len[b], 0), Skv))
        vis = np.broadcast_to(ki < L, (Sq, Skv)).copy()
        if mask == 2:
            vis &= ki <= qi + (L - Sq)
        if mask == 1 and Sq == Skv:
            vis &= qi < L
        for h in range(H):
            a = (qf[b, :, h] @ kf[b, :, h].T).astype(np.float32).astype(np.float64) * np.float64(np.float32(qk_scale))
            a = np.where(vis, a, -np.inf)
            m = np.max(a, axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)
            e = np.exp(a - m)
            x = e / np.maximum(e.sum(axis=1, keepdims=True), 1e-300) / p_scale
            step = 2.0 ** (np.floor(np.log2(np.maximum(x, 2.0 ** -6))) - 3)          # grid step at x (2^-9 below 2^-6)
            u = x / step
            near = vis & (np.abs(u - np.floor(u) - 0.5) * step <= tau * x)
            D[b * Sq:(b + 1) * Sq, h * Dh:(h + 1) * Dh] = ((near * step) @ np.abs(vf[b, :, h])) * cs[h * Dh:(h + 1) * Dh]
    return D


def assert_fp8_attn_codes(got, ref, decode, what="", flip_bound=None, clean_frac=5e-3):
    """E4M3 outputs of the FP8 attention against the oracle's, with the tolerance the oracle's own probabilities
    justify (fp8_attn_flip_bound): every decoded output is within flip_bound (the flips that are possible in its row)
    plus one step of the output grid (the final rounding of nearly equal fp32 values); and where no flip is possible
    (flip_bound == 0) the codes are the oracle's on all but clean_frac of the elements.  clean_frac is the class of
    the FP8 GEMMs (assert_fp8_codes): the matrix cores' PV sums are off by ~1e-4 of a typical sum, which moves an
    output across a boundary of its 2^-3 .. 2^-4 relative grid on ~1e-3 of the elements (measured 0.7e-3 .. 1.6e-3,
    independent of tau, i.e. not caused by probability flips)."""
    g, o = decode(got).astype(np.float64), decode(ref).astype(np.float64)
    D = np.zeros_like(o) if flip_bound is None else flip_bound
    assert D.shape == o.shape, (what, D.shape, o.shape)
    rms = np.sqrt(np.mean(o * o))
    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(o), 2.0 ** -6))) - 3), 2.0 ** -9)
    # 1e-3 rms: the accumulation error of the matrix cores is a fraction of the TYPICAL sum (acc_rel of the FP8 GEMM
    # class); an output near zero, whose own grid step is far finer than that, may move by several of its steps
    bad = np.abs(g - o) > D * 1.0001 + step * 1.0001 + 1e-3 * rms
    assert not bad.any(), f"{what}: {np.count_nonzero(bad)} outputs are further away than the possible flips + one output step, " \
                          f"worst excess {np.max(np.abs(g - o) - D - step):.3g} (rms {rms:.3g})"
    clean = D == 0
    ndiff = np.count_nonzero((got != ref) & clean)
    assert ndiff <= max(clean_frac * max(np.count_nonzero(clean), 1), 2.5), \
        f"{what}: {ndiff} of {np.count_nonzero(clean)} codes differ where no probability is near a rounding boundary"
    return float(np.mean(clean)), float(np.mean(got != ref))


def assert_fp8_attn_values(got_f32, ref_f32, what="", rel_l2=2e-2, flip_rel=0.25, flip_bound=None):
    """16-bit outputs of the FP8 attention.  With flip_bound (fp8_attn_flip_bound, kernel-level tests): every element
    within the possible flips of its row plus the 16-bit rounding of its own value plus the accumulation error of the
    matrix cores.  Without it (whole-layer tests,
    where a flipped code has passed through later operators): relative L2 within rel_l2 and every element within
    flip_rel x rms(ref) plus the 16-bit rounding of its own value."""
    g, o = got_f32.astype(np.float64), ref_f32.astype(np.float64)
    rms = np.sqrt(np.mean(o * o))
    if flip_bound is not None:
        # 1e-3 rms: the matrix cores' PV sums carry an error that is a fraction of the TYPICAL sum (the acc_rel of the
        # FP8 GEMM class), which an output much smaller than typical shows in full
        bad = np.abs(g - o) > flip_bound * 1.0001 + 2.0 ** -7 * np.abs(o) + 1e-3 * rms
        assert not bad.any(), f"{what}: {np.count_nonzero(bad)} outputs are further away than the possible flips + the 16-bit rounding"
        return 0.0
    bad = np.abs(g - o) > flip_rel * rms + 2e-2 * np.abs(o)
    assert not bad.any(), f"{what}: {np.count_nonzero(bad)} outputs are further away than {flip_rel} rms"
    l2 = np.sqrt(((g - o) ** 2).sum() / max((o * o).sum(), 1e-30))
    assert l2 <= rel_l2, f"{what}: relative L2 distance {l2:.2e} (limit {rel_l2:.0e})"
    return l2
