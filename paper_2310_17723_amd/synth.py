"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module draws random numbers and names shapes; it contains none of the method's
arithmetic (no quantization, no LayerNorm, no scale folding).  Everything is produced
with numpy's counter-based Philox generator, so the same (seed, shape) gives the same
bytes on every machine; the CPU oracle and the HIP library both consume these arrays.

The paper evaluates BERT-base on GLUE at sequence length 128 (Sec. 3, experiment
setting); those checkpoints and datasets are not available offline, so the shapes below
are BERT-base / BERT-large / GPT-like layers with synthetic values standing in for them:
weights N(0, w_std^2), activations N(0,1) with a small fraction of "outlier" channels
multiplied by a constant, LayerNorm gain 1+N(0,0.1^2) and bias N(0,0.02^2).
"""
from __future__ import annotations

import dataclasses

import numpy as np

POST_LN, PRE_LN = 0, 1
MASK_NONE, MASK_PADDING, MASK_CAUSAL = 0, 1, 2


@dataclasses.dataclass(frozen=True)
class LayerShape:
    name: str
    arch: int          # POST_LN (BERT) or PRE_LN (GPT)
    d: int             # hidden width
    H: int             # heads
    Dh: int            # head width
    f: int             # FFN width
    B: int             # sequences per batch
    S: int             # tokens per sequence fed to one call
    layers: int
    mask: int
    eps: float
    w_std: float
    outlier_frac: float
    outlier_mult: float
    kv_lo: int = 0     # padding mask: sequence lengths drawn in [kv_lo, kv_hi]
    kv_hi: int = 0
    cache_len: int = 0  # decode: tokens already in the KV cache
    steps: int = 1      # decode: tokens generated


# The five workloads the benchmark contract names.
CONFIGS = {
    0: LayerShape("bert-base-1x128", POST_LN, 768, 12, 64, 3072, 1, 128, 1, MASK_NONE, 1e-12, 0.02, 0.01, 20.0),
    2: LayerShape("bert-large-32x512", POST_LN, 1024, 16, 64, 4096, 32, 512, 24, MASK_PADDING, 1e-12, 0.02, 0.01,
                  20.0, kv_lo=256, kv_hi=512),
    3: LayerShape("gpt-prefill-8x2048", PRE_LN, 4096, 32, 128, 16384, 8, 2048, 4, MASK_CAUSAL, 1e-5, 0.01, 0.005,
                  50.0),
    4: LayerShape("gpt-decode-64x1", PRE_LN, 4096, 32, 128, 16384, 64, 1, 4, MASK_PADDING, 1e-5, 0.01, 0.005, 50.0,
                  cache_len=2048, steps=128),
}
# Config 1: the stand-alone GEMM sweep.
GEMM_M = (512, 2048, 8192)
GEMM_KN = ((1024, 3072), (1024, 4096), (4096, 1024))


def rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def small(shape: LayerShape, **kw) -> LayerShape:
    """Same architecture at a reduced size (for oracle-speed parity cases)."""
    return dataclasses.replace(shape, **kw)


def layer_params(seed: int, shape: LayerShape, layer: int = 0) -> dict:
    """fp32 parameters of one transformer layer.  Weights are the mathematical
    [in, out] matrices of Y = X W (paper Sec. 2.1)."""
    g = rng(seed, 1000 + layer)
    d, f, s = shape.d, shape.f, shape.w_std
    n = lambda *sh: g.standard_normal(sh, dtype=np.float32)
    return {
        "w_qkv": n(d, 3 * d) * s, "b_qkv": n(3 * d) * s,
        "w_o": n(d, d) * s, "b_o": n(d) * s,
        "w_1": n(d, f) * s, "b_1": n(f) * s,
        "w_2": n(f, d) * s, "b_2": n(d) * s,
        "ln1_g": 1.0 + 0.1 * n(d), "ln1_b": 0.02 * n(d),
        "ln2_g": 1.0 + 0.1 * n(d), "ln2_b": 0.02 * n(d),
    }


def embedding_ln_params(seed: int, shape: LayerShape) -> dict:
    """Gain and bias of the LayerNorm that produces the first layer's input."""
    g = rng(seed, 900)
    n = lambda *sh: g.standard_normal(sh, dtype=np.float32)
    return {"g": 1.0 + 0.1 * n(shape.d), "b": 0.02 * n(shape.d)}


def embedding_tables(seed: int, d: int, vocab: int = 30522, max_pos: int = 512, n_types: int = 2) -> dict:
    """fp32 token / position / sentence-type tables: N(0, 0.02^2) rows (the BERT initialiser), the token rows
    with a log-uniform per-row magnitude spread of 8x, so that per-row scales matter."""
    g = rng(seed, 910)
    n = lambda *sh: g.standard_normal(sh, dtype=np.float32)
    mag = np.exp(g.uniform(np.log(0.5), np.log(4.0), vocab)).astype(np.float32)
    return {"tok": n(vocab, d) * np.float32(0.02) * mag[:, None], "pos": n(max_pos, d) * np.float32(0.02),
            "type": n(n_types, d) * np.float32(0.02)}


def embedding_ids(seed: int, B: int, S: int, vocab: int = 30522, n_types: int = 2) -> dict:
    """int32 [B*S] token ids (Zipf-like: rank r drawn with weight 1/(r+10)), position ids t % S and
    sentence-type ids (0 up to a random split point of each sequence, 1 after it)."""
    g = rng(seed, 920)
    w = 1.0 / (np.arange(vocab, dtype=np.float64) + 10.0)
    tok = g.choice(vocab, size=B * S, p=w / w.sum()).astype(np.int32)
    pos = np.tile(np.arange(S, dtype=np.int32), B)
    split = g.integers(S // 4, S, B)
    typ = (np.arange(S)[None, :] >= split[:, None]).astype(np.int32).reshape(-1) % n_types
    return {"tok": tok, "pos": pos, "type": typ.astype(np.int32)}


def outlier_channels(seed: int, shape: LayerShape) -> np.ndarray:
    g = rng(seed, 800)
    k = int(round(shape.outlier_frac * shape.d))
    return np.sort(g.choice(shape.d, size=k, replace=False))


def activations(seed: int, shape: LayerShape, tokens: int, stream: int = 0) -> np.ndarray:
    """fp32 [tokens, d] hidden states: N(0,1), outlier channels (fixed per seed) scaled."""
    g = rng(seed, 2000 + stream)
    h = g.standard_normal((tokens, shape.d), dtype=np.float32)
    ch = outlier_channels(seed, shape)
    h[:, ch] *= np.float32(shape.outlier_mult)
    return h


def kv_lengths(seed: int, shape: LayerShape, B: int | None = None) -> np.ndarray:
    """int32 [B] sequence lengths, uniform in [kv_lo, kv_hi]."""
    g = rng(seed, 3000)
    B = shape.B if B is None else B
    return g.integers(shape.kv_lo, shape.kv_hi + 1, size=B, dtype=np.int32)


def int8_codes(seed: int, shape_, stream: int = 0) -> np.ndarray:
    """Uniform INT8 codes in [-127, 127]."""
    g = rng(seed, 4000 + stream)
    return g.integers(-127, 128, size=shape_, dtype=np.int8)


def gemm_case(seed: int, M: int, K: int, N: int, outlier_rows: bool = False) -> dict:
    """One case of the stand-alone W8A8 GEMM sweep: uniform INT8 codes, per-token and
    per-column fp32 scales; the outlier variant multiplies 1 % of the row scales by 20."""
    g = rng(seed, 5000)
    A = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    Bt = g.integers(-127, 128, size=(N, K), dtype=np.int8)
    a_s = (g.uniform(0.5, 2.0, size=M) / 127.0).astype(np.float32)
    b_s = (0.02 * g.uniform(0.5, 2.0, size=N) / 127.0).astype(np.float32)
    bias = (0.02 * g.standard_normal(N)).astype(np.float32)
    if outlier_rows:
        rows = g.choice(M, size=max(1, M // 100), replace=False)
        a_s[rows] *= np.float32(20.0)
    return {"A": A, "Bt": Bt, "a_row_scale": a_s, "b_col_scale": b_s, "bias": bias}
