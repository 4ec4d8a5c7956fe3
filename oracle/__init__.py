"""CPU oracle for the ZeroQuant-HERO W8A8 layer forward (numpy front-end).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` may import this package.  It never imports the
HIP library or its binding, and the HIP library never imports it.

The arithmetic lives in ``hero_oracle.cpp`` (plain C++17, one loop nest per equation of
the paper); this file only marshals numpy arrays into it.  ``layer.py`` chains the
operators into the paper's attention + MLP flow and holds the offline preparation
(calibration, scale folding, weight quantization).

16-bit floats are carried as ``numpy.uint16`` bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hero_oracle.cpp")
_LIB = os.path.join(_HERE, "libhero_oracle.so")

I8, U8, I32, F16, BF16, F32, F8 = range(7)
EPI_RAW_I32, EPI_DEQUANT, EPI_DEQUANT_GELU, EPI_REQUANT, EPI_GELU_REQUANT = range(5)
MASK_NONE, MASK_PADDING, MASK_CAUSAL = range(3)


_SAN_LIB = os.path.join(_HERE, "libhero_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the C++ oracle with g++ (no intrinsics, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized() -> str:
    """The same source with AddressSanitizer + UndefinedBehaviorSanitizer (a checker of the checker: the pins
    are re-run against this build by tests/test_oracle_sanitized.py).  Selected with HERO_ORACLE_SANITIZED=1 in a
    process that has the sanitizer runtime preloaded."""
    if not os.path.exists(_SAN_LIB) or os.path.getmtime(_SAN_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-Wall", "-o", _SAN_LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _SAN_LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_sanitized() if os.environ.get("HERO_ORACLE_SANITIZED") == "1" else build())
        _lib.orc_f32_to_bf16.restype = C.c_uint16
        _lib.orc_f32_to_bf16.argtypes = [C.c_float]
        _lib.orc_bf16_to_f32.restype = C.c_float
        _lib.orc_bf16_to_f32.argtypes = [C.c_uint16]
        _lib.orc_f32_to_f16.restype = C.c_uint16
        _lib.orc_f32_to_f16.argtypes = [C.c_float]
        _lib.orc_f16_to_f32.restype = C.c_float
        _lib.orc_f16_to_f32.argtypes = [C.c_uint16]
        _lib.orc_gelu.restype = C.c_double
        _lib.orc_gelu.argtypes = [C.c_double]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    """Pointer to a C-contiguous numpy array (None -> NULL)."""
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C-contiguous"
    return a.ctypes.data_as(C.c_void_p)


def _i64(x):
    return C.c_int64(int(x))


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ 16-bit formats
def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty(x.shape, np.uint16)
    lib().orc_f32_to_bf16_n(_p(x), _i64(x.size), _p(y))
    return y


def bf16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32).reshape(h.shape)


def f32_to_f16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty(x.shape, np.uint16)
    lib().orc_f32_to_f16_n(_p(x), _i64(x.size), _p(y))
    return y


def f16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    y = np.empty(h.shape, np.float32)
    lib().orc_f16_to_f32_n(_p(h), _i64(h.size), _p(y))
    return y


def hp_to_f32(h: np.ndarray, dt: int) -> np.ndarray:
    """Decode a stored activation (uint16 bit patterns or float32) to float32."""
    if dt == F32:
        return np.asarray(h, dtype=np.float32)
    if dt == BF16:
        return bf16_to_f32(h)
    return f16_to_f32(h)


_NP_OF = {I8: np.int8, U8: np.uint8, I32: np.int32, F16: np.uint16, BF16: np.uint16, F32: np.float32, F8: np.uint8}


# ------------------------------------------------------------------ O1 / O2
def quant_twq(x: np.ndarray):
    """Token-wise dynamic quantization (paper Sec. 2.1, TWQ)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, D = x.shape
    q = np.empty((M, D), np.int8)
    s = np.empty((M,), np.float32)
    lib().orc_quant_twq(_p(x), _i64(M), _i64(D), _p(q), _p(s))
    return q, s


def quant_static(x: np.ndarray, scale) -> np.ndarray:
    """FWQ (``scale`` a length-D vector) or SQ (``scale`` a python float) quantization."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, D = x.shape
    q = np.empty((M, D), np.int8)
    if np.ndim(scale) == 0:
        lib().orc_quant_static(_p(x), _i64(M), _i64(D), None, C.c_float(float(scale)), _p(q))
    else:
        cs = np.ascontiguousarray(scale, dtype=np.float32)
        assert cs.shape == (D,)
        lib().orc_quant_static(_p(x), _i64(M), _i64(D), _p(cs), C.c_float(0.0), _p(q))
    return q


def weight_quant(W: np.ndarray):
    """Column-wise weight quantization; W is [K, N]; returns codes [N, K] and scales [N]."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    Wt = np.empty((N, K), np.int8)
    s = np.empty((N,), np.float32)
    lib().orc_weight_quant(_p(W), _i64(K), _i64(N), _p(Wt), _p(s))
    return Wt, s


def weight_fold_quant(W, row_mult=None, col_div=None):
    """Fold static activation scales into a weight and quantize it column-wise (Sec. 2.2.2: W~_q = W_q / S_q,
    W~_o = S_attn W_o / S_o; Sec. 2.2.3: W~_2 = S_a W_2 / S_x2; Sec. 2.1 column-wise weight scales):
    W~[k][n] = row_mult[k] * W[k][n] / col_div[n] in fp64 (multiply, then divide), one cast to fp32, then
    weight_quant.  W is [K, N]; returns codes [N, K] and scales [N]."""
    Wd = np.asarray(W, np.float64)
    if row_mult is not None:
        Wd = np.asarray(row_mult, np.float64)[:, None] * Wd
    if col_div is not None:
        Wd = Wd / np.asarray(col_div, np.float64)[None, :]
    return weight_quant(Wd.astype(np.float32))


def weight_fold_quant_fp8(W, row_mult=None, col_div=None):
    """The FP8 variant (Sec. 2.1) of weight_fold_quant: the same folds in fp64 and one cast to fp32, then column-wise
    E4M3 codes with scale max|column| / 448 (the token-wise FP8 quantizer applied to the transposed weight).
    W is [K, N]; returns codes uint8 [N, K] and scales [N]."""
    Wd = np.asarray(W, np.float64)
    if row_mult is not None:
        Wd = np.asarray(row_mult, np.float64)[:, None] * Wd
    if col_div is not None:
        Wd = Wd / np.asarray(col_div, np.float64)[None, :]
    return quant_twq_fp8(np.ascontiguousarray(Wd.astype(np.float32).T))


def absmax_cols(x, running=None):
    """Calibration statistic of FWQ / SQ (Sec. 2.1, Sec. 3: the range recorded over calibration data, no
    truncation): per-column max |x| over the rows, combined with a running maximum.  x fp32 [T, D]."""
    m = np.abs(np.asarray(x, np.float32)).max(axis=0) if len(x) else np.zeros(np.shape(x)[1], np.float32)
    return m if running is None else np.maximum(m, np.asarray(running, np.float32))


# ------------------------------------------------------------------ O3 / O4
def gemm_i32(A: np.ndarray, Bt: np.ndarray) -> np.ndarray:
    A = np.ascontiguousarray(A, np.int8)
    Bt = np.ascontiguousarray(Bt, np.int8)
    M, K = A.shape
    N, K2 = Bt.shape
    assert K == K2
    Cm = np.empty((M, N), np.int32)
    lib().orc_gemm_i32(_p(A), _i64(K), _p(Bt), _i64(K), _i64(M), _i64(N), _i64(K), _p(Cm))
    return Cm


def gemm_i64(A: np.ndarray, Bt: np.ndarray) -> np.ndarray:
    A = np.ascontiguousarray(A, np.int8)
    Bt = np.ascontiguousarray(Bt, np.int8)
    M, K = A.shape
    N, _ = Bt.shape
    Cm = np.empty((M, N), np.int64)
    lib().orc_gemm_i64(_p(A), _i64(K), _p(Bt), _i64(K), _i64(M), _i64(N), _i64(K), _p(Cm))
    return Cm


def int8_gemm(A, Bt, *, a_row_scale=None, b_col_scale=None, bias=None, residual=None, res_dt=BF16,
              epi=EPI_RAW_I32, out_col_scale=None, c_dt=I32) -> np.ndarray:
    """GeMM^quant with its fused epilogue (paper Sec. 2.2.2 / 2.2.3)."""
    A = np.ascontiguousarray(A, np.int8)
    Bt = np.ascontiguousarray(Bt, np.int8)
    M, K = A.shape
    N, K2 = Bt.shape
    assert K == K2
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, np.float32)
    a_row_scale, b_col_scale, bias, out_col_scale = map(f32, (a_row_scale, b_col_scale, bias, out_col_scale))
    if residual is not None:
        residual = np.ascontiguousarray(residual, _NP_OF[res_dt])
        assert residual.shape == (M, N)
    Cm = np.empty((M, N), _NP_OF[c_dt])
    rc = lib().orc_int8_gemm(_p(A), _i64(K), _p(a_row_scale), _p(Bt), _i64(K), _p(b_col_scale), _p(bias),
                             _p(residual), C.c_int(res_dt), _i64(N), C.c_int(epi), _p(out_col_scale),
                             _p(Cm), C.c_int(c_dt), _i64(N), _i64(M), _i64(N), _i64(K))
    if rc != 0:
        raise ValueError("oracle int8_gemm: invalid epilogue / dtype combination")
    return Cm


# ------------------------------------------------------------------ O4f: the FP8 (OCP E4M3) variant
def e4m3_to_f32(c) -> np.ndarray:
    c = np.ascontiguousarray(c, np.uint8)
    out = np.empty(c.shape, np.float32)
    lib().orc_e4m3_to_f32_n(_p(c), _i64(c.size), _p(out))
    return out


def f32_to_e4m3(x) -> np.ndarray:
    """Round to nearest even, saturate to +-448, NaN -> 0x7F."""
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint8)
    lib().orc_f32_to_e4m3_n(_p(x), _i64(x.size), _p(out))
    return out


def quant_twq_fp8(x):
    """Token-wise FP8 quantization: s = max|x| / 448 per row, q = e4m3(x / s)."""
    x = np.ascontiguousarray(x, np.float32)
    M, D = x.shape
    q = np.empty((M, D), np.uint8)
    s = np.empty((M,), np.float32)
    lib().orc_quant_twq_fp8(_p(x), _i64(M), _i64(D), _p(q), _p(s))
    return q, s


def fp8_gemm(A, Bt, *, a_row_scale=None, b_col_scale=None, bias=None, residual=None, res_dt=BF16,
             epi=EPI_DEQUANT, out_col_scale=None, c_dt=F32) -> np.ndarray:
    """The FP8 GeMM^quant: E4M3 codes in, exact sum (fp64), the INT8 path's fp32 epilogue, E4M3 or 16-bit out."""
    A = np.ascontiguousarray(A, np.uint8)
    Bt = np.ascontiguousarray(Bt, np.uint8)
    M, K = A.shape
    N, K2 = Bt.shape
    assert K == K2
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, np.float32)
    a_row_scale, b_col_scale, bias, out_col_scale = map(f32, (a_row_scale, b_col_scale, bias, out_col_scale))
    if residual is not None:
        residual = np.ascontiguousarray(residual, _NP_OF[res_dt])
        assert residual.shape == (M, N)
    Cm = np.empty((M, N), _NP_OF[c_dt])
    rc = lib().orc_fp8_gemm(_p(A), _i64(K), _p(a_row_scale), _p(Bt), _i64(K), _p(b_col_scale), _p(bias),
                            _p(residual), C.c_int(res_dt), _i64(N), C.c_int(epi), _p(out_col_scale),
                            _p(Cm), C.c_int(c_dt), _i64(N), _i64(M), _i64(N), _i64(K))
    if rc != 0:
        raise ValueError("oracle fp8_gemm: invalid epilogue / dtype combination")
    return Cm


# ------------------------------------------------------------------ O5
def ln_quant(x, x_dt, x_row_scale, r, r_dt, r_col_scale, gamma, beta, eps, y_hp_dt=None, fp8=False):
    """LN^quant: LayerNorm of the sum of the inputs, token-wise quantized output (INT8, or E4M3 with fp8=True)."""
    x = np.ascontiguousarray(x, _NP_OF[x_dt])
    M, D = x.shape
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, np.float32)
    x_row_scale, r_col_scale, gamma, beta = map(f32, (x_row_scale, r_col_scale, gamma, beta))
    if r is not None:
        r = np.ascontiguousarray(r, _NP_OF[r_dt])
        assert r.shape == (M, D)
    y_q = np.empty((M, D), np.uint8 if fp8 else np.int8)
    y_s = np.empty((M,), np.float32)
    y_hp = None if y_hp_dt is None else np.empty((M, D), _NP_OF[y_hp_dt])
    fn = lib().orc_ln_quant_fp8 if fp8 else lib().orc_ln_quant
    rc = fn(_p(x), C.c_int(x_dt), _p(x_row_scale), _p(r), C.c_int(r_dt if r is not None else 0),
                            _p(r_col_scale), _p(gamma), _p(beta), C.c_float(eps), _i64(M), _i64(D),
                            _p(y_q), _p(y_s), _p(y_hp), C.c_int(y_hp_dt if y_hp_dt is not None else 0))
    if rc != 0:
        raise ValueError("oracle ln_quant: missing scale for an INT8 input")
    return y_q, y_s, y_hp


# ------------------------------------------------------------------ O5b
def embed_ln_quant(tok_ids, pos_ids, type_ids, tok_table, tok_scale, pos_table, type_table, pt_dt, gamma, beta, eps):
    """Embedding LN^quant (Sec. 2.2.1): INT8 token table with one TWQ scale per row + position (+ type)
    rows in pt_dt (BF16 / F16 / F32) -> LayerNorm -> token-wise INT8.  type_table may be None."""
    i32 = lambda a: None if a is None else np.ascontiguousarray(a, np.int32)
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, np.float32)
    tok_ids, pos_ids, type_ids = map(i32, (tok_ids, pos_ids, type_ids))
    tok_table = np.ascontiguousarray(tok_table, np.int8)
    V, D = tok_table.shape
    T = tok_ids.shape[0]
    pos_table = np.ascontiguousarray(pos_table, _NP_OF[pt_dt])
    if type_table is not None:
        type_table = np.ascontiguousarray(type_table, _NP_OF[pt_dt])
    tok_scale, gamma, beta = map(f32, (tok_scale, gamma, beta))
    y_q = np.empty((T, D), np.int8)
    y_s = np.empty((T,), np.float32)
    rc = lib().orc_embed_ln_quant(_p(tok_ids), _p(pos_ids), _p(type_ids), _p(tok_table), _p(tok_scale), _i64(V),
                                  _p(pos_table), _i64(pos_table.shape[0]), _p(type_table),
                                  _i64(0 if type_table is None else type_table.shape[0]), C.c_int(pt_dt),
                                  _p(gamma), _p(beta), C.c_float(eps), _i64(T), _i64(D), _p(y_q), _p(y_s))
    if rc != 0:
        raise ValueError("oracle embed_ln_quant: missing argument" if rc == -1 else "oracle embed_ln_quant: index out of range")
    return y_q, y_s


# ------------------------------------------------------------------ O6
def _strides(a: np.ndarray):
    """Element strides of a 4-d array as an int64[4] ctypes array."""
    assert a.ndim == 4
    st = [s // a.itemsize for s in a.strides]
    return (C.c_int64 * 4)(*st)


def int8_attn(q, k, v, *, qk_scale, p_scale, out_col_scale, out_scale_is_scalar=False,
              mask=MASK_NONE, kv_len=None, out_dt=I8, dump_p=False):
    """INT8 attention.  q [B,Sq,H,Dh], k/v [B,Skv,H,Dh] int8 (any strides, unit channel stride)."""
    B, Sq, H, Dh = q.shape
    Skv = k.shape[1]
    ocs = np.ascontiguousarray(out_col_scale, np.float32).reshape(-1)
    if kv_len is not None:
        kv_len = np.ascontiguousarray(kv_len, np.int32)
    out = np.empty((B * Sq, H * Dh), _NP_OF[out_dt])
    pd = np.zeros((B, H, Sq, Skv), np.uint8) if dump_p else None
    base = lambda a: C.c_void_p(a.ctypes.data)
    rc = lib().orc_int8_attn(base(q), _strides(q), base(k), _strides(k), base(v), _strides(v),
                             _i64(B), _i64(H), _i64(Sq), _i64(Skv), _i64(Dh),
                             C.c_float(qk_scale), C.c_float(p_scale), _p(ocs), C.c_int(int(out_scale_is_scalar)),
                             C.c_int(mask), _p(kv_len), _p(out), C.c_int(out_dt), _i64(H * Dh), _p(pd))
    if rc != 0:
        raise ValueError("oracle int8_attn: invalid arguments")
    return (out, pd) if dump_p else out


def fp8_attn(q, k, v, *, qk_scale, p_scale, out_col_scale, out_scale_is_scalar=False,
             mask=MASK_NONE, kv_len=None, out_dt=F8, dump_p=False):
    """FP8 attention (the flow of Sec. 2.2.2 with E4M3 codes).  q [B,Sq,H,Dh], k/v [B,Skv,H,Dh] uint8 E4M3 bytes
    (any strides, unit channel stride); out_dt F8 (per-column scales) or a 16-bit / fp32 type (scalar scale)."""
    B, Sq, H, Dh = q.shape
    Skv = k.shape[1]
    assert q.dtype == np.uint8 and k.dtype == np.uint8 and v.dtype == np.uint8
    ocs = np.ascontiguousarray(out_col_scale, np.float32).reshape(-1)
    if kv_len is not None:
        kv_len = np.ascontiguousarray(kv_len, np.int32)
    out = np.empty((B * Sq, H * Dh), _NP_OF[out_dt])
    pd = np.zeros((B, H, Sq, Skv), np.uint8) if dump_p else None
    base = lambda a: C.c_void_p(a.ctypes.data)
    rc = lib().orc_fp8_attn(base(q), _strides(q), base(k), _strides(k), base(v), _strides(v),
                            _i64(B), _i64(H), _i64(Sq), _i64(Skv), _i64(Dh),
                            C.c_float(qk_scale), C.c_float(p_scale), _p(ocs), C.c_int(int(out_scale_is_scalar)),
                            C.c_int(mask), _p(kv_len), _p(out), C.c_int(out_dt), _i64(H * Dh), _p(pd))
    if rc != 0:
        raise ValueError("oracle fp8_attn: invalid arguments")
    return (out, pd) if dump_p else out


def int8_attn_online(q, k, v, *, qk_scale_h, p_scale, out_col_scale, out_scale_is_scalar=False,
                     mask=MASK_NONE, kv_len=None, out_dt=I8, kv_block=64, dump_c=False):
    """INT8 attention with the online (quantize-then-normalise) Softmax^quant variant.  qk_scale_h: one d~ per
    head.  The other arguments as for int8_attn (the same out_col_scale and p_scale)."""
    B, Sq, H, Dh = q.shape
    Skv = k.shape[1]
    ocs = np.ascontiguousarray(out_col_scale, np.float32).reshape(-1)
    qsh = np.ascontiguousarray(np.broadcast_to(np.asarray(qk_scale_h, np.float32), (H,)))
    if kv_len is not None:
        kv_len = np.ascontiguousarray(kv_len, np.int32)
    out = np.empty((B * Sq, H * Dh), _NP_OF[out_dt])
    cd = np.zeros((B, H, Sq, Skv), np.uint8) if dump_c else None
    base = lambda a: C.c_void_p(a.ctypes.data)
    rc = lib().orc_int8_attn_online(base(q), _strides(q), base(k), _strides(k), base(v), _strides(v),
                                    _i64(B), _i64(H), _i64(Sq), _i64(Skv), _i64(Dh), _i64(kv_block),
                                    _p(qsh), C.c_float(p_scale), _p(ocs), C.c_int(int(out_scale_is_scalar)),
                                    C.c_int(mask), _p(kv_len), _p(out), C.c_int(out_dt), _i64(H * Dh), _p(cd))
    if rc != 0:
        raise ValueError("oracle int8_attn_online: invalid arguments")
    return (out, cd) if dump_c else out


# ------------------------------------------------------------------ BF16 side
def hp_gemm(A, Wt, bias=None, residual=None, gelu=False, dt=BF16) -> np.ndarray:
    """The 16-bit side of a switched module (Sec. 2.3): C = act(A W + bias) (+ residual), operands, residual and
    result in `dt` (BF16 or F16 bit patterns), fp64 sums rounded once."""
    A = np.ascontiguousarray(A, np.uint16)
    Wt = np.ascontiguousarray(Wt, np.uint16)
    M, K = A.shape
    N, _ = Wt.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32)
    if residual is not None:
        residual = np.ascontiguousarray(residual, np.uint16)
    Cm = np.empty((M, N), np.uint16)
    rc = lib().orc_hp_gemm(_p(A), _i64(K), _p(Wt), _i64(K), _p(bias), _p(residual), _i64(N), C.c_int(int(gelu)),
                           _p(Cm), _i64(N), _i64(M), _i64(N), _i64(K), C.c_int(dt))
    if rc != 0:
        raise ValueError("oracle hp_gemm: dt must be BF16 or F16")
    return Cm


def bf16_gemm(A, Wt, bias=None, residual=None, gelu=False) -> np.ndarray:
    return hp_gemm(A, Wt, bias, residual, gelu, BF16)


def hp_attn(q, k, v, *, scale, mask=MASK_NONE, kv_len=None, dt=BF16) -> np.ndarray:
    B, Sq, H, Dh = q.shape
    Skv = k.shape[1]
    if kv_len is not None:
        kv_len = np.ascontiguousarray(kv_len, np.int32)
    out = np.empty((B * Sq, H * Dh), np.uint16)
    base = lambda a: C.c_void_p(a.ctypes.data)
    rc = lib().orc_hp_attn(base(q), _strides(q), base(k), _strides(k), base(v), _strides(v),
                           _i64(B), _i64(H), _i64(Sq), _i64(Skv), _i64(Dh), C.c_float(scale),
                           C.c_int(mask), _p(kv_len), _p(out), _i64(H * Dh), C.c_int(dt))
    if rc != 0:
        raise ValueError("oracle hp_attn: dt must be BF16 or F16")
    return out


def bf16_attn(q, k, v, *, scale, mask=MASK_NONE, kv_len=None) -> np.ndarray:
    return hp_attn(q, k, v, scale=scale, mask=mask, kv_len=kv_len, dt=BF16)


def f32_to_hp(x, dt):
    return f32_to_bf16(x) if dt == BF16 else f32_to_f16(x)


def gelu(x: float) -> float:
    return float(lib().orc_gelu(float(x)))
