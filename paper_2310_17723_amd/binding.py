"""ctypes binding of libhero.so: same names as the C ABI, torch tensors in place of raw
pointers.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C

import torch

# enums of include/hero.h
I8, U8, I32, F16, BF16, F32 = range(6)
EPI_RAW_I32, EPI_DEQUANT, EPI_DEQUANT_GELU, EPI_REQUANT, EPI_GELU_REQUANT = range(5)
MASK_NONE, MASK_PADDING, MASK_CAUSAL = range(3)
ARCH_POST_LN, ARCH_PRE_LN = 0, 1
M_QKV, M_ATTN, M_ATTN_OUT, M_FC1, M_FC2, M_FP8, M_F16 = 1, 2, 4, 8, 16, 32, 64
MODE_M3 = M_QKV | M_ATTN | M_ATTN_OUT | M_FC1 | M_FC2
MODE_M2 = M_QKV | M_ATTN | M_ATTN_OUT | M_FC1
MODE_M1 = M_QKV | M_FC1
MODE_M0 = 0

F8E4M3 = 6
_DT = {torch.int8: I8, torch.uint8: U8, torch.int32: I32, torch.float16: F16, torch.bfloat16: BF16,
       torch.float32: F32, torch.float8_e4m3fn: F8E4M3}

vp, i64, f32, i32 = C.c_void_p, C.c_int64, C.c_float, C.c_int


class LayerDesc(C.Structure):
    _fields_ = [("arch", C.c_int32), ("d", C.c_int32), ("H", C.c_int32), ("Dh", C.c_int32), ("f", C.c_int32),
                ("eps", C.c_float), ("mask", C.c_int32), ("mode_mask", C.c_uint32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, vp) for n in (
        "w_qkv", "w_qkv_s", "b_qkv", "w_o", "w_o_s", "b_o", "w_1", "w_1_s", "b_1", "w_2", "w_2_s", "b_2",
        "w_o_bf16", "w_2_bf16", "ln1_g", "ln1_b", "ln2_g", "ln2_b", "S_o", "S_x2", "S_a", "attn_out_scale")] + \
        [("qk_scale", C.c_float), ("p_scale", C.c_float), ("w_qkv_hp", vp), ("w_1_hp", vp)]


class LayerIO(C.Structure):
    _fields_ = [("B", i64), ("S", i64), ("x_q", vp), ("x_scale", vp), ("out_q", vp), ("out_scale", vp),
                ("h", vp), ("kv_len", vp), ("k_cache", vp), ("v_cache", vp), ("Smax", i64), ("x_hp", vp), ("out_hp", vp),
                ("next_read", vp), ("next_read_bytes", C.c_size_t)]


SYMBOLS = {
    "hero_strerror": (C.c_char_p, [i32]),
    "hero_build_arch": (C.c_char_p, []),
    "hero_ln_quant": (i32, [vp, i32, vp, vp, i32, vp, vp, vp, f32, i64, i64, vp, vp, vp, i32, vp]),
    "hero_ln_quant_fp8": (i32, [vp, i32, vp, vp, i32, vp, vp, vp, f32, i64, i64, vp, vp, vp, i32, vp]),
    "hero_embed_ln_quant": (i32, [vp, vp, vp, vp, vp, i64, vp, i64, vp, i64, i32, vp, vp, f32, i64, i64, vp, vp, vp]),
    "hero_absmax_cols": (i32, [vp, i32, i64, i64, i64, vp, vp]),
    "hero_weight_fold_quant": (i32, [vp, i64, vp, vp, i64, i64, vp, i64, vp, vp]),
    "hero_weight_fold_quant_fp8": (i32, [vp, i64, vp, vp, i64, i64, vp, i64, vp, vp]),
    "hero_int8_gemm": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64, vp]),
    "hero_fp8_gemm": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64, vp]),
    "hero_int8_gemm_workspace_bytes": (C.c_size_t, [i64, i64, i64]),
    "hero_int8_gemm_ws": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64,
                                vp, C.c_size_t, vp]),
    "hero_int8_gemm_tile": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64, vp, i32]),
    "hero_fp8_gemm_tile": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64, vp, i32]),
    "hero_hp_gemm_tile": (i32, [vp, i64, vp, i64, vp, vp, i64, i32, vp, i64, i64, i64, i64, i32, vp, i32]),
    "hero_hp_gemm": (i32, [vp, i64, vp, i64, vp, vp, i64, i32, vp, i64, i64, i64, i64, i32, vp]),
    "hero_hp_attn": (i32, [vp, C.POINTER(i64), vp, C.POINTER(i64), vp, C.POINTER(i64), i64, i64, i64, i64, i64,
                           f32, i32, vp, vp, i64, i32, vp]),
    "hero_int8_gemm_static": (i32, [vp, i64, vp, vp, i64, vp, vp, vp, i32, i64, i32, vp, vp, i32, i64, i64, i64, i64, vp]),
    "hero_int8_attn": (i32, [vp, C.POINTER(i64), vp, C.POINTER(i64), vp, C.POINTER(i64), i64, i64, i64, i64, i64,
                             f32, f32, vp, i32, i32, vp, vp, i32, i64, vp]),
    "hero_fp8_attn": (i32, [vp, C.POINTER(i64), vp, C.POINTER(i64), vp, C.POINTER(i64), i64, i64, i64, i64, i64,
                            f32, f32, vp, i32, i32, vp, vp, i32, i64, vp]),
    "hero_int8_attn_online": (i32, [vp, C.POINTER(i64), vp, C.POINTER(i64), vp, C.POINTER(i64), i64, i64, i64, i64, i64,
                                    vp, f32, vp, i32, i32, vp, vp, i32, i64, vp]),
    "hero_layer_workspace_bytes": (C.c_size_t, [C.POINTER(LayerDesc), i64, i64]),
    "hero_layer_fwd": (i32, [C.POINTER(LayerDesc), C.POINTER(LayerWeights), C.POINTER(LayerIO), vp, C.c_size_t, vp]),
    "hero_bf16_gemm": (i32, [vp, i64, vp, i64, vp, vp, i64, i32, vp, i64, i64, i64, i64, vp]),
    "hero_bf16_attn": (i32, [vp, C.POINTER(i64), vp, C.POINTER(i64), vp, C.POINTER(i64), i64, i64, i64, i64, i64,
                             f32, i32, vp, vp, i64, vp]),
}


class HeroError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"libhero: {msg} (status {status})")
        self.status = status


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _strides4(t):
    assert t.dim() == 4
    return (i64 * 4)(*t.stride())


class Hero:
    def __init__(self, path: str):
        self.lib = C.CDLL(path)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(self.lib, name)      # AttributeError if the library lacks the symbol
            fn.restype, fn.argtypes = res, args

    # ------------------------------------------------------------------ helpers
    def strerror(self, status: int) -> str:
        return self.lib.hero_strerror(status).decode()

    def build_arch(self) -> str:
        return self.lib.hero_build_arch().decode()

    def _check(self, status: int):
        if status != 0:
            raise HeroError(status, self.strerror(status))

    # ------------------------------------------------------------------ LN^quant
    def hero_ln_quant(self, x, x_row_scale=None, r=None, r_col_scale=None, gamma=None, beta=None, eps=1e-5,
                      y_hp_dtype=None, y_q=None, y_scale=None, y_hp=None, stream=None, fp8=False):
        """Returns (y_q int8 [M,D] (float8_e4m3fn with fp8=True: hero_ln_quant_fp8), y_scale f32 [M], y_hp or None)."""
        M, D = x.shape
        dev = x.device
        y_q = torch.empty((M, D), dtype=torch.float8_e4m3fn if fp8 else torch.int8, device=dev) if y_q is None else y_q
        y_scale = torch.empty((M,), dtype=torch.float32, device=dev) if y_scale is None else y_scale
        if y_hp is None and y_hp_dtype is not None:
            y_hp = torch.empty((M, D), dtype=y_hp_dtype, device=dev)
        for t in (x, r):
            assert t is None or t.is_contiguous()
        fn = self.lib.hero_ln_quant_fp8 if fp8 else self.lib.hero_ln_quant
        st = fn(_ptr(x), _DT[x.dtype], _ptr(x_row_scale), _ptr(r),
                                    _DT[r.dtype] if r is not None else 0, _ptr(r_col_scale), _ptr(gamma), _ptr(beta),
                                    float(eps), M, D, _ptr(y_q), _ptr(y_scale), _ptr(y_hp),
                                    _DT[y_hp.dtype] if y_hp is not None else 0, _stream(stream))
        self._check(st)
        return y_q, y_scale, y_hp

    def hero_embed_ln_quant(self, tok_ids, pos_ids, type_ids, tok_table, tok_scale, pos_table, type_table,
                            gamma, beta, eps, y_q=None, y_scale=None, stream=None):
        """int32 id vectors [T]; tok_table [V,D] int8 + tok_scale [V]; pos/type tables bf16 or f16 (type may be None)."""
        T = tok_ids.shape[0]
        V, D = tok_table.shape
        if y_q is None:
            y_q = torch.empty((T, D), dtype=torch.int8, device=tok_table.device)
        if y_scale is None:
            y_scale = torch.empty((T,), dtype=torch.float32, device=tok_table.device)
        st = self.lib.hero_embed_ln_quant(_ptr(tok_ids), _ptr(pos_ids), _ptr(type_ids), _ptr(tok_table), _ptr(tok_scale), V,
                                          _ptr(pos_table), pos_table.shape[0], _ptr(type_table),
                                          type_table.shape[0] if type_table is not None else 0, _DT[pos_table.dtype],
                                          _ptr(gamma), _ptr(beta), float(eps), T, D, _ptr(y_q), _ptr(y_scale), _stream(stream))
        self._check(st)
        return y_q, y_scale

    # ------------------------------------------------------------------ model-load-time operators
    def hero_absmax_cols(self, x, col_absmax=None, stream=None):
        """Running per-column max |x| (x [T,D] f32 / bf16 / f16).  Returns the updated f32[D] tensor."""
        T, D = x.shape
        assert x.stride(1) == 1
        if col_absmax is None:
            col_absmax = torch.zeros(D, dtype=torch.float32, device=x.device)
        self._check(self.lib.hero_absmax_cols(_ptr(x), _DT[x.dtype], x.stride(0) if T > 1 else max(D, x.stride(0)), T, D,
                                              _ptr(col_absmax), _stream(stream)))
        return col_absmax

    def hero_weight_fold_quant(self, W, row_mult=None, col_div=None, stream=None, fp8=False):
        """W [K,N] f32 -> (codes [N,K] int8, col_scale [N] f32) of row_mult[:,None] * W / col_div[None,:];
        fp8=True: E4M3 codes (torch.float8_e4m3fn) with scale max / 448 (hero_weight_fold_quant_fp8)."""
        K, N = W.shape
        assert W.dtype == torch.float32 and W.stride(1) == 1
        Wt = torch.empty((N, K), dtype=torch.float8_e4m3fn if fp8 else torch.int8, device=W.device)
        s = torch.empty(N, dtype=torch.float32, device=W.device)
        fn = self.lib.hero_weight_fold_quant_fp8 if fp8 else self.lib.hero_weight_fold_quant
        self._check(fn(_ptr(W), W.stride(0) if K > 1 else max(N, W.stride(0)), _ptr(row_mult),
                       _ptr(col_div), K, N, _ptr(Wt), K, _ptr(s), _stream(stream)))
        return Wt, s

    # ------------------------------------------------------------------ GeMM^quant
    def hero_int8_gemm(self, A, Bt, a_row_scale=None, b_col_scale=None, bias=None, residual=None,
                       epi=EPI_RAW_I32, out_col_scale=None, out_dtype=torch.int32, C_out=None, stream=None,
                       workspace=None, static_scratch=False, tile=None):
        """A [M,K] int8, Bt [N,K] int8 (row strides may exceed K).  Returns C [M,N].
        workspace: optional uint8 tensor (hero_int8_gemm_workspace_bytes) -> hero_int8_gemm_ws;
        static_scratch=True -> hero_int8_gemm_static (the library's built-in scratch; pass C_out to allocate nothing);
        tile=<code> -> the test hook hero_int8_gemm_tile (include/hero_debug.h: the kernel forced)."""
        M, K = A.shape
        N = Bt.shape[0]
        assert Bt.shape[1] == K and A.stride(1) == 1 and Bt.stride(1) == 1
        if C_out is None:
            C_out = torch.empty((M, N), dtype=out_dtype, device=A.device)
        assert C_out.stride(1) == 1
        args = (_ptr(A), A.stride(0) if M > 1 else max(K, A.stride(0)), _ptr(a_row_scale),
                _ptr(Bt), Bt.stride(0) if N > 1 else max(K, Bt.stride(0)), _ptr(b_col_scale),
                _ptr(bias), _ptr(residual),
                _DT[residual.dtype] if residual is not None else 0,
                residual.stride(0) if residual is not None else 0, int(epi), _ptr(out_col_scale),
                _ptr(C_out), _DT[C_out.dtype], C_out.stride(0), M, N, K)
        if tile is not None:
            st = self.lib.hero_int8_gemm_tile(*args, _stream(stream), int(tile))
        elif static_scratch:
            st = self.lib.hero_int8_gemm_static(*args, _stream(stream))
        elif workspace is None:
            st = self.lib.hero_int8_gemm(*args, _stream(stream))
        else:
            st = self.lib.hero_int8_gemm_ws(*args, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream))
        self._check(st)
        return C_out

    def hero_fp8_gemm(self, A, Bt, a_row_scale, b_col_scale, bias=None, residual=None, epi=EPI_DEQUANT,
                      out_col_scale=None, out_dtype=torch.bfloat16, C_out=None, stream=None, tile=None):
        """The FP8 variant: A [M,K], Bt [N,K] hold E4M3 bytes (torch.float8_e4m3fn or uint8 storage).
        out_dtype torch.float8_e4m3fn for the REQUANT epilogues, float16 / bfloat16 for DEQUANT."""
        M, K = A.shape
        N = Bt.shape[0]
        assert Bt.shape[1] == K and A.stride(1) == 1 and Bt.stride(1) == 1 and A.element_size() == 1 and Bt.element_size() == 1
        if C_out is None:
            C_out = torch.empty((M, N), dtype=out_dtype, device=A.device)
        args = (_ptr(A), A.stride(0) if M > 1 else max(K, A.stride(0)), _ptr(a_row_scale),
                _ptr(Bt), Bt.stride(0) if N > 1 else max(K, Bt.stride(0)), _ptr(b_col_scale),
                _ptr(bias), _ptr(residual), _DT[residual.dtype] if residual is not None else 0,
                residual.stride(0) if residual is not None else 0, int(epi), _ptr(out_col_scale),
                _ptr(C_out), _DT[C_out.dtype], C_out.stride(0), M, N, K, _stream(stream))
        st = self.lib.hero_fp8_gemm(*args) if tile is None else self.lib.hero_fp8_gemm_tile(*args, int(tile))
        self._check(st)
        return C_out

    def hero_int8_gemm_workspace_bytes(self, M, N, K) -> int:
        return int(self.lib.hero_int8_gemm_workspace_bytes(M, N, K))

    # ------------------------------------------------------------------ INT8 attention
    def hero_int8_attn(self, q, k, v, qk_scale, p_scale, out_col_scale, out_scale_is_scalar=False,
                       mask=MASK_NONE, kv_len=None, out_dtype=torch.int8, out=None, stream=None):
        """q [B,Sq,H,Dh], k/v [B,Skv,H,Dh] int8 views (unit channel stride).  Returns [B*Sq, H*Dh]."""
        B, Sq, H, Dh = q.shape
        Skv = k.shape[1]
        if out is None:
            out = torch.empty((B * Sq, H * Dh), dtype=out_dtype, device=q.device)
        st = self.lib.hero_int8_attn(_ptr(q), _strides4(q), _ptr(k), _strides4(k), _ptr(v), _strides4(v),
                                     B, H, Sq, Skv, Dh, float(qk_scale), float(p_scale), _ptr(out_col_scale),
                                     int(bool(out_scale_is_scalar)), int(mask), _ptr(kv_len), _ptr(out),
                                     _DT[out.dtype], out.stride(0), _stream(stream))
        self._check(st)
        return out

    def hero_fp8_attn(self, q, k, v, qk_scale, p_scale, out_col_scale, out_scale_is_scalar=False,
                      mask=MASK_NONE, kv_len=None, out_dtype=torch.float8_e4m3fn, out=None, stream=None):
        """The FP8 variant: q [B,Sq,H,Dh], k/v [B,Skv,H,Dh] hold E4M3 bytes (torch.float8_e4m3fn or uint8 storage).
        out_dtype torch.float8_e4m3fn (per-column scales) or float16 / bfloat16 (scalar scale)."""
        B, Sq, H, Dh = q.shape
        Skv = k.shape[1]
        assert q.element_size() == 1 and k.element_size() == 1 and v.element_size() == 1
        if out is None:
            out = torch.empty((B * Sq, H * Dh), dtype=out_dtype, device=q.device)
        odt = F8E4M3 if out.element_size() == 1 else _DT[out.dtype]
        st = self.lib.hero_fp8_attn(_ptr(q), _strides4(q), _ptr(k), _strides4(k), _ptr(v), _strides4(v),
                                    B, H, Sq, Skv, Dh, float(qk_scale), float(p_scale), _ptr(out_col_scale),
                                    int(bool(out_scale_is_scalar)), int(mask), _ptr(kv_len), _ptr(out),
                                    odt, out.stride(0), _stream(stream))
        self._check(st)
        return out

    def hero_int8_attn_online(self, q, k, v, qk_scale_h, p_scale, out_col_scale, out_scale_is_scalar=False,
                              mask=MASK_NONE, kv_len=None, out_dtype=torch.int8, out=None, stream=None):
        """The single-sweep variant (online Softmax^quant); qk_scale_h: f32[H] device tensor, one d~ per head."""
        B, Sq, H, Dh = q.shape
        Skv = k.shape[1]
        assert qk_scale_h is None or (qk_scale_h.dtype == torch.float32 and qk_scale_h.numel() == H)
        if out is None:
            out = torch.empty((B * Sq, H * Dh), dtype=out_dtype, device=q.device)
        st = self.lib.hero_int8_attn_online(_ptr(q), _strides4(q), _ptr(k), _strides4(k), _ptr(v), _strides4(v),
                                            B, H, Sq, Skv, Dh, _ptr(qk_scale_h), float(p_scale), _ptr(out_col_scale),
                                            int(bool(out_scale_is_scalar)), int(mask), _ptr(kv_len), _ptr(out),
                                            _DT[out.dtype], out.stride(0), _stream(stream))
        self._check(st)
        return out

    # ------------------------------------------------------------------ BF16 side
    def hero_hp_gemm(self, A, Wt, bias=None, residual=None, gelu=False, C_out=None, stream=None, tile=None):
        """The 16-bit side of a switched module: A, Wt (and residual) bf16 or fp16 tensors of ONE type, which is
        also the result's."""
        M, K = A.shape
        N = Wt.shape[0]
        assert A.dtype == Wt.dtype and A.dtype in (torch.bfloat16, torch.float16)
        if C_out is None:
            C_out = torch.empty((M, N), dtype=A.dtype, device=A.device)
        args = (_ptr(A), A.stride(0), _ptr(Wt), Wt.stride(0), _ptr(bias), _ptr(residual),
                residual.stride(0) if residual is not None else 0, int(bool(gelu)),
                _ptr(C_out), C_out.stride(0), M, N, K, _DT[A.dtype], _stream(stream))
        st = self.lib.hero_hp_gemm(*args) if tile is None else self.lib.hero_hp_gemm_tile(*args, int(tile))
        self._check(st)
        return C_out

    def hero_bf16_gemm(self, A, Wt, bias=None, residual=None, gelu=False, C_out=None, stream=None, tile=None):
        if tile is not None:
            return self.hero_hp_gemm(A, Wt, bias, residual, gelu, C_out, stream, tile)
        M, K = A.shape
        N = Wt.shape[0]
        if C_out is None:
            C_out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
        st = self.lib.hero_bf16_gemm(_ptr(A), A.stride(0), _ptr(Wt), Wt.stride(0), _ptr(bias), _ptr(residual),
                                     residual.stride(0) if residual is not None else 0, int(bool(gelu)),
                                     _ptr(C_out), C_out.stride(0), M, N, K, _stream(stream))
        self._check(st)
        return C_out

    def hero_hp_attn(self, q, k, v, scale, mask=MASK_NONE, kv_len=None, out=None, stream=None):
        B, Sq, H, Dh = q.shape
        Skv = k.shape[1]
        assert q.dtype in (torch.bfloat16, torch.float16) and k.dtype == q.dtype and v.dtype == q.dtype
        if out is None:
            out = torch.empty((B * Sq, H * Dh), dtype=q.dtype, device=q.device)
        st = self.lib.hero_hp_attn(_ptr(q), _strides4(q), _ptr(k), _strides4(k), _ptr(v), _strides4(v),
                                   B, H, Sq, Skv, Dh, float(scale), int(mask), _ptr(kv_len), _ptr(out),
                                   out.stride(0), _DT[q.dtype], _stream(stream))
        self._check(st)
        return out

    def hero_bf16_attn(self, q, k, v, scale, mask=MASK_NONE, kv_len=None, out=None, stream=None):
        B, Sq, H, Dh = q.shape
        Skv = k.shape[1]
        if out is None:
            out = torch.empty((B * Sq, H * Dh), dtype=torch.bfloat16, device=q.device)
        st = self.lib.hero_bf16_attn(_ptr(q), _strides4(q), _ptr(k), _strides4(k), _ptr(v), _strides4(v),
                                     B, H, Sq, Skv, Dh, float(scale), int(mask), _ptr(kv_len), _ptr(out),
                                     out.stride(0), _stream(stream))
        self._check(st)
        return out

    # ------------------------------------------------------------------ layer
    def layer_desc(self, arch, d, H, Dh, f, eps, mask, mode_mask=MODE_M3) -> LayerDesc:
        return LayerDesc(int(arch), int(d), int(H), int(Dh), int(f), float(eps), int(mask), int(mode_mask))

    def layer_weights(self, tensors: dict, qk_scale: float, p_scale: float) -> LayerWeights:
        """tensors: device tensors keyed by the field names of hero_layer_weights; the dict
        must stay alive while the struct is in use."""
        w = LayerWeights()
        for name, _ in LayerWeights._fields_:
            if name in ("qk_scale", "p_scale"):
                continue
            t = tensors.get(name)
            setattr(w, name, None if t is None else t.data_ptr())
        w.qk_scale, w.p_scale = float(qk_scale), float(p_scale)
        return w

    def hero_layer_workspace_bytes(self, desc: LayerDesc, B: int, S: int) -> int:
        return int(self.lib.hero_layer_workspace_bytes(C.byref(desc), B, S))

    def hero_layer_fwd(self, desc, weights, B, S, workspace, *, x_q=None, x_scale=None, out_q=None, out_scale=None,
                       h=None, kv_len=None, k_cache=None, v_cache=None, x_hp=None, out_hp=None, next_read=None, stream=None):
        ptr = lambda t: None if t is None else t.data_ptr()
        io = LayerIO(B, S, *(ptr(t) for t in (x_q, x_scale, out_q, out_scale, h, kv_len, k_cache, v_cache)),
                     k_cache.shape[2] if k_cache is not None else 0, ptr(x_hp), ptr(out_hp),
                     ptr(next_read), 0 if next_read is None else next_read.numel() * next_read.element_size())
        st = self.lib.hero_layer_fwd(C.byref(desc), C.byref(weights), C.byref(io), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream))
        self._check(st)
