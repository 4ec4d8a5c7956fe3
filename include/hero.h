/* hero.h -- C ABI of libhero: the W8A8 transformer-layer forward of ZeroQuant-HERO
 * (arXiv 2310.17723) for AMD MI355X (gfx950).
 *
 * Common rules for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned, valid
 *     until the work enqueued by the call has finished.  Nothing is retained afterwards.
 *   - The library allocates no device memory and keeps no state between calls.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise with the host.
 *   - Arguments are validated on the host BEFORE anything is launched; on error nothing
 *     has been enqueued and a non-zero hero_status is returned.  No exceptions cross the ABI.
 *   - Sizes and strides are int64_t, in ELEMENTS.  Outputs must not alias inputs unless
 *     the entry point says so.
 *   - Numeric conventions (Sec. 2.1 quantizes symmetrically and uniformly to 8-bit integers): codes
 *     lie in [-127,127]; rounding is to nearest, ties to even; a dynamic scale is absmax/127 (1.0 for an
 *     all-zero row).  Integer contractions are exact in int32.  The DEFINITION of every quantization
 *     divides by the scale with IEEE fp32 division, and the entry points whose results are bit-exact
 *     against that definition compute exactly that: REQUANT / DEQUANT / raw GeMM^quant (their scales are
 *     multiplied, never divided by), LN^quant without LayerNorm (pure token-wise quantization), the
 *     weight preparation.  Three places multiply by a reciprocal instead, all behind fp32 transcendental
 *     or statistical arithmetic whose own rounding already differs from the definition's, so that their
 *     codes agree with it up to +-1 step on <= 0.1 % of the elements (the tolerance class of those paths):
 *     LN^quant behind a LayerNorm (v_rcp_f32 of the row scale, v_rsq_f32 of the variance), GELU^quant
 *     (1 / S_a[j]: v_rcp_f32, or the correctly rounded quotient in the overlapped-epilogue kernel), and
 *     Softmax^quant (the normaliser and 1 / S_p are folded into the exponent).
 *   - The kernel an entry point runs is chosen from the problem size alone; the library reads no
 *     environment variable.  (include/hero_debug.h has test hooks that force a kernel.)
 */
#ifndef HERO_H
#define HERO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HERO_OK = 0,
    HERO_ERR_NULL = 1,        /* a required pointer is NULL                           */
    HERO_ERR_SHAPE = 2,       /* a size is negative / inconsistent                    */
    HERO_ERR_ALIGN = 3,       /* a pointer or leading dimension breaks 16-byte rule   */
    HERO_ERR_UNSUPPORTED = 4, /* valid request this build has no kernel for           */
    HERO_ERR_WORKSPACE = 5,   /* workspace missing or too small                       */
    HERO_ERR_LAUNCH = 6       /* the HIP runtime refused a launch                     */
} hero_status;

typedef enum { HERO_I8 = 0, HERO_U8 = 1, HERO_I32 = 2, HERO_F16 = 3, HERO_BF16 = 4, HERO_F32 = 5,
               HERO_F8E4M3 = 6 /* OCP E4M3: bias 7, max 448, no infinities */ } hero_dtype;

typedef enum {
    HERO_EPI_RAW_I32 = 0,      /* C = acc                                   (int32)        */
    HERO_EPI_DEQUANT = 1,      /* C = y (+ residual)                        (f16/bf16)     */
    HERO_EPI_DEQUANT_GELU = 2, /* C = GELU(y)                               (f16/bf16)     */
    HERO_EPI_REQUANT = 3,      /* C = sat(rne(y))                           (int8)         */
    HERO_EPI_GELU_REQUANT = 4  /* C = sat(rne(GELU(y) / out_col_scale[j]))  (int8; +-1 LSB class, see above) */
} hero_epilogue;

typedef enum { HERO_MASK_NONE = 0, HERO_MASK_PADDING = 1, HERO_MASK_CAUSAL = 2 } hero_mask;

const char* hero_strerror(hero_status s);

/* LN^quant: LayerNorm of the SUM of its inputs with a token-wise (TWQ) INT8 output.
 * Paper: Sec. 2.1 (TWQ is computed on the fly and fused into LayerNorm), Sec. 2.2.2 last
 * line of the quantized attention flow  S_out X_out,int8 = LN^quant(S_in X_in,int8, X_o,int8 S_o),
 * Sec. 2.2.3 last line of the quantized MLP flow.
 *
 *   s[i][j] = x[i][j] * x_row_scale[i] + r[i][j] * r_col_scale[j]
 *   y       = (s - mean_j s) / sqrt(var_j s + eps) * gamma[j] + beta[j]     (biased variance)
 *   y_scale[i] = max_j |y[i][j]| / 127 ;  y_q[i][j] = sat(rne(y[i][j] / y_scale[i]))
 *
 *   x        [M,D] row-major.  HERO_I8 with x_row_scale[M] (TWQ), or HERO_BF16/HERO_F16
 *            with x_row_scale == NULL.
 *   r        optional second addend [M,D] (NULL = none): HERO_I8 with r_col_scale[D] (FWQ),
 *            or HERO_BF16/HERO_F16 with r_col_scale == NULL.
 *   gamma, beta  f32[D].  gamma == NULL: no LayerNorm, the sum itself is quantized per
 *            token (then beta must be NULL too).  beta may be NULL (= 0).
 *   y_q [M,D] int8 and y_scale[M] f32 are always written.
 *   y_hp     optional [M,D] copy of y in y_hp_dt (HERO_BF16/HERO_F16) for a BF16 consumer.
 *   The 8-bit inputs may hold OCP E4M3 codes instead (x_dt / r_dt = HERO_F8E4M3, the same scales; the
 *   FP8 variant of Sec. 2.1); two 8-bit addends must be of one format (else HERO_ERR_UNSUPPORTED).
 * Constraints: D % 16 == 0, 16 <= D <= 8192 for INT8 x, <= 4096 for 16-bit x (a row lives in one
 * wavefront's registers; HERO_ERR_UNSUPPORTED beyond).  M == 0 is a no-op.
 * Statistics are fp32 (mean, then variance about the mean) with the row held in registers.
 */
hero_status hero_ln_quant(const void* x, hero_dtype x_dt, const float* x_row_scale,
                          const void* r, hero_dtype r_dt, const float* r_col_scale,
                          const float* gamma, const float* beta, float eps,
                          int64_t M, int64_t D,
                          int8_t* y_q, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream);

/* LN^quant with a token-wise FP8 output (Sec. 2.1: the 8-bit format may be FP8): everything as for
 * hero_ln_quant, except
 *   y_scale[i] = max_j |y[i][j]| / 448 ;  y_q[i][j] = e4m3(y[i][j] / y_scale[i])
 * (OCP E4M3 bytes, IEEE fp32 division, round to nearest even, saturated to +-448): the A operand and
 * a_row_scale of hero_fp8_gemm. */
hero_status hero_ln_quant_fp8(const void* x, hero_dtype x_dt, const float* x_row_scale,
                              const void* r, hero_dtype r_dt, const float* r_col_scale,
                              const float* gamma, const float* beta, float eps,
                              int64_t M, int64_t D,
                              void* y_q, float* y_scale, void* y_hp, hero_dtype y_hp_dt, void* stream);

/* Embedding LN^quant.  Paper: Sec. 2.2.1,
 *   S_emb X_emb,int8 = LN^quant(S_xt X_t,int8, X_p, X_s)
 * the token embedding is stored as INT8 codes with one TWQ scale per table row, the (small) position
 * and sentence-type tables stay in 16-bit floating point; the LayerNorm of their sum is quantized
 * per token exactly as in hero_ln_quant:
 *   h[i][j] = tok_scale[t] * tok_table[t][j] + pos_table[p][j] (+ type_table[s][j]),
 *             t = tok_ids[i], p = pos_ids[i], s = type_ids[i]
 *   y = LayerNorm_j(h) * gamma + beta ;  y_scale[i] = max_j |y| / 127 ;  y_q = sat(rne(y / y_scale[i]))
 *   tok_ids, pos_ids, type_ids   int32[T] (device).  An index outside its table cannot be reported
 *            from an asynchronous call: it is clamped into the table.
 *   tok_table [V,D] int8, tok_scale [V] f32;  pos_table [P,D], type_table [NT,D] in pt_dt
 *            (HERO_BF16 / HERO_F16);  type_table == NULL: no third addend (type_ids ignored).
 *   gamma [D] required, beta [D] or NULL;  y_q [T,D] int8 and y_scale [T] f32 are written.
 * Constraints: D % 16 == 0, 16 <= D <= 8192; tables and y_q 16-byte aligned.  T == 0 is a no-op.
 */
hero_status hero_embed_ln_quant(const int32_t* tok_ids, const int32_t* pos_ids, const int32_t* type_ids,
                                const int8_t* tok_table, const float* tok_scale, int64_t V,
                                const void* pos_table, int64_t P,
                                const void* type_table, int64_t NT, hero_dtype pt_dt,
                                const float* gamma, const float* beta, float eps,
                                int64_t T, int64_t D, int8_t* y_q, float* y_scale, void* stream);

/* GeMM^quant: INT8 x INT8 -> INT32 GEMM with the dequantization and the static FWQ/SQ
 * scales fused behind it.  Paper: Sec. 2.1 (Y = XW, column-wise weight scales, weights in
 * column-major format), Sec. 2.2.2 (dequantization and pre-determined scales fused into
 * the INT8 GeMM; X_q,int8 = Round(GeMM^quant(X_in,int8, W_q,int8, S_in, S_q)) once S_q is
 * folded into the weight), Sec. 2.2.3 (GELU^quant).
 *
 *   acc[i][j] = sum_k A[i][k] * Bt[j][k]                      exact int32
 *   t = float(acc);  t = t * a_row_scale[i]  (skipped if NULL);
 *   y = fma(t, b_col_scale[j], bias[j])      (bias NULL = 0)   -- this order, fp32
 *   then the epilogue `epi` (see hero_epilogue).  GELU is the exact erf form.
 *
 *   A   [M,K] int8 row-major, leading dimension lda.
 *   Bt  [N,K] int8, K contiguous (the paper's column-major W[K,N]), leading dimension ldb.
 *   residual  optional [M,N] HERO_BF16/HERO_F16 (DEQUANT only), leading dimension ldr; added
 *       in fp32 before the final rounding.  C may alias residual when ldc == ldr and the
 *       dtypes match (in-place residual stream).
 *   out_col_scale[N]  required for GELU_REQUANT (the FWQ scale S_a), ignored otherwise.
 *   C   [M,N] in c_dt, leading dimension ldc: HERO_I32 (RAW), HERO_F16/HERO_BF16 (DEQUANT*),
 *       HERO_I8 (REQUANT*).  Other pairs -> HERO_ERR_UNSUPPORTED.
 * Constraints: K % 64 == 0; lda, ldb multiples of 16; ldc, ldr multiples of 4; base
 * pointers 16-byte aligned; M, N arbitrary (>= 0; zero is a no-op); M < 2^23 (HERO_ERR_SHAPE beyond).
 * The tile shape is chosen from the problem size; every choice gives the same result.
 */
hero_status hero_int8_gemm(const int8_t* A, int64_t lda, const float* a_row_scale,
                           const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                           const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                           hero_epilogue epi, const float* out_col_scale,
                           void* C, hero_dtype c_dt, int64_t ldc,
                           int64_t M, int64_t N, int64_t K, void* stream);

/* The same GeMM^quant (Sec. 2.1, 2.2.2, 2.2.3; identical arguments, results and constraints) with a
 * caller-owned scratch buffer for skinny problems with a long K (M <= 128, K >= 8192, few output tiles:
 * the widest linear of a decode step): K is split over several workgroups per output tile so that
 * every CU streams a share of the weights; the exact
 * int32 partial sums go through the scratch and a second kernel adds them and applies the
 * epilogue, so the result does not depend on the split.
 *   hero_int8_gemm_workspace_bytes(M, N, K): bytes of scratch this shape can use (0: it would not
 *       split; any buffer, or none, is accepted then).
 *   workspace  device memory, 256-byte aligned (else HERO_ERR_WORKSPACE), at least that many bytes
 *       (NULL or smaller: the call runs like hero_int8_gemm).  Pure scratch: no initialisation is
 *       needed and nothing is kept between calls, so consecutive calls ON ONE STREAM can share it;
 *       calls that may overlap on the GPU (different streams) need buffers of their own.
 */
size_t hero_int8_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
hero_status hero_int8_gemm_ws(const int8_t* A, int64_t lda, const float* a_row_scale,
                              const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                              const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                              hero_epilogue epi, const float* out_col_scale,
                              void* C, hero_dtype c_dt, int64_t ldc,
                              int64_t M, int64_t N, int64_t K,
                              void* workspace, size_t workspace_bytes, void* stream);

/* hero_int8_gemm for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Arguments, results (bit for bit) and constraints are those of
 * hero_int8_gemm_ws; the split-K scratch is a fixed array of HERO_STATIC_SCRATCH_BYTES inside the library (one
 * copy per GPU, held until the process ends) instead of a caller's buffer.  The call allocates nothing.
 *   - A shape whose split needs more than HERO_STATIC_SCRATCH_BYTES (hero_int8_gemm_workspace_bytes(M, N, K))
 *     is refused with HERO_ERR_WORKSPACE before anything is launched; shapes that do not split need no scratch
 *     and always run.
 *   - Every call on one GPU shares that GPU's array: calls that may overlap on the GPU (different streams,
 *     concurrently replayed graphs) race on it.  Calls on one stream are ordered and safe.  The array is pure
 *     scratch: every plane is written before it is read, nothing needs clearing between calls.
 *   - The device current at the call must be the one `stream` belongs to. */
#define HERO_STATIC_SCRATCH_BYTES (16u << 20)
hero_status hero_int8_gemm_static(const int8_t* A, int64_t lda, const float* a_row_scale,
                                  const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                  const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                  hero_epilogue epi, const float* out_col_scale,
                                  void* C, hero_dtype c_dt, int64_t ldc,
                                  int64_t M, int64_t N, int64_t K, void* stream);

/* The FP8 variant of GeMM^quant (Sec. 2.1 names FP8 as an 8-bit format the method applies to as well): the
 * same operation and epilogue as hero_int8_gemm with OCP E4M3 operands and fp32 accumulation on the
 * matrix cores.
 *   acc[i][j] = sum_k A[i][k] * Bt[j][k]     every product exact; the sum in fp32 (hardware order)
 *   then t = acc * a_row_scale[i] (skipped if NULL); y = fma(t, b_col_scale[j], bias[j]); epilogue:
 *   DEQUANT / DEQUANT_GELU -> C in HERO_F16 / HERO_BF16 (residual as for hero_int8_gemm);
 *   REQUANT -> e4m3(y), GELU_REQUANT -> e4m3(GELU(y) / out_col_scale[j]): C in HERO_F8E4M3, round
 *   to nearest even, saturated to +-448.  HERO_EPI_RAW_I32 does not exist here.
 *   A [M,K], Bt [N,K] E4M3 bytes, K contiguous.  Constraints as for hero_int8_gemm.
 * Token-wise FP8 activations use scale = max|x| / 448 per row; static scales fold as for INT8.
 * The order of the fp32 accumulation depends on the tile the library picks for a shape (fixed for a
 * given shape and build), so results are reproducible but not bit-identical across tile choices. */
hero_status hero_fp8_gemm(const void* A, int64_t lda, const float* a_row_scale,
                          const void* Bt, int64_t ldb, const float* b_col_scale,
                          const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                          hero_epilogue epi, const float* out_col_scale,
                          void* C, hero_dtype c_dt, int64_t ldc,
                          int64_t M, int64_t N, int64_t K, void* stream);

/* INT8 attention: QK^T, Softmax^quant, PV.  Paper: Sec. 2.2.2 quantized flow
 *   A = S_q S_k X_q,int8 X_k,int8^T / sqrt(d)   (not quantized; d~ = S_q S_k / sqrt(d))
 *   S_p P_int8 = Softmax^quant(A)               (unsigned codes: softmax has no negatives)
 *   X_attn,int8 S_attn = S_p S_v P_int8 X_v,int8
 * Per (batch b, head h), query i, key k, channel e (j = h*Dh + e):
 *   a[i][k]  = float(sum_e q k) * qk_scale                 keys outside the mask are left out
 *   p        = softmax_k(a)   (fp32);   P[i][k] = sat_[0,255](rne(p / p_scale))
 *   acc[i][e]= sum_k P[i][k] * v[k][e]                     exact int32
 *   out_dt == HERO_I8 :  out[b*Sq+i][j] = sat(rne(float(acc) * out_col_scale[j]))
 *   out_dt == HERO_BF16/HERO_F16 :  out = float(acc) * out_col_scale[0]   (out_scale_is_scalar = 1)
 *
 *   q [B,Sq,H,Dh], k/v [B,Skv,H,Dh] int8 given by a base pointer and 4 element strides in
 *   the order (batch, position, head, channel); the channel stride must be 1 and the
 *   others multiples of 16, so the operands can be views into a fused [T,3d] QKV buffer
 *   or a [B,H,Smax,Dh] KV cache.
 *   mask: key k is visible to query i iff k < kv_len[b] (when kv_len != NULL; required for
 *   HERO_MASK_PADDING) and, for HERO_MASK_CAUSAL, k <= i + (len_b - Sq) with len_b =
 *   min(kv_len[b], Skv) (or Skv): the last query sees the last valid key.  With
 *   HERO_MASK_PADDING and Sq == Skv (self-attention over a padded batch) the positions
 *   i >= kv_len[b] are padding as queries too and see no key.  A query that sees no key
 *   outputs 0.  The same rules hold for every attention entry point of this header.
 *   out [B*Sq, H*Dh] row-major with leading dimension ldo.
 * Constraints: Dh in {64, 128}; B, H, Sq, Skv >= 0 (zero is a no-op).
 * The softmax is normalised BEFORE it is quantized, as the equation says, so the kernel
 * makes two passes over the keys (row max and sum first, codes and PV second).
 */
hero_status hero_int8_attn(const int8_t* q, const int64_t q_strides[4],
                           const int8_t* k, const int64_t k_strides[4],
                           const int8_t* v, const int64_t v_strides[4],
                           int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                           float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                           hero_mask mask, const int32_t* kv_len,
                           void* out, hero_dtype out_dt, int64_t ldo, void* stream);

/* INT8 attention with an ONLINE Softmax^quant: a single-sweep VARIANT of the flow above, not the
 * equation of Sec. 2.2.2 (which normalises before it quantizes).  The probabilities are quantized
 * un-normalised, in blocks of 64 keys, against the running row maximum, and normalised once at the
 * end; the largest weight of a row always has code 255 whatever the sequence length.
 * Per (b, h), query i, visible keys 0 .. n-1 in blocks t = [64t, 64t + 64) (aligned to key 0):
 *   a[k]   = float(sum_e q k) * qk_scale_h[h]              one d~ per head (device array f32[H])
 *   m_t    = max(m_{t-1}, max_{k in t} a[k])               running maximum
 *   c[k]   = sat_[0,255](rne(255 exp(a[k] - m_t)))         unsigned codes of block t
 *   O[e]   = sum_t exp(m_t - m_T) sum_{k in t} c[k] v[k][e]   (integer inner sums, exact)
 *   L      = sum_t exp(m_t - m_T) sum_{k in t} c[k]
 *   y      = O[e] / L * out_col_scale[j] / p_scale ;  INT8: sat(rne(y)), 16-bit: y with
 *            out_col_scale[0]
 * out_col_scale and p_scale mean what they mean for hero_int8_attn (S_p S_v / S_attn[j] and S_p;
 * S_p cancels), so the two are interchangeable; masks, strides, constraints and errors are the
 * same, plus HERO_ERR_NULL without qk_scale_h.  Any Sq runs through the same kernel (a one-query
 * decode call is served but not specialised). */
hero_status hero_int8_attn_online(const int8_t* q, const int64_t q_strides[4],
                                  const int8_t* k, const int64_t k_strides[4],
                                  const int8_t* v, const int64_t v_strides[4],
                                  int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                                  const float* qk_scale_h, float p_scale, const float* out_col_scale,
                                  int out_scale_is_scalar, hero_mask mask, const int32_t* kv_len,
                                  void* out, hero_dtype out_dt, int64_t ldo, void* stream);

/* FP8 attention: the quantized attention flow of Sec. 2.2.2 with E4M3 as the 8-bit format (Sec. 2.1
 * allows INT8 or FP8).  q, k, v hold OCP E4M3 bytes (device; the same shapes, element strides and
 * views as hero_int8_attn).  Per (b, h), query i, visible keys k:
 *   a[k]  = (sum_e q[i][e] k[k][e]) * qk_scale          fp32 accumulation on the matrix cores
 *   p     = softmax(a)                                   fp32, normalised BEFORE it is quantized
 *   P_f8  = e4m3(min(p / p_scale, 448))                  non-negative E4M3 codes; p_scale = 1/448 maps
 *                                                        p = 1 to the largest code
 *   acc[e] = sum_k P_f8[k] v[k][e]                       fp32 accumulation on the matrix cores
 *   out_dt HERO_F8E4M3: e4m3(sat(acc[e] * out_col_scale[h*Dh+e])), out_col_scale = S_p S_v / S_attn[j]
 *   out_dt HERO_F16 / HERO_BF16: acc[e] * out_col_scale[0]  (out_scale_is_scalar must be 1)
 * Masks, kv_len, constraints (Dh 64 or 128, strides multiples of 16, 16-byte aligned bases, ldo) and
 * errors as for hero_int8_attn; the 8-bit output type is HERO_F8E4M3 (HERO_I8 -> HERO_ERR_UNSUPPORTED).
 * A query with no visible key outputs 0.  A one-query call (Sq == 1, Skv <= 16384) takes the
 * cache-streaming kernel, as for INT8 (fp32 sums on the vector ALU there).  The matrix cores add the 8 products of a lane group with 13
 * fractional bits below the largest of them, so results agree with an exactly accumulated reference
 * up to an adjacent E4M3 code on a small fraction of the outputs, not bit for bit. */
hero_status hero_fp8_attn(const void* q, const int64_t q_strides[4],
                          const void* k, const int64_t k_strides[4],
                          const void* v, const int64_t v_strides[4],
                          int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh,
                          float qk_scale, float p_scale, const float* out_col_scale, int out_scale_is_scalar,
                          hero_mask mask, const int32_t* kv_len,
                          void* out, hero_dtype out_dt, int64_t ldo, void* stream);

/* ---- one transformer layer (Sec. 2.2.2 + 2.2.3 chained, Sec. 2.3 / Table 1 modes) ---- */

typedef enum { HERO_ARCH_POST_LN = 0, HERO_ARCH_PRE_LN = 1 } hero_arch;

/* mode_mask: one bit per switchable module (Sec. 2.3; the columns of Table 1 after "Embedding"); set = INT8,
 * clear = 16-bit.  Table 1's modes are HERO_MODE_M1 / M2 / M3; HERO_MODE_M0 (no module bit) is the all-16-bit
 * layer, the FP16 row of Table 2.  A 16-bit module hands 16-bit values on and the method has no stand-alone
 * quantization kernel, so: ATTN set needs QKV set (the INT8 attention reads SQ codes), ATTN_OUT set needs ATTN
 * set, FC2 set needs FC1 set (GELU^quant codes); any other subset is HERO_ERR_UNSUPPORTED.
 * HERO_M_F16: the 16-bit type of the layer -- switched modules, the 16-bit copies between them, the PRE_LN
 * residual stream h -- is FP16 instead of BF16.
 * HERO_M_FP8 (only together with all five module bits): the 8-bit format of the whole layer is OCP E4M3
 * instead of INT8 (Sec. 2.1).  Every int8_t* of hero_layer_weights / hero_layer_io then holds E4M3 bytes
 * (weights quantized column-wise to max|column| / 448, static scales calibrated to 448, p_scale = 1/448),
 * and the layer runs hero_ln_quant_fp8 / hero_fp8_gemm / hero_fp8_attn in place of the INT8 entry points. */
enum { HERO_M_QKV = 1, HERO_M_ATTN = 2, HERO_M_ATTN_OUT = 4, HERO_M_FC1 = 8, HERO_M_FC2 = 16, HERO_M_FP8 = 32,
       HERO_M_F16 = 64 };
#define HERO_MODE_M3 (HERO_M_QKV | HERO_M_ATTN | HERO_M_ATTN_OUT | HERO_M_FC1 | HERO_M_FC2)
#define HERO_MODE_M2 (HERO_M_QKV | HERO_M_ATTN | HERO_M_ATTN_OUT | HERO_M_FC1)
#define HERO_MODE_M1 (HERO_M_QKV | HERO_M_FC1)
#define HERO_MODE_M0 0

typedef struct {
    int32_t arch;       /* hero_arch                                          */
    int32_t d, H, Dh, f; /* hidden width, heads, head width (H*Dh == d), FFN width */
    float eps;          /* LayerNorm epsilon                                  */
    int32_t mask;       /* hero_mask                                          */
    uint32_t mode_mask; /* HERO_M_* bits                                      */
} hero_layer_desc;

/* Prepared (folded, column-quantized) parameters, all device pointers.  INT8 weights are
 * [N][K] (K contiguous); *_s are their f32 column scales; biases are f32 and already
 * folded with the output scale where the output is requantized.  A 16-bit module takes its
 * weight in *_bf16 / *_hp ([N][K] in the layer's 16-bit type -- bf16, or fp16 with HERO_M_F16 --,
 * unfolded) and ignores the INT8 fields. */
typedef struct {
    const int8_t* w_qkv; const float* w_qkv_s; const float* b_qkv;          /* [3d][d] */
    const int8_t* w_o;   const float* w_o_s;   const float* b_o;            /* [d][d]  */
    const int8_t* w_1;   const float* w_1_s;   const float* b_1;            /* [f][d]  */
    const int8_t* w_2;   const float* w_2_s;   const float* b_2;            /* [d][f]  */
    const void* w_o_bf16; const void* w_2_bf16;                             /* 16-bit attention-output / FC2 */
    const float* ln1_g; const float* ln1_b; const float* ln2_g; const float* ln2_b;
    const float* S_o;   /* [d] FWQ scale of X_o  (POST_LN, INT8 attention-output)      */
    const float* S_x2;  /* [d] FWQ scale of X_2  (POST_LN, INT8 FC2)                   */
    const float* S_a;   /* [f] FWQ scale of A = GELU(X_1) (INT8 FC2)                   */
    const float* attn_out_scale; /* [d] S_p S_v / S_attn[j] (INT8 attention-output) or
                                    1 float S_p S_v (16-bit attention-output)          */
    float qk_scale;     /* d~ = S_q S_k / sqrt(Dh)  (INT8 attention) or 1/sqrt(Dh) (16-bit) */
    float p_scale;      /* S_p                                                         */
    const void* w_qkv_hp; const void* w_1_hp;                               /* 16-bit QKV / FC1 */
} hero_layer_weights;

typedef struct {
    int64_t B, S;            /* sequences and new tokens per sequence; T = B*S rows    */
    /* POST_LN: TWQ input (read when the QKV module is INT8) and output (always written) */
    const int8_t* x_q; const float* x_scale;     /* [T,d] int8, [T] f32               */
    int8_t* out_q;     float* out_scale;         /* [T,d] int8, [T] f32               */
    /* PRE_LN: 16-bit residual stream, updated IN PLACE */
    void* h;                                     /* [T,d] bf16 (fp16 with HERO_M_F16)  */
    const int32_t* kv_len;   /* [B] visible keys per sequence INCLUDING this call's S tokens;
                                NULL = S for every sequence (no cache, no padding)     */
    /* optional INT8 KV cache [B,H,Smax,Dh] (PRE_LN or POST_LN; INT8 attention only): this call's K/V codes
       are written at positions kv_len[b]-S .. kv_len[b]-1 and attention reads the cache.   */
    int8_t* k_cache; int8_t* v_cache; int64_t Smax;
    /* POST_LN with a 16-bit QKV module: the layer input [T,d] in the layer's 16-bit type (x_q / x_scale are then
       not read).  out_hp (optional, any mode): the 16-bit copy of the layer output, i.e. the x_hp of a successor
       whose QKV module is 16-bit. */
    const void* x_hp; void* out_hp;
    /* optional hint (may be NULL / 0; never written, changes no result): device memory that the caller's NEXT call
       reads first, typically the next layer's w_qkv.  The layer's last GeMM^quant requests its lines while it runs, so
       that they wait in the cache hierarchy instead of in HBM when the next call's first tiles ask for them.  At most
       next_read_bytes bytes from next_read are read; 4-byte aligned; a region above 8 MB is ignored (it would not
       survive in the cache until it is used). */
    const void* next_read; size_t next_read_bytes;
} hero_layer_io;

/* Bytes of scratch hero_layer_fwd needs for T = B*S rows of this layer. */
size_t hero_layer_workspace_bytes(const hero_layer_desc* desc, int64_t B, int64_t S);

/* One W8A8 layer: enqueues LN^quant, the four GeMM^quant, the attention and (POST_LN) the
 * closing LN^quant on `stream`, with no host synchronisation.  Paper: Sec. 2.2.2, 2.2.3,
 * Sec. 2.3 Table 1.  `workspace` is device scratch of at least
 * hero_layer_workspace_bytes() bytes, 256-byte aligned, owned by the caller; its contents
 * are undefined afterwards.  Supported mode masks: see mode_mask above. */
hero_status hero_layer_fwd(const hero_layer_desc* desc, const hero_layer_weights* w, const hero_layer_io* io,
                           void* workspace, size_t workspace_bytes, void* stream);

/* 16-bit side of a switched module (Sec. 2.3, Table 1: a module that is not INT8 runs in FP16 / BF16):
 * C = act(A Wt^T + bias) (+ residual).  dt = HERO_BF16 or HERO_F16 is the type of A [M,K] (lda), Wt [N][K] (ldb),
 * residual [M,N] or NULL (ldr; C may alias it) and C [M,N] (ldc); bias f32[N] or NULL; gelu != 0 applies erf-GELU
 * before the residual.  fp32 accumulation on the matrix cores.  Constraints: K % 32 == 0; lda, ldb multiples of 8,
 * ldc, ldr of 4; base pointers 16-byte aligned.  hero_bf16_gemm is hero_hp_gemm with dt = HERO_BF16. */
hero_status hero_hp_gemm(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                         const float* bias, const void* residual, int64_t ldr, int gelu,
                         void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, void* stream);
hero_status hero_bf16_gemm(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                           const float* bias, const void* residual, int64_t ldr, int gelu,
                           void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream);

/* 16-bit attention core softmax(q k^T * scale) v with the same operand description and mask rules as
 * hero_int8_attn (strides multiples of 8 elements); q, k, v and out [B*Sq, H*Dh] in dt (HERO_BF16 / HERO_F16).
 * hero_bf16_attn is hero_hp_attn with dt = HERO_BF16. */
hero_status hero_hp_attn(const void* q, const int64_t q_strides[4],
                         const void* k, const int64_t k_strides[4],
                         const void* v, const int64_t v_strides[4],
                         int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                         hero_mask mask, const int32_t* kv_len, void* out, int64_t ldo, hero_dtype dt, void* stream);
hero_status hero_bf16_attn(const void* q, const int64_t q_strides[4],
                           const void* k, const int64_t k_strides[4],
                           const void* v, const int64_t v_strides[4],
                           int64_t B, int64_t H, int64_t Sq, int64_t Skv, int64_t Dh, float scale,
                           hero_mask mask, const int32_t* kv_len, void* out, int64_t ldo, void* stream);

/* Model-load-time operators (not on the hot path): the pre-processing phase of the method on the GPU.
 *
 * hero_absmax_cols -- calibration statistic of the static scales (Sec. 2.1: FWQ / SQ scales are
 *   calibrated in a pre-processing phase; Sec. 3: ranges recorded over calibration batches):
 *     col_absmax[j] = max(col_absmax[j], max_i |x[i][j]|)
 *   x [T,D] HERO_F32 / HERO_BF16 / HERO_F16, leading dimension ldx; col_absmax f32[D] is a RUNNING
 *   maximum (in/out: zero it before the first batch).  An FWQ scale is col_absmax[j] / 127, an SQ
 *   scale the maximum over j divided by 127.  Exact (a maximum has no rounding).
 *
 * hero_weight_fold_quant -- scale folding (Sec. 2.2.2: W~_q = W_q / S_q, W~_o = S_attn W_o / S_o;
 *   Sec. 2.2.3: W~_2 = S_a W_2 / S_x2) and column-wise weight quantization (Sec. 2.1):
 *     W~[k][n] = row_mult[k] * W[k][n] / col_div[n]     fp64: multiply, then divide; one cast to fp32
 *     col_scale[n] = max_k |W~[k][n]| / 127  (1 for an all-zero column)
 *     Wt[n][k] = sat(rne(W~[k][n] / col_scale[n]))       IEEE fp32 division
 *   W [K,N] f32 row-major (the paper's W: input rows, output columns), leading dimension ldw;
 *   row_mult f32[K] or NULL (= 1), col_div f32[N] or NULL (= 1); Wt [N,K] int8, leading dimension
 *   ldwt (K contiguous: the operand layout of hero_int8_gemm); col_scale f32[N].
 *   hero_weight_fold_quant_fp8: the FP8 variant (Sec. 2.1): the same fold, col_scale[n] = max / 448 and
 *   Wt[n][k] = e4m3(W~[k][n] / col_scale[n]) (OCP E4M3 bytes: the operand of hero_fp8_gemm).
 * All return HERO_ERR_SHAPE / HERO_ERR_NULL / HERO_ERR_UNSUPPORTED before any launch. */
hero_status hero_absmax_cols(const void* x, hero_dtype x_dt, int64_t ldx, int64_t T, int64_t D,
                             float* col_absmax, void* stream);
hero_status hero_weight_fold_quant(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                   int64_t K, int64_t N, int8_t* Wt, int64_t ldwt, float* col_scale, void* stream);
hero_status hero_weight_fold_quant_fp8(const float* W, int64_t ldw, const float* row_mult, const float* col_div,
                                       int64_t K, int64_t N, void* Wt, int64_t ldwt, float* col_scale, void* stream);

/* Library build identification: target architecture string, e.g. "gfx950". */
const char* hero_build_arch(void);

#ifdef __cplusplus
}
#endif
#endif /* HERO_H */
