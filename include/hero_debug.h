/* hero_debug.h -- test and tuning hooks of libhero.  NOT part of the product interface (include/hero.h): the
 * product entry points choose their kernel from the problem size alone and read no environment variable.
 * Each hook is the entry point of the same name without the suffix, with one more argument that forces the
 * kernel; arguments, constraints, error behaviour and results are otherwise identical (for INT8 operands every
 * kernel gives bit-identical results; for FP8 and BF16 operands the order of the fp32 accumulation, and with it
 * the last bits, depends on the tile).  A forced kernel that cannot run the shape falls back to its closest
 * relative; an unknown tile code returns HERO_ERR_UNSUPPORTED.  All pointers are device pointers. */
#ifndef HERO_DEBUG_H
#define HERO_DEBUG_H

#include "hero.h"

#ifdef __cplusplus
extern "C" {
#endif

/* GeMM^quant (Sec. 2.1, 2.2.2, 2.2.3) with the kernel forced.  tile: 0 = 128x128 tile staged through registers,
 * 1 = 256x256 direct-to-LDS, one tile per workgroup, 2 = 64x64 (small and skinny problems), 7 = 256x256
 * persistent, 8 = 128x128 persistent (two workgroups per CU), 9 = 256x128 persistent with the epilogue of a tile
 * inside the main loop of the next one (K >= 1024, no fused residual).  Never splits K. */
hero_status hero_int8_gemm_tile(const int8_t* A, int64_t lda, const float* a_row_scale,
                                const int8_t* Bt, int64_t ldb, const float* b_col_scale,
                                const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                                hero_epilogue epi, const float* out_col_scale,
                                void* C, hero_dtype c_dt, int64_t ldc,
                                int64_t M, int64_t N, int64_t K, void* stream, int tile);

/* The FP8 variant (Sec. 2.1).  tile: 0 = register-staged kernels, 7 / 8 = persistent 256x256 / 128x128. */
hero_status hero_fp8_gemm_tile(const void* A, int64_t lda, const float* a_row_scale,
                               const void* Bt, int64_t ldb, const float* b_col_scale,
                               const float* bias, const void* residual, hero_dtype res_dt, int64_t ldr,
                               hero_epilogue epi, const float* out_col_scale,
                               void* C, hero_dtype c_dt, int64_t ldc,
                               int64_t M, int64_t N, int64_t K, void* stream, int tile);

/* The 16-bit side of a switched module (Sec. 2.3, Table 1; hero_hp_gemm).  tile: 0 = the plain 128x128 kernel,
 * 7 / 8 = the persistent 256x256 / 128x128 kernel. */
hero_status hero_hp_gemm_tile(const void* A, int64_t lda, const void* Wt, int64_t ldb,
                              const float* bias, const void* residual, int64_t ldr, int gelu,
                              void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hero_dtype dt, void* stream, int tile);

#ifdef __cplusplus
}
#endif
#endif /* HERO_DEBUG_H */
