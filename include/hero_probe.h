/* hero_probe.h -- C ABI of libhero_probe, the measuring instruments of bench.py.  NOT part of the product
 * library: nothing in libhero calls these and only the benchmark loads them.  They measure, on the machine at
 * hand, what the hardware sustains, beside the published peaks the roofline fractions are quoted against.
 * All pointers are device pointers (except `ops` outputs, host); every call only enqueues work on `stream`.
 * Return value: 0 ok, 1 NULL pointer, 2 bad size / mode, 3 misaligned, 4 unsupported combination, 6 launch failed. */
#ifndef HERO_PROBE_H
#define HERO_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Register-only loop of v_mfma_i32_32x32x32_i8: one 512-thread workgroup per CU, `iters` x 16 instructions per
 * wave, on near-constant (random_bytes == 0) or random operand bytes.  *ops (host, may be NULL) receives the
 * integer operations the launch performs; sink is one device int32 the kernel may write. */
int hero_probe_mfma_i8(int random_bytes, int64_t iters, int32_t* sink, double* ops, void* stream);

/* Matrix and vector instructions on one SIMD.  mode 0: every wave issues, `iters` times, 8 x (one matrix
 * instruction, valu_per_mfma fp32 fma); mode 1: the fma alone; mode 2: the same work split by wave (one wave of
 * each SIMD issues only matrix instructions, the other only fma).  valu_per_mfma in {0 (mode 0 only), 4, 8}.
 * *mfma_ops / *valu_wave_instr (host, may be NULL): integer operations and 64-lane vector instructions issued. */
int hero_probe_coissue(int mode, int valu_per_mfma, int64_t iters, int32_t* sink, double* mfma_ops,
                       double* valu_wave_instr, void* stream);

/* HBM streams over `bytes` (a multiple of 16; 16-byte aligned): a copy with 1 or 4 independent 16-byte loads in
 * flight per lane, a read-only pass, a write-only pass, the runtime's device-to-device copy. */
int hero_probe_copy(const void* src, void* dst, int64_t bytes, int loads_in_flight, void* stream);
int hero_probe_read(const void* src, int64_t bytes, int32_t* sink, void* stream);
int hero_probe_write(void* dst, int64_t bytes, void* stream);
int hero_probe_memcpy(const void* src, void* dst, int64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HERO_PROBE_H */
