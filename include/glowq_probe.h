/* glowq_probe.h -- two measured ceilings that the benchmark prints beside the published
 * peaks of the MI355X.  They are measurement aids in the same shared library as the GlowQ
 * forward (include/glowq.h) and no part of the method.  Return value: 0 on success, -1 a
 * required pointer is NULL, -2 a size is out of range, -7 the launch failed.  Both calls
 * enqueue one kernel on `stream` (a hipStream_t as void*, NULL = default) and return. */
#ifndef GLOWQ_PROBE_H
#define GLOWQ_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One launch that reads `bytes` (a multiple of 32768) from src (DEVICE, 16-byte aligned)
 * with 128-bit loads, eight 1 KiB wave loads in flight per wave, and does nothing else:
 * the shape of a weight stream without its arithmetic.  sink: DEVICE, one word, never
 * written in practice (it keeps the loads alive). */
int32_t glowq_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

/* One launch of 256 x waves_per_simd workgroups of 4 waves (waves_per_simd in 1..8: that
 * many waves on every SIMD of the chip) in which every wave issues iters x 8 independent
 * 16x16x32 matrix-core instructions (binary16, or bfloat16 if bf16 == 1) on operands that
 * stay in registers; bf16 == 2: the block-scaled 16x16x128 instruction on fp8 x fp4 operands,
 * bf16 == 3: on fp4 x fp4 operands; bf16 == 4: the 32x32x64 shape of it on fp8 x fp4 operands
 * (four chains).  *flops (HOST) receives the floating-point operations of the
 * launch.  sink: DEVICE, one float, never written in practice. */
int32_t glowq_probe_mfma(int32_t iters, int32_t bf16, int32_t waves_per_simd, float* sink,
                         double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GLOWQ_PROBE_H */
