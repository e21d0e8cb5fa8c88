/*
 * lra_attn_measure.h - machine probes for benchmarks of the Flash-LoRA-Attention library.
 *
 * Not part of the attention path.  Two kernels that show what the GPU at hand gives a plain
 * streaming read and a register-resident bf16 MFMA loop, to be timed by the caller with events
 * around the call, so that a benchmark can hold the library's kernels against the machine's
 * measured ceilings as well as against the published peaks.  (The other measurement aid,
 * lra_tuning.measure_main_kernel_only, is described in lra_attn.h.)
 */
#ifndef LRA_ATTN_MEASURE_H
#define LRA_ATTN_MEASURE_H

#include "lra_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * One kernel reads `bytes` (a multiple of 16 is read; >= 16) from the device buffer src
 * (16-byte aligned) once, coalesced, 16 bytes per lane and request.  Use a buffer larger than
 * the 256 MB memory-side cache, or rotating buffers, for an HBM figure.  sink: 4 writable
 * device bytes (written only for one improbable value of the checksum).
 */
lra_status lra_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * One kernel of two workgroups per CU, every wave issuing iters x 4 independent
 * v_mfma_f32_32x32x16_bf16 on register operands (1 <= iters <= 2^24).  random_operands == 0:
 * two smooth operand values throughout; != 0: four registers of pseudo-random values in
 * rotation, so that consecutive products see unrelated bits as in a real kernel (the clock the
 * chip holds under matrix load depends on the data).  *flops (host, may be NULL) receives the
 * floating-point operations of the launch.  sink: 4 writable device bytes.
 *
 * Both are asynchronous on `stream`; LRA_ERR_NULL / LRA_ERR_SHAPE on bad arguments.
 */
lra_status lra_probe_mfma_bf16(int32_t iters, int32_t random_operands, int64_t* flops, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LRA_ATTN_MEASURE_H */
