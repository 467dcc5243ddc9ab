/*
 * mfma_probe.h -- C ABI of libmfma_probe, a measurement aid that only the benchmark loads: the
 * matrix-core ceiling of the machine, reported next to the attention kernels.  Not part of the method.
 *
 * mfma_probe_launch enqueues 512 workgroups of 512 threads in which every wave issues `iters` x 32
 * independent 32x32x16 bf16 MFMAs on caller-supplied operands (constant operands reach the nominal rate;
 * random ones expose the power-limited sustained rate).
 *   operands : in,  device, mfma_probe_operand_bytes() bytes of bf16 data, 16-byte aligned
 *   sink     : out, device, mfma_probe_sink_bytes() bytes (keeps the work alive; content unspecified)
 *   stream   : a hipStream_t passed as void*
 * mfma_probe_flops(iters) is the number of floating-point operations one launch performs.  The caller
 * times the launch (events on `stream`).  Returns 0 or a negative MFMA_PROBE_ERR_* code; arguments are
 * checked on the host before any HIP call.
 */
#ifndef MFMA_PROBE_H
#define MFMA_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MFMA_PROBE_OK 0
#define MFMA_PROBE_ERR_INVALID_ARG (-1)
#define MFMA_PROBE_ERR_MISALIGNED (-3)
#define MFMA_PROBE_ERR_LAUNCH (-5)

size_t mfma_probe_operand_bytes(void);
size_t mfma_probe_sink_bytes(void);
double mfma_probe_flops(int iters);
int mfma_probe_launch(const void *operands, void *sink, int iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MFMA_PROBE_H */
