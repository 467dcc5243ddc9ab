/*
 * machine_probes.h -- C ABI of libmachine_probes, measurement aids that only the benchmark and the probe
 * driver load.  Not part of the method, not part of libsigattn.  Every probe only enqueues one kernel on
 * `stream` (a hipStream_t passed as void*); the caller times it with events on that stream.  Return
 * value: 0 or a negative MACHINE_PROBE_ERR_* code; arguments are checked on the host before any HIP call.
 * All buffers are DEVICE memory owned by the caller.
 *
 * mfma:   512 workgroups of 512 threads, every wave issues iters x 32 independent 32x32x16 bf16 MFMAs on
 *         caller-supplied operands (constant operands reach the nominal rate, random ones the power-limited
 *         sustained rate).  operands: machine_probe_mfma_operand_bytes() bytes of bf16, 16-byte aligned;
 *         sink: machine_probe_sink_bytes() bytes, written (content unspecified).
 *         machine_probe_mfma_flops(iters) = floating-point operations of one launch.
 * atomic: `blocks` workgroups of 4 waves add 1.0f (atomic != 0: fp32 atomic add, no return value; atomic == 0:
 *         plain store) to [32 x 64] tiles of 48 slabs of 8192 x 64 floats, the pattern in which a fused
 *         backward pass would flush partial dQ tiles.  buffer: at least machine_probe_atomic_bytes() bytes.
 *         machine_probe_atomic_updates(blocks, iters) = 4-byte updates of one launch.
 * loop:   a model of the dK/dV kernel's inner loop on 256 workgroups of 8 waves (two per SIMD): per slot one
 *         MFMA (bit 2 of `components`), one operand fetch from LDS (bit 1) and six VALU instructions of the
 *         backward's mix (bit 0); a barrier every 32 slots.  components = 8: all three, with two 16x16x32
 *         MFMAs per slot in place of the one 32x32x16 (same FLOPs).  sink as for mfma.
 *         machine_probe_loop_wave_slots_per_simd(iters) = wave-slots each SIMD executes in one launch.
 * valu:   the backward's vector work for four score elements per iteration (4 exp, 4 rcp, 22 plain instructions)
 *         on two waves per SIMD, nothing else: arrangement 0 = as the kernels issue them, 1 = all transcendentals
 *         in one run, 2 = single transcendentals evenly spread, 3 = the plain instructions only, 4 = the
 *         transcendentals only.  sink as for mfma.
 */
#ifndef MACHINE_PROBES_H
#define MACHINE_PROBES_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MACHINE_PROBE_OK 0
#define MACHINE_PROBE_ERR_INVALID_ARG (-1)
#define MACHINE_PROBE_ERR_MISALIGNED (-3)
#define MACHINE_PROBE_ERR_LAUNCH (-5)

size_t machine_probe_mfma_operand_bytes(void);
size_t machine_probe_sink_bytes(void);
double machine_probe_mfma_flops(int iters);
int machine_probe_mfma(const void *operands, void *sink, int iters, void *stream);

size_t machine_probe_atomic_bytes(void);
double machine_probe_atomic_updates(int blocks, int iters);
int machine_probe_atomic(void *buffer, size_t bytes, int atomic, int blocks, int iters, void *stream);

double machine_probe_loop_wave_slots_per_simd(int iters);
int machine_probe_loop(void *sink, int iters, int components, void *stream);
int machine_probe_valu(void *sink, int iters, int arrangement, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MACHINE_PROBES_H */
