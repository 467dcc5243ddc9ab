// Measurement aid, not part of the method and not part of libsigattn: a library of its own that only the
// benchmark loads.  The rate at which the matrix cores run when nothing else competes for the CU.  Every wave
// issues independent v_mfma_f32_32x32x16_bf16 back to back on operands the caller supplies.  With
// constant operands the chip reaches its nominal dense bf16 rate; with random operands the datapath
// toggles and the sustained clock drops under the power limit.  bench.py reports both next to the
// attention kernels, as the ceiling any bf16 contraction on this machine lives under.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 512;          // 8 waves; two workgroups per CU give 4 waves per SIMD
constexpr int PROBE_BLOCKS = 512;
constexpr int PROBE_MFMA_PER_ITER = 32;

__global__ void __launch_bounds__(PROBE_THREADS) probe_kernel(const u32x4 *operands, float *sink, int iters) {
    bf16x8 a[8], b[8];   // 16 operands of 16 bytes per lane
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, operands[threadIdx.x * 16 + i]);
        b[i] = __builtin_bit_cast(bf16x8, operands[threadIdx.x * 16 + 8 + i]);
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + 1) & 7], b[i], c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[(i + 3) & 7], c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + 5) & 7], b[(i + 2) & 7], c3, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    sink[blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

extern "C" {

size_t mfma_probe_operand_bytes(void) { return (size_t)PROBE_THREADS * 16 * 16; }
size_t mfma_probe_sink_bytes(void) { return (size_t)PROBE_BLOCKS * PROBE_THREADS * sizeof(float); }

double mfma_probe_flops(int iters) {
    return iters <= 0 ? 0.0
                      : (double)PROBE_BLOCKS * (PROBE_THREADS / 64) * (double)iters * PROBE_MFMA_PER_ITER * (2.0 * 32 * 32 * 16);
}

int mfma_probe_launch(const void *operands, void *sink, int iters, void *stream) {
    if (!operands || !sink || iters <= 0) return MFMA_PROBE_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return MFMA_PROBE_ERR_MISALIGNED;
    hipLaunchKernelGGL(probe_kernel, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(operands), static_cast<float *>(sink), iters);
    return hipGetLastError() == hipSuccess ? MFMA_PROBE_OK : MFMA_PROBE_ERR_LAUNCH;
}

}  // extern "C"
