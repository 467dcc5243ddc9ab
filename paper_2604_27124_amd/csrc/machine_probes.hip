// Measurement aids, not part of the method and not part of libsigattn: a library of its own that only the
// benchmark and the probe driver load.  Three questions about the machine that the attention kernels'
// design rests on, each answered by a small kernel the caller times with events on its stream:
//
//   mfma   the rate at which the matrix cores run when nothing else competes for the CU (constant operands
//          reach the nominal dense bf16 rate; random operands toggle the datapath and the sustained clock
//          drops under the power limit);
//   atomic the rate of fire-and-forget fp32 global atomic adds in the pattern a fused backward pass would
//          use to accumulate dQ (against plain stores in the same pattern);
//   loop   a model of the dK/dV kernel's inner loop -- per slot one 32x32x16 MFMA, one operand fetch from
//          LDS (row-wise 16-byte reads and pairs of transposing 8-byte reads), the backward's share of
//          VALU and transcendental instructions, a barrier every 32 slots, two waves per SIMD -- from which
//          each of the three components can be left out, to see what each of them costs the loop.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "machine_probes.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------------- mfma

constexpr int MFMA_THREADS = 512;          // 8 waves; two workgroups per CU give 4 waves per SIMD
constexpr int MFMA_BLOCKS = 512;
constexpr int MFMA_PER_ITER = 32;

__global__ void __launch_bounds__(MFMA_THREADS) mfma_kernel(const u32x4 *operands, float *sink, int iters) {
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
    sink[blockIdx.x * MFMA_THREADS + threadIdx.x] = s;
}

// -------------------------------------------------------------------------------------------- atomic

constexpr int ATOMIC_THREADS = 256;        // 4 waves
constexpr int ATOMIC_SLAB_ROWS = 8192;     // one slab = one (z, h) slice of an fp32 dQ: 8192 rows x 64 columns
constexpr int ATOMIC_SLABS = 48;
constexpr size_t ATOMIC_BYTES = (size_t)ATOMIC_SLABS * ATOMIC_SLAB_ROWS * 64 * sizeof(float);

// Every wave walks over [32 rows x 64 columns] tiles of its slab and updates a tile the way a wave would
// flush a transposed 32x32x16 accumulator pair: 32 instructions of 64 lanes x 4 bytes, each covering two
// 128-byte row segments.  All addresses stay inside the slab: tile < rows / 32, row < 32, column < 64.
template <bool ATOMIC>
__global__ void __launch_bounds__(ATOMIC_THREADS) atomic_kernel(float *ws, int iters) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int slab = blockIdx.x % ATOMIC_SLABS;
    float *base = ws + (size_t)slab * ATOMIC_SLAB_ROWS * 64;
    const int c = lane & 31, g = lane >> 5;
    constexpr int NTILES = ATOMIC_SLAB_ROWS / 32;
    int tile = (blockIdx.x / ATOMIC_SLABS * 4 + wave) % NTILES;
    for (int it = 0; it < iters; ++it) {
        tile = (tile + 7) % NTILES;
        float *t = base + (size_t)tile * 32 * 64;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = 8 * (i >> 2) + 4 * g + (i & 3);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float *p = t + row * 64 + 32 * half + c;
                if (ATOMIC) __hip_atomic_fetch_add(p, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else *p = 1.0f;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- loop

constexpr int LOOP_THREADS = 512;          // 8 waves on one CU: two per SIMD, as in the backward kernels
constexpr int LOOP_BLOCKS = 256;
constexpr int LOOP_LDS_BYTES = 80 * 1024;  // more than half a CU's LDS: one workgroup per CU
constexpr int LOOP_SLOTS = 16;             // slots per iteration (= per 32-row block of the dK/dV kernel)
constexpr int LOOP_RING = 8;

#define PROBE_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define PROBE_FMA(i) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(ca), "v"(cb))
#define PROBE_MUL(i) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x[i]) : "v"(ca))
#define PROBE_EXP(i) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]))
#define PROBE_RCP(i) asm volatile("v_rcp_f32 %0, %0" : "+v"(x[i]))
#define PROBE_CVT(i) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x[i]) : "v"(cb))

template <int I, int N, class F>
__device__ __forceinline__ void probe_static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        probe_static_for<I + 1, N>(f);
    }
}

template <bool VALU, bool LDSR, bool MFMA, bool SMALL = false>
__global__ void __launch_bounds__(LOOP_THREADS) loop_kernel(float *sink, int iters, float seed) {
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    // four tiles of 64 rows x 72 elements (the kernels' LDS row stride) plus slack, filled with bf16 values of
    // random sign and significand, so that operands toggle the datapath the way real data does
    for (int i = threadIdx.x; i < 36 * 1024; i += LOOP_THREADS) {
        unsigned h = (unsigned)i * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        lds[i] = (unsigned short)(0x3f00u | (h & 0x80ffu) | ((h >> 9) & 0x0080u));
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5, i16 = lane & 15, g16 = (lane >> 4) & 1;
    const unsigned short *rd = lds + c * 72 + 8 * g;                                   // row-wise operand
    const unsigned short *tr = lds + (4 * g + (i16 >> 2)) * 72 + 16 * g16 + 4 * (i16 & 3);   // transposed operand
    float x[8];
    for (int j = 0; j < 8; ++j) x[j] = seed + threadIdx.x * 1e-3f + j;
    const float ca = 1.0001f + seed * 1e-6f, cb = 0.5f + seed * 1e-6f;
    f32x16 acc[4];
    for (int a = 0; a < 4; ++a)
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
    f32x4 acs[8];                                    // SMALL: two 16x16x32 MFMAs per slot, same FLOPs
    for (int a = 0; a < 8; ++a)
        for (int i = 0; i < 4; ++i) acs[a][i] = 0.f;
    bf16x8 ring[LOOP_RING], b, b2;
    for (int j = 0; j < 8; ++j) {
        unsigned h = (unsigned)(threadIdx.x * 8 + j) * 2654435761u;
        h ^= h >> 15; h *= 2246822519u;
        b[j] = (__bf16)(((int)(h >> 20) - 2048) * (1.0f / 1024.0f) + seed * 1e-3f);
        b2[j] = (__bf16)(((int)((h >> 8) & 4095) - 2048) * (1.0f / 1024.0f) + seed * 1e-3f);
    }
#pragma unroll
    for (int r = 0; r < LOOP_RING; ++r) ring[r] = *reinterpret_cast<const bf16x8 *>(rd + r * 16);
    // slot s of an iteration: s < 8 one 16-byte row-wise read, s >= 8 two transposing 8-byte reads; all inside
    // tile (it & 3): rows < 64, columns < 72
    auto fetch = [&](auto s_, int it) -> bf16x8 {
        constexpr int s = decltype(s_)::value;
        const int tile = (it & 3) * 64 * 72;
        if constexpr (s < 8) {
            return *reinterpret_cast<const bf16x8 *>(rd + tile + ((s & 1) * 32) * 72 + (s >> 1) * 16);
        } else {
            const unsigned short *a = tr + tile + ((s & 1) * 16 + ((s >> 1) & 1) * 32) * 72 + 32 * ((s >> 2) & 1);
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PROBE_LDS_PTR(s16x4, a));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PROBE_LDS_PTR(s16x4, a + 8 * 72));
            s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, r);
        }
    };
    for (int it = 0; it < iters; ++it) {
        probe_static_for<0, LOOP_SLOTS>([&](auto s_) {
            constexpr int s = decltype(s_)::value;
            if constexpr (MFMA && SMALL) {
                acs[(2 * s) & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[s % LOOP_RING], b, acs[(2 * s) & 7], 0, 0, 0);
                acs[(2 * s + 1) & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[s % LOOP_RING], b2, acs[(2 * s + 1) & 7], 0, 0, 0);
            } else if constexpr (MFMA)
                acc[s & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[s % LOOP_RING], b, acc[s & 3], 0, 0, 0);
            else
                asm volatile("" ::"v"(ring[s % LOOP_RING]));      // the operand is still consumed here
            if constexpr (LDSR) ring[(s + LOOP_RING - 1) % LOOP_RING] = fetch(s_, it);
            if constexpr (VALU) {     // per two slots: 2 transcendentals, 2 packs, 8 plain operations
                if constexpr ((s & 1) == 0) {
                    PROBE_EXP(s & 7); PROBE_FMA((s + 2) & 7); PROBE_MUL((s + 3) & 7); PROBE_FMA((s + 4) & 7);
                    PROBE_CVT((s + 5) & 7); PROBE_CVT((s + 6) & 7);
                } else {
                    PROBE_RCP(s & 7); PROBE_FMA((s + 2) & 7); PROBE_MUL((s + 3) & 7); PROBE_FMA((s + 4) & 7);
                    PROBE_FMA((s + 1) & 7); PROBE_MUL((s + 5) & 7);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (it & 1) asm volatile("s_waitcnt lgkmcnt(8)\n\ts_barrier" ::: "memory");
    }
    float s = 0;
    for (int j = 0; j < 8; ++j) s += x[j];
    for (int a = 0; a < 4; ++a)
        for (int i = 0; i < 16; ++i) s += acc[a][i];
    for (int a = 0; a < 8; ++a)
        for (int i = 0; i < 4; ++i) s += acs[a][i];
#pragma unroll
    for (int r = 0; r < LOOP_RING; ++r) s += (float)ring[r][0];
    sink[blockIdx.x * LOOP_THREADS + threadIdx.x] = s;
}

// ---------------------------------------------------------------------------------------------- valu

// The backward's vector work for four score elements -- 4 exp, 4 rcp, 22 plain instructions of which 3 packs --
// in different arrangements of the transcendentals among the plain ones; two waves per SIMD, nothing else.
#define PV_F(i) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(ca), "v"(cb));
#define PV_M(i) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x[i]) : "v"(ca));
#define PV_E(i) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
#define PV_R(i) asm volatile("v_rcp_f32 %0, %0" : "+v"(x[i]));
#define PV_C(i) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x[i]) : "v"(cb));

template <int PAT>
__global__ void __launch_bounds__(LOOP_THREADS) valu_kernel(float *sink, int iters, float seed) {
    float x[32];
    for (int j = 0; j < 32; ++j) x[j] = seed + threadIdx.x * 1e-3f + j * 0.01f;
    const float ca = 0.999f + seed * 1e-6f, cb = 0.5f + seed * 1e-6f;
    for (int it = 0; it < iters; ++it) {
        if constexpr (PAT == 0) {   // as the kernels issue them: per two elements  exp exp | fma fma rcp rcp | muls, packs
            PV_E(0) PV_E(1) PV_F(8) PV_F(9) PV_R(2) PV_R(3) PV_M(10) PV_M(11) PV_M(12) PV_M(13) PV_M(14) PV_M(15) PV_C(16)
            PV_E(4) PV_E(5) PV_F(17) PV_F(18) PV_R(6) PV_R(7) PV_M(19) PV_M(20) PV_M(21) PV_M(22) PV_M(23) PV_M(24) PV_C(25) PV_C(26)
        }
        if constexpr (PAT == 1) {   // all eight transcendentals in one run
            PV_E(0) PV_E(1) PV_E(4) PV_E(5) PV_R(2) PV_R(3) PV_R(6) PV_R(7) PV_F(8) PV_F(9) PV_M(10) PV_M(11) PV_M(12) PV_M(13) PV_M(14)
            PV_M(15) PV_C(16) PV_F(17) PV_F(18) PV_M(19) PV_M(20) PV_M(21) PV_M(22) PV_M(23) PV_M(24) PV_C(25) PV_C(26)
        }
        if constexpr (PAT == 2) {   // single transcendentals, evenly spread
            PV_E(0) PV_F(8) PV_F(9) PV_M(10) PV_E(1) PV_M(11) PV_M(12) PV_M(13) PV_R(2) PV_M(14) PV_M(15) PV_C(16) PV_R(3) PV_F(17) PV_F(18)
            PV_M(19) PV_E(4) PV_M(20) PV_M(21) PV_E(5) PV_M(22) PV_M(23) PV_R(6) PV_M(24) PV_C(25) PV_R(7) PV_C(26)
        }
        if constexpr (PAT == 3) {   // the 22 plain instructions only
            PV_F(8) PV_F(9) PV_M(10) PV_M(11) PV_M(12) PV_M(13) PV_M(14) PV_M(15) PV_C(16) PV_F(17) PV_F(18) PV_M(19) PV_M(20) PV_M(21)
            PV_M(22) PV_M(23) PV_M(24) PV_C(25) PV_C(26) PV_F(27) PV_F(28) PV_F(29)
        }
        if constexpr (PAT == 4) {   // the 8 transcendentals only
            PV_E(0) PV_E(1) PV_E(4) PV_E(5) PV_R(2) PV_R(3) PV_R(6) PV_R(7)
        }
    }
    float s = 0;
    for (int j = 0; j < 32; ++j) s += x[j];
    sink[blockIdx.x * LOOP_THREADS + threadIdx.x] = s;
}

template <int PAT>
int launch_valu(float *sink, int iters, hipStream_t stream) {
    auto kern = valu_kernel<PAT>;      // LDS only to force one workgroup per CU: two waves per SIMD
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LOOP_LDS_BYTES) != hipSuccess)
        return MACHINE_PROBE_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(LOOP_BLOCKS), dim3(LOOP_THREADS), LOOP_LDS_BYTES, stream, sink, iters, 0.5f);
    return hipGetLastError() == hipSuccess ? MACHINE_PROBE_OK : MACHINE_PROBE_ERR_LAUNCH;
}

template <bool VALU, bool LDSR, bool MFMA, bool SMALL = false>
int launch_loop(float *sink, int iters, hipStream_t stream) {
    auto kern = loop_kernel<VALU, LDSR, MFMA, SMALL>;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LOOP_LDS_BYTES) != hipSuccess)
        return MACHINE_PROBE_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(LOOP_BLOCKS), dim3(LOOP_THREADS), LOOP_LDS_BYTES, stream, sink, iters, 0.5f);
    return hipGetLastError() == hipSuccess ? MACHINE_PROBE_OK : MACHINE_PROBE_ERR_LAUNCH;
}

}  // namespace

extern "C" {

size_t machine_probe_mfma_operand_bytes(void) { return (size_t)MFMA_THREADS * 16 * 16; }
size_t machine_probe_sink_bytes(void) { return (size_t)MFMA_BLOCKS * MFMA_THREADS * sizeof(float); }

double machine_probe_mfma_flops(int iters) {
    return iters <= 0 ? 0.0
                      : (double)MFMA_BLOCKS * (MFMA_THREADS / 64) * (double)iters * MFMA_PER_ITER * (2.0 * 32 * 32 * 16);
}

int machine_probe_mfma(const void *operands, void *sink, int iters, void *stream) {
    if (!operands || !sink || iters <= 0) return MACHINE_PROBE_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return MACHINE_PROBE_ERR_MISALIGNED;
    hipLaunchKernelGGL(mfma_kernel, dim3(MFMA_BLOCKS), dim3(MFMA_THREADS), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(operands), static_cast<float *>(sink), iters);
    return hipGetLastError() == hipSuccess ? MACHINE_PROBE_OK : MACHINE_PROBE_ERR_LAUNCH;
}

size_t machine_probe_atomic_bytes(void) { return ATOMIC_BYTES; }

double machine_probe_atomic_updates(int blocks, int iters) {
    return (blocks <= 0 || iters <= 0) ? 0.0 : (double)blocks * (ATOMIC_THREADS / 64) * (double)iters * 32.0 * 64.0;
}

int machine_probe_atomic(void *buffer, size_t bytes, int atomic, int blocks, int iters, void *stream) {
    if (!buffer || bytes < ATOMIC_BYTES || blocks <= 0 || blocks > 65536 || iters <= 0) return MACHINE_PROBE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(buffer) & 3u) return MACHINE_PROBE_ERR_MISALIGNED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (atomic) hipLaunchKernelGGL(atomic_kernel<true>, dim3(blocks), dim3(ATOMIC_THREADS), 0, s, static_cast<float *>(buffer), iters);
    else hipLaunchKernelGGL(atomic_kernel<false>, dim3(blocks), dim3(ATOMIC_THREADS), 0, s, static_cast<float *>(buffer), iters);
    return hipGetLastError() == hipSuccess ? MACHINE_PROBE_OK : MACHINE_PROBE_ERR_LAUNCH;
}

double machine_probe_loop_wave_slots_per_simd(int iters) {
    // every SIMD of the 256 CUs hosts two waves, each running iters x 16 slots
    return iters <= 0 ? 0.0 : (double)iters * LOOP_SLOTS * 2.0;
}

int machine_probe_valu(void *sink, int iters, int arrangement, void *stream) {
    if (!sink || iters <= 0 || arrangement < 0 || arrangement > 4) return MACHINE_PROBE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(sink) & 3u) return MACHINE_PROBE_ERR_MISALIGNED;
    float *out = static_cast<float *>(sink);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (arrangement) {
        case 0: return launch_valu<0>(out, iters, s);
        case 1: return launch_valu<1>(out, iters, s);
        case 2: return launch_valu<2>(out, iters, s);
        case 3: return launch_valu<3>(out, iters, s);
        default: return launch_valu<4>(out, iters, s);
    }
}

int machine_probe_loop(void *sink, int iters, int components, void *stream) {
    if (!sink || iters <= 0 || components < 0 || components > 8) return MACHINE_PROBE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(sink) & 3u) return MACHINE_PROBE_ERR_MISALIGNED;
    float *out = static_cast<float *>(sink);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (components) {      // bit 0: VALU, bit 1: LDS reads, bit 2: MFMA; 8: all three with two 16x16x32 MFMAs per slot
        case 8: return launch_loop<true, true, true, true>(out, iters, s);
        case 0: return launch_loop<false, false, false>(out, iters, s);
        case 1: return launch_loop<true, false, false>(out, iters, s);
        case 2: return launch_loop<false, true, false>(out, iters, s);
        case 3: return launch_loop<true, true, false>(out, iters, s);
        case 4: return launch_loop<false, false, true>(out, iters, s);
        case 5: return launch_loop<true, false, true>(out, iters, s);
        case 6: return launch_loop<false, true, true>(out, iters, s);
        default: return launch_loop<true, true, true>(out, iters, s);
    }
}

}  // extern "C"
