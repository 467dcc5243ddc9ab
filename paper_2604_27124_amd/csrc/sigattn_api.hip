// Host side of libsigattn: argument validation, kernel selection and launch behind the C ABI
// declared in include/sigmoid_attn.h.  Validation happens before any HIP call.
#include "sigattn_kernels.hpp"
#include "sigmoid_attn.h"

#include <cmath>
#include <mutex>

using namespace sigattn;

// Scratch of the entry point that allocates nothing: one array per GPU the library runs on, held until the
// process ends.  In host code this name is only a stand-in; the array's device address comes from
// hipGetSymbolAddress, once per device (static_scratch() below), and only that pointer is ever handed on.
static __device__ __align__(256) unsigned char scratch[SIGATTN_STATIC_SCRATCH_BYTES];

namespace {

int check_shape(int B, int N, int H, int d) {
    if (B <= 0 || N <= 0 || H <= 0) return SIGATTN_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return SIGATTN_ERR_UNSUPPORTED_D;
    if ((long long)B * H > 2147483647LL) return SIGATTN_ERR_TOO_LARGE;     // grid.x limit
    if ((long long)B * N * H * d >= (1LL << 40)) return SIGATTN_ERR_TOO_LARGE;
    if ((long long)H * d > (1LL << 20)) return SIGATTN_ERR_TOO_LARGE;      // 32-bit lane offsets within one streamed tile
    if (B > MAP_MAX_B && (long long)N > 256LL * MAP_CLASSES) return SIGATTN_ERR_TOO_LARGE;   // tile-count classes of the work mapping
    return SIGATTN_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int MODE, int D, int QB, int NW, int BN, int LD1, int LD2, int OCC, int RING, bool WITH_DB = false>
int launch(const Params &p, hipStream_t stream) {
    using C = Cfg<MODE, D, QB, NW, BN, LD1, LD2, RING>;
    const long long tiles = ((long long)p.N + C::BM - 1) / C::BM;
    const long long wgs = tiles * p.B * p.H;                                // one workgroup per owner tile
    if (wgs > 2147483647LL) return SIGATTN_ERR_TOO_LARGE;
    dim3 grid((unsigned)wgs, 1, 1);
    dim3 block(C::THREADS, 1, 1);
    auto kern = sigattn_kernel<MODE, D, QB, NW, BN, LD1, LD2, OCC, RING, WITH_DB>;
    if (C::LDS_BYTES > 65536) {   // more dynamic LDS than the default limit: opt in (idempotent, host-side only)
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)C::LDS_BYTES) != hipSuccess)
            return SIGATTN_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(kern, grid, block, C::LDS_BYTES, stream, p);
    return hipGetLastError() == hipSuccess ? SIGATTN_OK : SIGATTN_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int sigmoid_attn_version(void) { return 300; }

const char *sigmoid_attn_strerror(int code) {
    switch (code) {
        case SIGATTN_OK: return "success";
        case SIGATTN_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive dimension or non-finite scale)";
        case SIGATTN_ERR_UNSUPPORTED_D: return "unsupported head dimension (must be 64 or 128)";
        case SIGATTN_ERR_MISALIGNED: return "tensor pointer is not 16-byte aligned";
        case SIGATTN_ERR_WORKSPACE: return "workspace missing or too small";
        case SIGATTN_ERR_LAUNCH: return "HIP kernel launch failed";
        case SIGATTN_ERR_TOO_LARGE: return "problem too large: more workgroups than one launch holds, H*d > 2^20, more than 256 sequences padded beyond 262144 rows, or more query tiles than the static scratch array holds";
        default: return "unknown error code";
    }
}

size_t sigmoid_attn_bwd_workspace_bytes(int B, int N_max, int H, int d) {
    if (check_shape(B, N_max, H, d) != SIGATTN_OK) return 0;
    return 0;   // the backward pass owns each output tile exclusively: no scratch, no atomics
}

// ---- common implementations: separate query-side and key-side lengths (self-attention passes them twice)

static int fwd_impl(const void *q, const void *k, const void *v, void *o,
                    const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                    int B, int L_q, int L_k, int H, int d, void *stream) {
    if (!q || !k || !v || !o || !seqlens_q || !seqlens_k || !bias || !std::isfinite(scale)) return SIGATTN_ERR_INVALID_ARG;
    if (int e = check_shape(B, L_q, H, d)) return e;
    if (int e = check_shape(B, L_k, H, d)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return SIGATTN_ERR_MISALIGNED;

    Params p{};
    p.q = static_cast<const bf16_t *>(q);
    p.k = static_cast<const bf16_t *>(k);
    p.v = static_cast<const bf16_t *>(v);
    p.d_o = nullptr;
    p.out0 = static_cast<bf16_t *>(o);
    p.out1 = nullptr;
    p.seqlens = seqlens_q;          // owner side: queries
    p.seqlens_str = seqlens_k;      // streamed side: keys / values
    p.bias = bias;
    p.scale = scale;
    p.B = B; p.N = L_q; p.N_str = L_k; p.H = H;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d == 64) {
        // 512-row owner tiles (two owner blocks per wave) feed two MFMAs from every LDS operand read and win
        // on long sequences; 256-row tiles need half the registers, so two workgroups share a CU, and they
        // halve the granularity of the grid: measured better up to 4096 streamed rows unless the grid of
        // 512-row tiles still fills the chip four times over (the host sees the padded lengths only).
        const long long wgs512 = (long long)B * H * ((L_q + 511) / 512);
        if (L_k > 4096 || (L_k >= 2048 && wgs512 >= 1024)) return launch<FWD, 64, 2, 8, 64, 72, 72, 1, 4>(p, s);
        return launch<FWD, 64, 1, 8, 64, 72, 72, 4, 4>(p, s);
    }
    // d = 128: K is only read row-wise (272-byte rows), V only through the transposing reads, which at that
    // stride ran at a quarter of their rate; 288-byte rows with the split column layout are conflict-free.
    return launch<FWD, 128, 1, 8, 64, 136, 144, 1, 4>(p, s);
}

static int bwd_impl(const void *q, const void *k, const void *v, const void *d_o,
                    void *dq, void *dk, void *dv,
                    const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                    int B, int L_q, int L_k, int H, int d, void *stream, bool want_dq, bool want_dkdv) {
    if (!q || !k || !v || !d_o || !seqlens_q || !seqlens_k || !bias || !std::isfinite(scale)) return SIGATTN_ERR_INVALID_ARG;
    if ((want_dq && !dq) || (want_dkdv && (!dk || !dv))) return SIGATTN_ERR_INVALID_ARG;
    if (int e = check_shape(B, L_q, H, d)) return e;
    if (int e = check_shape(B, L_k, H, d)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o)) return SIGATTN_ERR_MISALIGNED;
    if ((want_dq && !aligned16(dq)) || (want_dkdv && (!aligned16(dk) || !aligned16(dv))))
        return SIGATTN_ERR_MISALIGNED;

    Params p{};
    p.q = static_cast<const bf16_t *>(q);
    p.k = static_cast<const bf16_t *>(k);
    p.v = static_cast<const bf16_t *>(v);
    p.d_o = static_cast<const bf16_t *>(d_o);
    p.bias = bias;
    p.scale = scale;
    p.B = B; p.H = H;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (want_dkdv) {         // Alg. 3: dK, dV (owner = key tile, streamed = queries and dO)
        Params pk = p;
        pk.seqlens = seqlens_k; pk.N = L_k;
        pk.seqlens_str = seqlens_q; pk.N_str = L_q;
        pk.out0 = static_cast<bf16_t *>(dk);
        pk.out1 = static_cast<bf16_t *>(dv);
        // d = 64: eight waves of 32 keys at two waves per SIMD.  d = 128: the fp32 accumulators of dK and dV
        // (128 registers) fit only with the whole register file of a SIMD for one wave, so four waves of 32
        // keys, one per SIMD (both streamed tensors are read row-wise and transposed: 288-byte LDS rows).
        const int e = (d == 64) ? launch<DKDV, 64, 1, 8, 64, 72, 72, 1, 8>(pk, s)
                                : launch<DKDV, 128, 1, 4, 64, 144, 144, 1, 4>(pk, s);
        if (e) return e;
    }
    if (want_dq) {           // Alg. 2: dQ (owner = query tile, streamed = keys and values)
        Params pq = p;
        pq.seqlens = seqlens_q; pq.N = L_q;
        pq.seqlens_str = seqlens_k; pq.N_str = L_k;
        pq.out0 = static_cast<bf16_t *>(dq);
        pq.out1 = nullptr;
        const int e = (d == 64) ? launch<DQ, 64, 1, 8, 64, 72, 72, 1, 4>(pq, s)
                                : launch<DQ, 128, 1, 8, 64, 144, 136, 1, 4>(pq, s);
        if (e) return e;
    }
    return SIGATTN_OK;
}

int sigmoid_attn_fwd(const void *q, const void *k, const void *v, void *o,
                     const int32_t *seqlens, const float *bias, float scale,
                     int B, int N_max, int H, int d, void *stream) {
    return fwd_impl(q, k, v, o, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d, stream);
}

int sigmoid_attn_bwd(const void *q, const void *k, const void *v, const void *d_o,
                     void *dq, void *dk, void *dv,
                     const int32_t *seqlens, const float *bias, float scale,
                     int B, int N_max, int H, int d,
                     void *workspace, size_t workspace_bytes, void *stream) {
    if (!dq || !dk || !dv) return SIGATTN_ERR_INVALID_ARG;
    const int e0 = bwd_impl(q, k, v, d_o, dq, dk, dv, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d, nullptr, false, false);
    if (e0) return e0;       // argument errors first, as the header orders them
    const size_t need = sigmoid_attn_bwd_workspace_bytes(B, N_max, H, d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return SIGATTN_ERR_WORKSPACE;
    return bwd_impl(q, k, v, d_o, dq, dk, dv, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d, stream, true, true);
}

int sigmoid_attn_bwd_dq(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                        const int32_t *seqlens, const float *bias, float scale,
                        int B, int N_max, int H, int d, void *stream) {
    return bwd_impl(q, k, v, d_o, dq, nullptr, nullptr, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d, stream, true, false);
}

int sigmoid_attn_bwd_dkdv(const void *q, const void *k, const void *v, const void *d_o, void *dk, void *dv,
                          const int32_t *seqlens, const float *bias, float scale,
                          int B, int N_max, int H, int d, void *stream) {
    return bwd_impl(q, k, v, d_o, nullptr, dk, dv, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d, stream, false, true);
}

// dQ workgroups own 256 query rows at either head dimension: one partial per workgroup.
static long long dq_workgroups(int B, int N, int H) { return (((long long)N + 255) / 256) * B * H; }

size_t sigmoid_attn_bwd_dq_dbias_workspace_bytes(int B, int N_max, int H, int d) {
    if (check_shape(B, N_max, H, d) != SIGATTN_OK) return 0;
    return (size_t)dq_workgroups(B, N_max, H) * (sizeof(float) + sizeof(int32_t));
}

size_t sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(int B, int L_q, int L_k, int H, int d) {
    if (check_shape(B, L_k, H, d) != SIGATTN_OK) return 0;
    return sigmoid_attn_bwd_dq_dbias_workspace_bytes(B, L_q, H, d);     // one partial per 256-row query tile
}

static int dq_dbias_impl(const void *q, const void *k, const void *v, const void *d_o, void *dq, float *dbias,
                         const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                         int B, int L_q, int L_k, int H, int d,
                         void *workspace, size_t workspace_bytes, void *stream) {
    if (!q || !k || !v || !d_o || !dq || !dbias || !seqlens_q || !seqlens_k || !bias || !std::isfinite(scale))
        return SIGATTN_ERR_INVALID_ARG;
    if (int e = check_shape(B, L_q, H, d)) return e;
    if (int e = check_shape(B, L_k, H, d)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq)) return SIGATTN_ERR_MISALIGNED;
    const size_t need = sigmoid_attn_bwd_dq_dbias_workspace_bytes(B, L_q, H, d);
    if (!workspace || workspace_bytes < need) return SIGATTN_ERR_WORKSPACE;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(dbias) & 3u)) return SIGATTN_ERR_MISALIGNED;

    const long long nwg = dq_workgroups(B, L_q, H);
    Params p{};
    p.q = static_cast<const bf16_t *>(q);
    p.k = static_cast<const bf16_t *>(k);
    p.v = static_cast<const bf16_t *>(v);
    p.d_o = static_cast<const bf16_t *>(d_o);
    p.out0 = static_cast<bf16_t *>(dq);
    p.seqlens = seqlens_q;          // owner side: queries
    p.seqlens_str = seqlens_k;      // streamed side: keys / values
    p.bias = bias;
    p.scale = scale;
    p.B = B; p.N = L_q; p.N_str = L_k; p.H = H;
    p.db_part = static_cast<float *>(workspace);
    p.db_seq = reinterpret_cast<int32_t *>(p.db_part + nwg);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int e = (d == 64) ? launch<DQ, 64, 1, 8, 64, 72, 72, 1, 4, true>(p, s)
                            : launch<DQ, 128, 1, 8, 64, 144, 136, 1, 2, true>(p, s);
    if (e) return e;
    hipLaunchKernelGGL(sigattn_db_reduce, dim3((unsigned)B), dim3(256), 0, s, p.db_part, p.db_seq, (int)nwg, dbias);
    return hipGetLastError() == hipSuccess ? SIGATTN_OK : SIGATTN_ERR_LAUNCH;
}

int sigmoid_attn_bwd_dq_dbias(const void *q, const void *k, const void *v, const void *d_o, void *dq, float *dbias,
                              const int32_t *seqlens, const float *bias, float scale,
                              int B, int N_max, int H, int d,
                              void *workspace, size_t workspace_bytes, void *stream) {
    return dq_dbias_impl(q, k, v, d_o, dq, dbias, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d,
                         workspace, workspace_bytes, stream);
}

// Device address of this GPU's copy of `scratch`: looked up on the first call on each device, with that
// device current, and kept.  Every GPU holds its own copy of the array at its own address.
static void *static_scratch() {
    constexpr int MAX_DEVICES = 64;
    static std::mutex lock;
    static void *ptr[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> hold(lock);
    if (!ptr[dev]) {
        void *a = nullptr;
        if (hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)) != hipSuccess || !a) return nullptr;
        ptr[dev] = a;
    }
    return ptr[dev];
}

int sigmoid_attn_bwd_dq_dbias_static(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                                     float *dbias, const int32_t *seqlens, const float *bias, float scale,
                                     int B, int N_max, int H, int d, void *stream) {
    // Argument errors first, on the host, exactly as the workspace form reports them (a non-null, aligned
    // stand-in of sufficient size takes the place of the workspace for that pass; nothing is launched).
    if (!q || !k || !v || !d_o || !dq || !dbias || !seqlens || !bias || !std::isfinite(scale)) return SIGATTN_ERR_INVALID_ARG;
    if (int e = check_shape(B, N_max, H, d)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) ||
        (reinterpret_cast<uintptr_t>(dbias) & 3u))
        return SIGATTN_ERR_MISALIGNED;
    const size_t need = sigmoid_attn_bwd_dq_dbias_workspace_bytes(B, N_max, H, d);
    if (need > (size_t)SIGATTN_STATIC_SCRATCH_BYTES) return SIGATTN_ERR_TOO_LARGE;   // more query tiles than the array holds
    void *ws = static_scratch();
    if (!ws) return SIGATTN_ERR_LAUNCH;
    // Every workgroup writes its own partial and the second kernel reads exactly those: nothing has to start at zero.
    return dq_dbias_impl(q, k, v, d_o, dq, dbias, seqlens, seqlens, bias, scale, B, N_max, N_max, H, d,
                         ws, (size_t)SIGATTN_STATIC_SCRATCH_BYTES, stream);
}

int sigmoid_attn_cross_bwd_dq_dbias(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                                    float *dbias, const int32_t *seqlens_q, const int32_t *seqlens_k,
                                    const float *bias, float scale, int B, int L_q, int L_k, int H, int d,
                                    void *workspace, size_t workspace_bytes, void *stream) {
    return dq_dbias_impl(q, k, v, d_o, dq, dbias, seqlens_q, seqlens_k, bias, scale, B, L_q, L_k, H, d,
                         workspace, workspace_bytes, stream);
}

int sigmoid_attn_cross_fwd(const void *q, const void *k, const void *v, void *o,
                           const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                           int B, int L_q, int L_k, int H, int d, void *stream) {
    return fwd_impl(q, k, v, o, seqlens_q, seqlens_k, bias, scale, B, L_q, L_k, H, d, stream);
}

int sigmoid_attn_cross_bwd(const void *q, const void *k, const void *v, const void *d_o,
                           void *dq, void *dk, void *dv,
                           const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                           int B, int L_q, int L_k, int H, int d, void *stream) {
    if (!dq || !dk || !dv) return SIGATTN_ERR_INVALID_ARG;
    return bwd_impl(q, k, v, d_o, dq, dk, dv, seqlens_q, seqlens_k, bias, scale, B, L_q, L_k, H, d, stream, true, true);
}

}  // extern "C"
