/*
 * sigmoid_attn.h -- C ABI of libsigattn: padded bidirectional sigmoid attention on MI355X (gfx950).
 *
 * Operation (paper Sec. 3, the sigmoid-attention equation; appendix Alg. 1 for the padding rules):
 *
 *     O[z,i,h,:] = sum_{j < n_z} sigma(scale * <Q[z,i,h,:], K[z,j,h,:]> + bias[z]) * V[z,j,h,:]   for i < n_z
 *     O[z,i,h,:] = 0                                                                            for i >= n_z
 *
 * with sigma(a) = 1 / (1 + exp(-a)) applied element-wise, no row normalisation, and n_z = seqlens[z]
 * the number of valid (non-padded) tokens of sequence z, which occupy rows [0, n_z) (right padding).
 * The paper's default bias is b = -log(n); the library takes bias[z] as data.
 *
 * Backward (appendix Alg. 2 and Alg. 3; the Jacobian of sigma is diagonal, so no row statistics and no
 * saved forward state are needed -- scores are recomputed):
 *
 *     dP_ij = <dO_i, V_j>,   dS_ij = P_ij (1 - P_ij) dP_ij
 *     dV_j = sum_i P_ij dO_i,   dK_j = scale * sum_i dS_ij Q_i,   dQ_i = scale * sum_j dS_ij K_j
 *
 * over valid i, j only; padded rows of dQ, dK, dV are written as zero.  1 - P is formed without
 * cancellation (as exp(-x) P), so dS keeps its relative accuracy on both saturated tails of sigma,
 * for every score and bias whose exponentials fp32 can hold (|bias| up to about 80).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All tensor pointers are DEVICE pointers to bf16 data, contiguous [B, N_max, H, d] with d fastest,
 *    16-byte aligned, owned by the caller.  d must be 64 or 128.
 *  - seqlens: DEVICE pointer, int32[B].  Values outside [0, N_max] are clamped inside the kernels.
 *  - bias:    DEVICE pointer, float[B].
 *  - stream:  a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work and
 *    return without synchronising; they are stream-ordered with the caller's other work.
 *  - Outputs are fully overwritten (padded rows with exact zeros); inputs are never modified; values
 *    held by padded input rows never influence a valid output as long as they are finite.
 *  - The library allocates nothing and keeps no state between calls.
 *  - Return value: SIGATTN_OK (0) or a negative SIGATTN_ERR_* code.  Arguments are validated on the
 *    host before any HIP call is made, so every error except SIGATTN_ERR_LAUNCH can be observed on a
 *    machine without a GPU.  On error nothing has been enqueued.
 */
#ifndef SIGMOID_ATTN_H
#define SIGMOID_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIGATTN_OK 0
#define SIGATTN_ERR_INVALID_ARG (-1)      /* null pointer, non-positive B / N_max / H, non-finite scale   */
#define SIGATTN_ERR_UNSUPPORTED_D (-2)    /* head dimension other than 64 or 128                           */
#define SIGATTN_ERR_MISALIGNED (-3)       /* a tensor pointer is not 16-byte aligned                       */
#define SIGATTN_ERR_WORKSPACE (-4)        /* workspace missing or smaller than ..._workspace_bytes()      */
#define SIGATTN_ERR_LAUNCH (-5)           /* the HIP runtime refused a launch (see hipGetLastError)       */
#define SIGATTN_ERR_TOO_LARGE (-6)        /* B*H or the tile count exceeds one grid, H*d > 2^20, or more  */
                                          /* than 256 sequences padded to more than 262144 rows            */

/* Library version: major * 10000 + minor * 100 + patch. */
int sigmoid_attn_version(void);

/* Static, human-readable text for a return code (never NULL). */
const char *sigmoid_attn_strerror(int code);

/*
 * Forward pass (Sec. 3 equation; Alg. 1).
 *   q, k, v : in,  device bf16 [B, N_max, H, d]
 *   o       : out, device bf16 [B, N_max, H, d]; rows >= seqlens[z] are written as 0
 *   seqlens : in,  device int32 [B]          bias : in, device float [B]
 *   scale   : the factor on Q K^T (the paper uses 1/sqrt(d))
 */
int sigmoid_attn_fwd(const void *q, const void *k, const void *v, void *o,
                     const int32_t *seqlens, const float *bias, float scale,
                     int B, int N_max, int H, int d, void *stream);

/*
 * Backward pass (Alg. 2: dQ; Alg. 3: dK, dV).  Needs only the forward inputs and dO.
 *   q, k, v, d_o : in,  device bf16 [B, N_max, H, d]  (rows >= seqlens[z] of d_o are ignored)
 *   dq, dk, dv   : out, device bf16 [B, N_max, H, d]; padded rows are written as 0
 *   workspace    : device scratch of at least sigmoid_attn_bwd_workspace_bytes(...) bytes, owned by
 *                  the caller, contents irrelevant on entry and undefined on exit.  That size is 0 for
 *                  every shape (each kernel owns its output tiles), so NULL / 0 is accepted.
 */
int sigmoid_attn_bwd(const void *q, const void *k, const void *v, const void *d_o,
                     void *dq, void *dk, void *dv,
                     const int32_t *seqlens, const float *bias, float scale,
                     int B, int N_max, int H, int d,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two halves of the backward pass on their own, as the paper states them: Alg. 2 (dQ only) and
 * Alg. 3 (dK and dV only).  Arguments as for sigmoid_attn_bwd; neither needs a workspace.
 * sigmoid_attn_bwd is equivalent to calling both on one stream.
 */
int sigmoid_attn_bwd_dq(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                        const int32_t *seqlens, const float *bias, float scale,
                        int B, int N_max, int H, int d, void *stream);
int sigmoid_attn_bwd_dkdv(const void *q, const void *k, const void *v, const void *d_o, void *dk, void *dv,
                          const int32_t *seqlens, const float *bias, float scale,
                          int B, int N_max, int H, int d, void *stream);

/*
 * Separate query and key lengths (appendix Alg. 1-3 are printed with L_q, L_k and n_q, n_k of their own).
 *   q, o, d_o, dq : device bf16 [B, L_q, H, d]        k, v, dk, dv : device bf16 [B, L_k, H, d]
 *   seqlens_q, seqlens_k : device int32 [B]; valid queries are rows [0, seqlens_q[z]), valid keys rows
 *                          [0, seqlens_k[z]); values outside [0, L] are clamped inside the kernels
 *   O_i = sum_{j < n_k} sigma(scale <q_i, k_j> + bias[z]) v_j for i < n_q, else 0 (also 0 when n_k = 0);
 *   dQ over j < n_k; dK, dV over i < n_q; padded rows of every output are written as 0.
 * Everything else (layout, ownership, stream, errors) as for the self-attention entry points, which
 * are these with L_q = L_k and seqlens_q = seqlens_k.  No workspace is needed.
 */
int sigmoid_attn_cross_fwd(const void *q, const void *k, const void *v, void *o,
                           const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                           int B, int L_q, int L_k, int H, int d, void *stream);
int sigmoid_attn_cross_bwd(const void *q, const void *k, const void *v, const void *d_o,
                           void *dq, void *dk, void *dv,
                           const int32_t *seqlens_q, const int32_t *seqlens_k, const float *bias, float scale,
                           int B, int L_q, int L_k, int H, int d, void *stream);

/*
 * dQ together with the gradient of the bias (Sec. 3 allows a learnable b; x_ij = scale s_ij + b_z, hence
 * db_z = sum over heads and valid pairs of dS_ij).  The sum rides on the dQ kernel (Alg. 2).
 *   dq        : out, device bf16 [B, N_max, H, d] as for sigmoid_attn_bwd_dq
 *   dbias     : out, device float [B]; fully overwritten (0 for an empty sequence)
 *   workspace : device scratch of at least sigmoid_attn_bwd_dq_dbias_workspace_bytes(...) bytes, 16-byte
 *               aligned, owned by the caller; contents irrelevant on entry, undefined on exit
 * The summation order is fixed: results are bitwise reproducible.  nwg = B * H * ceil(N_max / 256)
 * must be below 2^31 (SIGATTN_ERR_TOO_LARGE).
 */
size_t sigmoid_attn_bwd_dq_dbias_workspace_bytes(int B, int N_max, int H, int d);
int sigmoid_attn_bwd_dq_dbias(const void *q, const void *k, const void *v, const void *d_o, void *dq, float *dbias,
                              const int32_t *seqlens, const float *bias, float scale,
                              int B, int N_max, int H, int d,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same with separate query and key lengths (layouts and lengths as for sigmoid_attn_cross_bwd):
 * db_z sums dS_ij over heads, i < n_q and j < n_k.  The workspace is sized by the query side,
 * nwg = B * H * ceil(L_q / 256).
 */
size_t sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(int B, int L_q, int L_k, int H, int d);
int sigmoid_attn_cross_bwd_dq_dbias(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                                    float *dbias, const int32_t *seqlens_q, const int32_t *seqlens_k,
                                    const float *bias, float scale, int B, int L_q, int L_k, int H, int d,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * sigmoid_attn_bwd_dq_dbias for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as sigmoid_attn_bwd_dq_dbias, minus the workspace: the per-workgroup partial sums go
 * to an array of SIGATTN_STATIC_SCRATCH_BYTES bytes that lives in the library's device image (each GPU
 * the library runs on holds its own copy until the process ends).  The call allocates and frees nothing.
 *   limit : B * H * ceil(N_max / 256) * 8 bytes must fit the array (131072 query tiles); beyond that the
 *           call returns SIGATTN_ERR_TOO_LARGE and enqueues nothing.
 *   races : every call on one GPU uses that GPU's one array, whatever the stream.  Calls whose kernels
 *           may overlap on one GPU (different streams, or graphs replayed concurrently) race on it; calls
 *           on one stream are ordered and safe.  The array keeps the last call's partials; no call relies
 *           on its contents on entry.
 * SIGATTN_ERR_LAUNCH is also returned if the array's device address cannot be obtained.
 */
#define SIGATTN_STATIC_SCRATCH_BYTES (1 << 20)
int sigmoid_attn_bwd_dq_dbias_static(const void *q, const void *k, const void *v, const void *d_o, void *dq,
                                     float *dbias, const int32_t *seqlens, const float *bias, float scale,
                                     int B, int N_max, int H, int d, void *stream);

/* Scratch bytes sigmoid_attn_bwd needs for this shape (0 on invalid shapes). */
size_t sigmoid_attn_bwd_workspace_bytes(int B, int N_max, int H, int d);

#ifdef __cplusplus
}
#endif
#endif /* SIGMOID_ATTN_H */
