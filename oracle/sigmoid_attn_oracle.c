/*
 * Oracle for padded bidirectional sigmoid attention -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU path must compute,
 * written in fp64 from the paper.  It is used by the tests, the smoke check and
 * the CPU-baseline leg of the benchmark.  It shares no code, header, table or
 * helper with the HIP library and must never be called from the product path.
 *
 * Definition (paper Sec. 3, the sigmoid-attention equation; appendix Alg. 1-3
 * for the padding rules and the gradients):
 *
 *   for a sequence z with n = seqlens[z] valid tokens (a prefix of the N rows),
 *   a head h, q_i = Q[z,i,h,:], k_j = K[z,j,h,:], v_j = V[z,j,h,:]:
 *
 *     x_ij = scale * <q_i, k_j> + bias[z]          i, j < n
 *     P_ij = sigma(x_ij) = 1 / (1 + exp(-x_ij))
 *     O_i  = sum_{j<n} P_ij v_j                     i < n ;  O_i = 0 for i >= n
 *
 *   and, for an upstream gradient dO (rows >= n ignored):
 *
 *     dP_ij = <dO_i, v_j>
 *     dS_ij = P_ij (1 - P_ij) dP_ij                 (diagonal Jacobian of sigma)
 *     dV_j  = sum_{i<n} P_ij dO_i
 *     dK_j  = scale * sum_{i<n} dS_ij q_i
 *     dQ_i  = scale * sum_{j<n} dS_ij k_j
 *     dQ_i = dK_j = dV_j = 0 for i, j >= n
 *
 * Padded positions are handled as a select (masked score -> P = 0), never as
 * (-inf)*0 arithmetic; padded input rows are never read.
 *
 * Layout: every tensor is [B, N, H, d] with d fastest.  Inputs are float32
 * holding bf16-representable values and are widened exactly to double; every
 * intermediate and every output is double.  No tiling, no blocking, no
 * reordering beyond what the definition states.  OpenMP only spreads
 * independent output rows over threads.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* sigma(x), evaluated without overflow on either tail. */
static double sigma(double x)
{
    if (x >= 0.0) {
        return 1.0 / (1.0 + exp(-x));
    } else {
        double e = exp(x);
        return e / (1.0 + e);
    }
}

static size_t at(int z, int i, int h, int N, int H, int d)
{
    return (((size_t)z * (size_t)N + (size_t)i) * (size_t)H + (size_t)h) * (size_t)d;
}

static int valid_len(const int32_t *seqlens, int z, int N)
{
    int n = seqlens[z];
    if (n < 0) n = 0;
    if (n > N) n = N;
    return n;
}

int sigattn_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Forward for one (z, h) slice; writes rows [0, N) of o for that slice. */
void sigattn_oracle_fwd_slice(const float *q, const float *k, const float *v, double *o,
                              const int32_t *seqlens, const double *bias, double scale,
                              int B, int N, int H, int d, int z, int h)
{
    (void)B;
    const int n = valid_len(seqlens, z, N);
#pragma omp parallel for schedule(dynamic, 8)
    for (int i = 0; i < N; ++i) {
        double *oi = o + at(z, i, h, N, H, d);
        for (int c = 0; c < d; ++c) oi[c] = 0.0;
        if (i >= n) continue;
        const float *qi = q + at(z, i, h, N, H, d);
        for (int j = 0; j < n; ++j) {
            const float *kj = k + at(z, j, h, N, H, d);
            const float *vj = v + at(z, j, h, N, H, d);
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
            const double p = sigma(scale * s + bias[z]);
            for (int c = 0; c < d; ++c) oi[c] += p * (double)vj[c];
        }
    }
}

/* Backward for one (z, h) slice; writes rows [0, N) of dq, dk, dv for that slice. */
void sigattn_oracle_bwd_slice(const float *q, const float *k, const float *v, const float *d_o,
                              double *dq, double *dk, double *dv,
                              const int32_t *seqlens, const double *bias, double scale,
                              int B, int N, int H, int d, int z, int h)
{
    (void)B;
    const int n = valid_len(seqlens, z, N);
    /* dQ: one query row at a time. */
#pragma omp parallel for schedule(dynamic, 8)
    for (int i = 0; i < N; ++i) {
        double *dqi = dq + at(z, i, h, N, H, d);
        for (int c = 0; c < d; ++c) dqi[c] = 0.0;
        if (i >= n) continue;
        const float *qi = q + at(z, i, h, N, H, d);
        const float *doi = d_o + at(z, i, h, N, H, d);
        for (int j = 0; j < n; ++j) {
            const float *kj = k + at(z, j, h, N, H, d);
            const float *vj = v + at(z, j, h, N, H, d);
            double s = 0.0, dp = 0.0;
            for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
            for (int c = 0; c < d; ++c) dp += (double)doi[c] * (double)vj[c];
            const double x = scale * s + bias[z];
            const double ds = sigma(x) * sigma(-x) * dp; /* P (1 - P) dP */
            for (int c = 0; c < d; ++c) dqi[c] += ds * (double)kj[c];
        }
        for (int c = 0; c < d; ++c) dqi[c] *= scale;
    }
    /* dK, dV: one key row at a time. */
#pragma omp parallel for schedule(dynamic, 8)
    for (int j = 0; j < N; ++j) {
        double *dkj = dk + at(z, j, h, N, H, d);
        double *dvj = dv + at(z, j, h, N, H, d);
        for (int c = 0; c < d; ++c) { dkj[c] = 0.0; dvj[c] = 0.0; }
        if (j >= n) continue;
        const float *kj = k + at(z, j, h, N, H, d);
        const float *vj = v + at(z, j, h, N, H, d);
        for (int i = 0; i < n; ++i) {
            const float *qi = q + at(z, i, h, N, H, d);
            const float *doi = d_o + at(z, i, h, N, H, d);
            double s = 0.0, dp = 0.0;
            for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
            for (int c = 0; c < d; ++c) dp += (double)doi[c] * (double)vj[c];
            const double x = scale * s + bias[z];
            const double p = sigma(x);
            const double ds = p * sigma(-x) * dp;
            for (int c = 0; c < d; ++c) dvj[c] += p * (double)doi[c];
            for (int c = 0; c < d; ++c) dkj[c] += ds * (double)qi[c];
        }
        for (int c = 0; c < d; ++c) dkj[c] *= scale;
    }
}

/* All slices. */
void sigattn_oracle_fwd(const float *q, const float *k, const float *v, double *o,
                        const int32_t *seqlens, const double *bias, double scale,
                        int B, int N, int H, int d)
{
    for (int z = 0; z < B; ++z)
        for (int h = 0; h < H; ++h)
            sigattn_oracle_fwd_slice(q, k, v, o, seqlens, bias, scale, B, N, H, d, z, h);
}

void sigattn_oracle_bwd(const float *q, const float *k, const float *v, const float *d_o,
                        double *dq, double *dk, double *dv,
                        const int32_t *seqlens, const double *bias, double scale,
                        int B, int N, int H, int d)
{
    for (int z = 0; z < B; ++z)
        for (int h = 0; h < H; ++h)
            sigattn_oracle_bwd_slice(q, k, v, d_o, dq, dk, dv, seqlens, bias, scale, B, N, H, d, z, h);
}

/*
 * The n x n matrices of one slice, for the invariants the paper states about
 * them (weights in (0,1); |dS| <= |dP| / 4).  p, dp, ds are [N][N] row-major,
 * zero outside the valid n x n corner.  d_o may be NULL (then dp, ds are not
 * written).
 */
void sigattn_oracle_matrices(const float *q, const float *k, const float *v, const float *d_o,
                             double *p, double *dp, double *ds,
                             const int32_t *seqlens, const double *bias, double scale,
                             int B, int N, int H, int d, int z, int h)
{
    (void)B;
    const int n = valid_len(seqlens, z, N);
    for (int i = 0; i < N; ++i) {
        for (int j = 0; j < N; ++j) {
            const size_t ij = (size_t)i * (size_t)N + (size_t)j;
            p[ij] = 0.0;
            if (d_o) { dp[ij] = 0.0; ds[ij] = 0.0; }
            if (i >= n || j >= n) continue;
            const float *qi = q + at(z, i, h, N, H, d);
            const float *kj = k + at(z, j, h, N, H, d);
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
            const double x = scale * s + bias[z];
            p[ij] = sigma(x);
            if (d_o) {
                const float *doi = d_o + at(z, i, h, N, H, d);
                const float *vj = v + at(z, j, h, N, H, d);
                double g = 0.0;
                for (int c = 0; c < d; ++c) g += (double)doi[c] * (double)vj[c];
                dp[ij] = g;
                ds[ij] = sigma(x) * sigma(-x) * g;
            }
        }
    }
}

/*
 * ---------------------------------------------------------------------------
 * Separate query and key lengths, and the gradient of the bias.
 *
 * Appendix Alg. 1-3 are written for q in [Z, L_q, H, D] and k, v in
 * [Z, L_k, H, D] with valid lengths n_q and n_k of their own; Sec. 3 allows
 * the bias b to be learnable.  Same definition as above with i < n_q, j < n_k:
 *
 *   O_i  = sum_{j<n_k} P_ij v_j      (i < n_q; 0 for i >= n_q, and 0 when n_k = 0)
 *   dV_j = sum_{i<n_q} P_ij dO_i,  dK_j = scale sum_{i<n_q} dS_ij q_i   (j < n_k)
 *   dQ_i = scale sum_{j<n_k} dS_ij k_j                                  (i < n_q)
 *   db_z = sum_h sum_{i<n_q} sum_{j<n_k} dS_ij      (x_ij = scale s_ij + b_z, so dx_ij/db_z = 1)
 *
 * Plain loops again; nothing is shared with the functions above except sigma()
 * and the index helper.  db may be NULL.
 * ---------------------------------------------------------------------------
 */
void sigattn_oracle_cross_fwd(const float *q, const float *k, const float *v, double *o,
                              const int32_t *seqlens_q, const int32_t *seqlens_k, const double *bias,
                              double scale, int B, int Lq, int Lk, int H, int d)
{
    for (int z = 0; z < B; ++z) {
        const int nq = valid_len(seqlens_q, z, Lq), nk = valid_len(seqlens_k, z, Lk);
        for (int h = 0; h < H; ++h) {
#pragma omp parallel for schedule(dynamic, 8)
            for (int i = 0; i < Lq; ++i) {
                double *oi = o + at(z, i, h, Lq, H, d);
                for (int c = 0; c < d; ++c) oi[c] = 0.0;
                if (i >= nq) continue;
                const float *qi = q + at(z, i, h, Lq, H, d);
                for (int j = 0; j < nk; ++j) {
                    const float *kj = k + at(z, j, h, Lk, H, d);
                    const float *vj = v + at(z, j, h, Lk, H, d);
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
                    const double p = sigma(scale * s + bias[z]);
                    for (int c = 0; c < d; ++c) oi[c] += p * (double)vj[c];
                }
            }
        }
    }
}

void sigattn_oracle_cross_bwd(const float *q, const float *k, const float *v, const float *d_o,
                              double *dq, double *dk, double *dv, double *db,
                              const int32_t *seqlens_q, const int32_t *seqlens_k, const double *bias,
                              double scale, int B, int Lq, int Lk, int H, int d)
{
    for (int z = 0; z < B; ++z) {
        const int nq = valid_len(seqlens_q, z, Lq), nk = valid_len(seqlens_k, z, Lk);
        double dbz = 0.0;
        for (int h = 0; h < H; ++h) {
            /* dQ and the bias gradient: one query row at a time. */
            double dbh = 0.0;
#pragma omp parallel for schedule(dynamic, 8) reduction(+ : dbh)
            for (int i = 0; i < Lq; ++i) {
                double *dqi = dq + at(z, i, h, Lq, H, d);
                for (int c = 0; c < d; ++c) dqi[c] = 0.0;
                if (i >= nq) continue;
                const float *qi = q + at(z, i, h, Lq, H, d);
                const float *doi = d_o + at(z, i, h, Lq, H, d);
                for (int j = 0; j < nk; ++j) {
                    const float *kj = k + at(z, j, h, Lk, H, d);
                    const float *vj = v + at(z, j, h, Lk, H, d);
                    double s = 0.0, dp = 0.0;
                    for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
                    for (int c = 0; c < d; ++c) dp += (double)doi[c] * (double)vj[c];
                    const double x = scale * s + bias[z];
                    const double ds = sigma(x) * sigma(-x) * dp;
                    dbh += ds;
                    for (int c = 0; c < d; ++c) dqi[c] += ds * (double)kj[c];
                }
                for (int c = 0; c < d; ++c) dqi[c] *= scale;
            }
            dbz += dbh;
            /* dK, dV: one key row at a time. */
#pragma omp parallel for schedule(dynamic, 8)
            for (int j = 0; j < Lk; ++j) {
                double *dkj = dk + at(z, j, h, Lk, H, d);
                double *dvj = dv + at(z, j, h, Lk, H, d);
                for (int c = 0; c < d; ++c) { dkj[c] = 0.0; dvj[c] = 0.0; }
                if (j >= nk) continue;
                const float *kj = k + at(z, j, h, Lk, H, d);
                const float *vj = v + at(z, j, h, Lk, H, d);
                for (int i = 0; i < nq; ++i) {
                    const float *qi = q + at(z, i, h, Lq, H, d);
                    const float *doi = d_o + at(z, i, h, Lq, H, d);
                    double s = 0.0, dp = 0.0;
                    for (int c = 0; c < d; ++c) s += (double)qi[c] * (double)kj[c];
                    for (int c = 0; c < d; ++c) dp += (double)doi[c] * (double)vj[c];
                    const double x = scale * s + bias[z];
                    const double p = sigma(x);
                    const double ds = p * sigma(-x) * dp;
                    for (int c = 0; c < d; ++c) dvj[c] += p * (double)doi[c];
                    for (int c = 0; c < d; ++c) dkj[c] += ds * (double)qi[c];
                }
                for (int c = 0; c < d; ++c) dkj[c] *= scale;
            }
        }
        if (db) db[z] = dbz;
    }
}
