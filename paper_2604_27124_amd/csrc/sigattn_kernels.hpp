// Device code for padded bidirectional sigmoid attention on gfx950 (CDNA4).
//
// One kernel template serves the three passes of the method (paper appendix Alg. 1-3):
//
//   FWD   (Alg. 1): owner = a tile of queries,  streamed = key/value tiles.   Out = O
//   DQ    (Alg. 2): owner = a tile of queries,  streamed = key/value tiles.   Out = dQ
//   DKDV  (Alg. 3): owner = a tile of keys,     streamed = query/dO tiles.    Out = dK, dV
//
// "Owner" rows are held in registers for the whole kernel as MFMA B operands; "streamed" tiles go
// HBM -> registers -> LDS (double buffered) and are read from LDS as MFMA A operands, either row-wise
// (contraction over the head dimension) or through the transposing LDS read (contraction over tokens).
// Every score tile is computed transposed, streamed x owner, so that the fp32 accumulator of one lane
// holds one owner column and several streamed rows: after the fused sigmoid those registers are, without
// any shuffle, the bf16 B operand of the next contraction over streamed tokens.
//
// v_mfma_f32_32x32x16_bf16 operand layout used below (lane l, c = l % 32, g = l / 32):
//   A[32 x 16]: lane holds row c,    k = 8 g + 0..7
//   B[16 x 32]: lane holds column c, k = 8 g + 0..7
//   C[32 x 32]: lane holds column c, register i holds row 8 (i / 4) + 4 g + (i % 4)
// ds_read_b64_tr_b16 within a group of 16 lanes: destination lane i, element e comes from the 8 bytes
// addressed by lane (i / 4 + 4 e), 16-bit column (i % 4).  With lane r of the group pointing at
// (row r / 4, column 4 (r % 4)) of a row-major [4 x 16] block, lane i receives column i, rows 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sigattn {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum Mode { FWD = 0, DQ = 1, DKDV = 2 };

template <int V>
struct IntC {
    static constexpr int value = V;
};

struct Params {
    const bf16_t *q, *k, *v, *d_o;   // inputs  [B, N, H, D]
    bf16_t *out0;                    // FWD: O;  DQ: dQ;  DKDV: dK
    bf16_t *out1;                    // DKDV: dV
    const int32_t *seqlens;          // [B]
    const float *bias;               // [B]
    float scale;
    int B, N, H;
};

#define SIGATTN_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

__device__ __forceinline__ bf16x8 lds_read_rows(const bf16_t *p) {
    return *reinterpret_cast<const bf16x8 *>(p);
}

// Two transposing reads -> the 8 contraction slots of one A operand.
__device__ __forceinline__ bf16x8 lds_read_tr(const bf16_t *p_lo, const bf16_t *p_hi) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SIGATTN_LDS_PTR(s16x4, p_lo));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SIGATTN_LDS_PTR(s16x4, p_hi));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(unsigned, h);
}

// Registers 8 half .. 8 half + 7 of a score accumulator -> bf16 B operand (contraction slots = streamed rows).
__device__ __forceinline__ bf16x8 acc_to_operand(const f32x16 &a, int half) {
    u32x4 r;
    r[0] = pack_bf16(a[8 * half + 0], a[8 * half + 1]);
    r[1] = pack_bf16(a[8 * half + 2], a[8 * half + 3]);
    r[2] = pack_bf16(a[8 * half + 4], a[8 * half + 5]);
    r[3] = pack_bf16(a[8 * half + 6], a[8 * half + 7]);
    return __builtin_bit_cast(bf16x8, r);
}

template <int MODE, int D, int QB, int NW, int BN, int LD1, int LD2>
struct Cfg {
    static constexpr int BM = NW * 32 * QB;        // owner rows per workgroup
    static constexpr int THREADS = NW * 64;
    static constexpr int KS = D / 16;              // MFMA steps over the head dimension
    static constexpr int MB = D / 32;              // 32-row blocks of a transposed [D x 32] output
    static constexpr int NB = BN / 32;             // 32-row blocks of a streamed tile
    static constexpr int CH = D / 8;               // 16-byte chunks per row
    static constexpr int PER = (BN * CH) / THREADS;  // chunks per thread per streamed tensor
    static constexpr int NBUF = 4;                 // LDS ring: tile t lives in slot t % 4
    static constexpr size_t LDS_BYTES = (size_t)NBUF * BN * (LD1 + LD2) * sizeof(bf16_t);
    static_assert((BN * CH) % THREADS == 0, "tile does not split evenly over the workgroup");
    static_assert(D % 32 == 0 && BN % 64 == 0, "tile shape (an even number of 32-row blocks per tile)");
    static_assert(LD1 % 8 == 0 && LD2 % 8 == 0 && LD1 >= D && LD2 >= D, "LDS row stride");
};

// Write zeros over owner rows [row0, row1) of one (z, h) slice of `out`.
template <int D, int THREADS>
__device__ __forceinline__ void zero_rows(bf16_t *out, size_t slice_base, size_t row_stride, int row0, int row1) {
    constexpr int CH = D / 8;
    const int total = (row1 - row0) * CH;
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int c = threadIdx.x; c < total; c += THREADS) {
        const int r = row0 + c / CH;
        *reinterpret_cast<u32x4 *>(out + slice_base + (size_t)r * row_stride + (size_t)(c % CH) * 8) = z;
    }
}

// bf16 x 8 times a float, rounded back to bf16 (used once per kernel, on the owner rows).
__device__ __forceinline__ bf16x8 scale_bf16x8(const bf16x8 v, const float f) {
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = pack_bf16((float)v[2 * j] * f, (float)v[2 * j + 1] * f);
    return __builtin_bit_cast(bf16x8, r);
}

// The fused elementwise step on one 32 x 32 score block held in MFMA accumulator layout.
//   in : s  = t' = -(log2 e) scale <q, k>   (the factor is already inside the contraction)
//        dp = dP (backward only);  cb = 2^(-bias log2 e)
//   out: s  = P = sigma(x) = 1 / (1 + cb 2^t');  dp = dS = P (1 - P) dP, computed as P dP - P (P dP)
// cb is finite and non-zero, so cb * 2^t' is 0, finite or +inf but never NaN, and P lands in [0, 1].
// Streamed rows >= n (register i <-> row srow0 + 8 (i / 4) + i % 4) get P = 0 when MASKED.
template <bool HAS2, bool MASKED>
__device__ __forceinline__ void sigmoid_block(f32x16 &s, f32x16 &dp, const float cb, const int srow0, const int n) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float e = __builtin_amdgcn_exp2f(s[i]);
        float pr = __builtin_amdgcn_rcpf(__builtin_fmaf(cb, e, 1.0f));
        if (MASKED) pr = (srow0 + 8 * (i >> 2) + (i & 3) < n) ? pr : 0.f;
        s[i] = pr;
        if (HAS2) {
            const float t1 = pr * dp[i];
            dp[i] = __builtin_fmaf(-pr, t1, t1);
        }
    }
}

// Longest-first work mapping.  The launch is a 1-D grid with one workgroup per owner tile of every
// (z, h); hardware hands consecutive workgroup ids to the 8 XCDs round-robin and to free CUs in order.
// Ids are therefore mapped so that the tiles of the LONGEST sequences come first (their cost is
// proportional to the sequence's valid length) and every XCD receives every 8th tile of that sorted list;
// wholly padded tiles, which only write zeros, come last.  Sequences are ranked inside the kernel from
// seqlens (B <= MAP_MAX_B; larger batches keep batch order), so the host never needs the lengths.
constexpr int MAP_MAX_B = 256;

template <int BM, int THREADS>
__device__ __forceinline__ void map_work(const Params &p, int &z, int &h, int &n, int &m0) {
    __shared__ int s_len[MAP_MAX_B];      // clamped valid length, by batch index
    __shared__ int s_seq[MAP_MAX_B];      // batch index, by rank (longest first)
    const int T = (p.N + BM - 1) / BM;    // owner tiles per (z, h), padded ones included
    const int id = blockIdx.x;
    const bool sorted = p.B <= MAP_MAX_B;
    if (sorted) {
        for (int t = threadIdx.x; t < p.B; t += THREADS) {
            const int v = p.seqlens[t];
            s_len[t] = v < 0 ? 0 : (v > p.N ? p.N : v);
        }
        __syncthreads();
        for (int t = threadIdx.x; t < p.B; t += THREADS) {
            const int mine = s_len[t];
            int rank = 0;
            for (int u = 0; u < p.B; ++u) {
                const int o = s_len[u];
                rank += (o > mine || (o == mine && u < t)) ? 1 : 0;
            }
            s_seq[rank] = t;
        }
        __syncthreads();
    }
    auto len_of = [&](int b) {
        if (sorted) return s_len[b];
        const int v = p.seqlens[b];
        return v < 0 ? 0 : (v > p.N ? p.N : v);
    };
    // valid tiles, longest sequence first; then the padded tiles
    int rest = id;
    bool found = false;
    z = 0; h = 0; n = 0; m0 = 0;
    for (int r = 0; r < p.B && !found; ++r) {
        const int b = sorted ? s_seq[r] : r;
        const int len = len_of(b);
        const int cnt = ((len + BM - 1) / BM) * p.H;
        if (rest < cnt) {
            z = b; n = len; h = rest % p.H; m0 = (rest / p.H) * BM;
            found = true;
        } else {
            rest -= cnt;
        }
    }
    for (int b = 0; b < p.B && !found; ++b) {
        const int len = len_of(b);
        const int first = (len + BM - 1) / BM;
        const int cnt = (T - first) * p.H;
        if (rest < cnt) {
            z = b; n = len; h = rest % p.H; m0 = (first + rest / p.H) * BM;
            found = true;
        } else {
            rest -= cnt;
        }
    }
}

template <int MODE, int D, int QB, int NW, int BN, int LD1, int LD2, int OCC>
__global__ void __launch_bounds__(NW * 64, OCC) sigattn_kernel(const Params p) {
    using C = Cfg<MODE, D, QB, NW, BN, LD1, LD2>;
    constexpr bool HAS2 = (MODE != FWD);             // a second owner tensor and a second score tile (dP)
    constexpr int Q2 = HAS2 ? QB : 1;
    constexpr float LOG2E = 1.4426950408889634f;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *y1s = reinterpret_cast<bf16_t *>(smem);                 // [NBUF][BN][LD1]
    bf16_t *y2s = y1s + C::NBUF * BN * LD1;                         // [NBUF][BN][LD2]

    // Work mapping (1-D grid over every owner tile of every (z, h)): see map_work().
    int z, h, n, m0;
    map_work<C::BM, C::THREADS>(p, z, h, n, m0);
    z = __builtin_amdgcn_readfirstlane(z);      // uniform across the workgroup: keep them in scalar registers
    h = __builtin_amdgcn_readfirstlane(h);
    n = __builtin_amdgcn_readfirstlane(n);
    m0 = __builtin_amdgcn_readfirstlane(m0);
    const int m1 = (m0 + C::BM < p.N) ? m0 + C::BM : p.N;
    const size_t row_stride = (size_t)p.H * D;
    const size_t slice = ((size_t)z * p.N * p.H + h) * D;           // element offset of row 0 of (z, h)

    if (m0 >= n) {   // wholly padded owner tile: write zeros, do nothing else (block-sparse early exit)
        zero_rows<D, C::THREADS>(p.out0, slice, row_stride, m0, m1);
        if (MODE == DKDV) zero_rows<D, C::THREADS>(p.out1, slice, row_stride, m0, m1);
        return;
    }

    const bf16_t *x1 = (MODE == DKDV) ? p.k : p.q;                  // owner tensors
    const bf16_t *x2 = (MODE == DKDV) ? p.v : p.d_o;
    const bf16_t *y1 = (MODE == DKDV) ? p.q : p.k;                  // streamed tensors
    const bf16_t *y2 = (MODE == DKDV) ? p.d_o : p.v;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, g = lane >> 5;
    const int wrow0 = m0 + wave * 32 * QB;                          // first owner row of this wave

    // sigma(x) = 1 / (1 + cb 2^t') with t' = c1 <q, k>, c1 = -scale log2 e, cb = 2^(-bias log2 e).
    // c1 is folded into the owner operand of the score contraction (one extra bf16 rounding of that
    // operand), so t' leaves the MFMA ready for exp2; cb rides on the FMA that forms the denominator.
    // The exponent of cb is clamped to +-126 (|bias| <= 87.3 is exact; beyond that sigma is saturated).
    const float c1 = -p.scale * LOG2E;
    const float cb = __builtin_amdgcn_exp2f(__builtin_fminf(__builtin_fmaxf(-p.bias[z] * LOG2E, -126.0f), 126.0f));

    // ---- owner rows -> registers (B operands): lane holds row c of each 32-block, d = 16 ks + 8 g + 0..7
    bf16x8 xa[QB][C::KS];
    bf16x8 xb[Q2][HAS2 ? C::KS : 1];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int r = wrow0 + 32 * qb + c;
        const bool ok = r < n;
        const size_t off = slice + (size_t)(ok ? r : 0) * row_stride + 8 * g;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (ok) t = *reinterpret_cast<const u32x4 *>(x1 + off + 16 * ks);
            xa[qb][ks] = scale_bf16x8(__builtin_bit_cast(bf16x8, t), c1);
            if (HAS2) {
                u32x4 t2 = {0u, 0u, 0u, 0u};
                if (ok) t2 = *reinterpret_cast<const u32x4 *>(x2 + off + 16 * ks);
                xb[qb][ks] = __builtin_bit_cast(bf16x8, t2);
            }
        }
    }

    f32x16 acc0[QB][C::MB];                        // FWD: O^T;  DQ: dQ^T;  DKDV: dK^T
    f32x16 acc1[MODE == DKDV ? QB : 1][MODE == DKDV ? C::MB : 1];   // DKDV: dV^T
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc0[qb][mb][i] = 0.f;
            if (MODE == DKDV) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc1[qb][mb][i] = 0.f;
            }
        }

    // ---- streamed tile movement: HBM -> registers -> LDS ring slot
    const int ntiles = (n + BN - 1) / BN;
    u32x4 st1[C::PER], st2[C::PER];
    auto load_tile = [&](int t) {   // branch-free: rows beyond the valid length read a clamped row, then become 0
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            const int cid = tid + it * C::THREADS;
            const int r = t * BN + cid / C::CH;
            const int col = (cid % C::CH) * 8;
            const bool ok = r < n;
            const size_t off = slice + (size_t)(ok ? r : n - 1) * row_stride + col;
            const u32x4 a = *reinterpret_cast<const u32x4 *>(y1 + off);
            const u32x4 b = *reinterpret_cast<const u32x4 *>(y2 + off);
            const u32x4 z4 = {0u, 0u, 0u, 0u};
            st1[it] = ok ? a : z4;
            st2[it] = ok ? b : z4;
        }
    };
    auto store_tile = [&](int slot) {
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            const int cid = tid + it * C::THREADS;
            const int r = cid / C::CH;
            const int col = (cid % C::CH) * 8;
            *reinterpret_cast<u32x4 *>(y1s + (slot * BN + r) * LD1 + col) = st1[it];
            *reinterpret_cast<u32x4 *>(y2s + (slot * BN + r) * LD2 + col) = st2[it];
        }
    };

    // lane-constant pieces of the LDS addresses
    const int rd_off1 = c * LD1 + 8 * g;           // row-wise A operand: row c, columns 16 ks + 8 g
    const int rd_off2 = c * LD2 + 8 * g;
    const int i16 = lane & 15, g16 = (lane >> 4) & 1;
    const int tr_row = 4 * g + (i16 >> 2);         // transposed A operand: rows 4 g + 0..3 (and + 8)
    const int tr_col = 16 * g16 + 4 * (i16 & 3);   // 16 output rows (head-dim columns) per 16-lane group
    const int tr_off1 = tr_row * LD1 + tr_col;
    const int tr_off2 = tr_row * LD2 + tr_col;

    // Stage A of a 32-row block: transposed scores t'^T[streamed 32 x owner 32] = Y1 (c1 X1)^T,
    // and dP^T = Y2 X2^T (backward).
    auto stage_scores = [&](const bf16_t *t1, const bf16_t *t2, f32x16 (&s)[QB], f32x16 (&dp)[Q2]) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16x8 a1 = lds_read_rows(t1 + rd_off1 + 16 * ks);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, xa[qb][ks], ks == 0 ? zero : s[qb], 0, 0, 0);
            if (HAS2) {
                const bf16x8 a2 = lds_read_rows(t2 + rd_off2 + 16 * ks);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    dp[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, xb[qb][ks], ks == 0 ? zero : dp[qb], 0, 0, 0);
            }
        }
    };

    // Stage C of a 32-row block: the contractions over its 32 streamed rows (two MFMA steps of 16), from
    // the bf16 operands stage B left behind.
    auto stage_outputs = [&](const bf16_t *t1, const bf16_t *t2, const bf16x8 (&pb)[QB][2], const bf16x8 (&dsb)[Q2][2]) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb) {
                if (MODE == FWD) {          // O^T += V^T P^T
                    const bf16_t *a = t2 + 16 * half * LD2 + tr_off2 + 32 * mb;
                    const bf16x8 vt = lds_read_tr(a, a + 8 * LD2);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        acc0[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt, pb[qb][half], acc0[qb][mb], 0, 0, 0);
                } else {                    // dQ^T += K^T dS^T   |   dK^T += Q^T dS
                    const bf16_t *a = t1 + 16 * half * LD1 + tr_off1 + 32 * mb;
                    const bf16x8 yt = lds_read_tr(a, a + 8 * LD1);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        acc0[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yt, dsb[qb][half], acc0[qb][mb], 0, 0, 0);
                    if (MODE == DKDV) {     // dV^T += dO^T P
                        const bf16_t *a2 = t2 + 16 * half * LD2 + tr_off2 + 32 * mb;
                        const bf16x8 gt = lds_read_tr(a2, a2 + 8 * LD2);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            acc1[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, pb[qb][half], acc1[qb][mb], 0, 0, 0);
                    }
                }
            }
        }
    };

    // Score accumulators and bf16 operands, double buffered by block parity.
    f32x16 sbuf[2][QB], dbuf[2][Q2];
    bf16x8 pbuf[2][QB][2], dsbuf[2][Q2][2];

    // One pipeline step for the block of parity PAR.  Three independent pieces of work sit in one basic
    // block: the score MFMAs of the NEXT block, the output MFMAs of the PREVIOUS block, and the sigmoid of
    // THIS block on the VALU, so that the matrix pipe and the VALU can run side by side within one wave.
    auto step = [&](auto masked_c, auto has_next_c, auto par_c, const bf16_t *n1, const bf16_t *n2,
                    const bf16_t *p1, const bf16_t *p2, const int srow0) {
        constexpr bool MASKED = decltype(masked_c)::value;
        constexpr bool HAS_NEXT = decltype(has_next_c)::value;
        constexpr int PAR = decltype(par_c)::value;
        if (HAS_NEXT) stage_scores(n1, n2, sbuf[PAR ^ 1], dbuf[PAR ^ 1]);
        stage_outputs(p1, p2, pbuf[PAR ^ 1], dsbuf[PAR ^ 1]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            sigmoid_block<HAS2, MASKED>(sbuf[PAR][qb], dbuf[PAR][HAS2 ? qb : 0], cb, srow0, n);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                pbuf[PAR][qb][half] = acc_to_operand(sbuf[PAR][qb], half);
                if (HAS2) dsbuf[PAR][qb][half] = acc_to_operand(dbuf[PAR][qb], half);
            }
        }
    };
    using std_true = IntC<1>;
    using std_false = IntC<0>;

    // ---- prologue: tiles 0 and 1 into the ring, tile 2 into registers, scores of block 0 computed
    load_tile(0);
    store_tile(0);
    if (ntiles > 1) {
        load_tile(1);
        store_tile(1);
    }
    __syncthreads();
    load_tile(2);

    stage_scores(y1s, y2s, sbuf[0], dbuf[0]);
    {   // the "previous block" of block 0 contributes nothing: zero operands
        const u32x4 z4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                pbuf[1][qb][half] = __builtin_bit_cast(bf16x8, z4);
                if (HAS2) dsbuf[1][qb][half] = __builtin_bit_cast(bf16x8, z4);
            }
    }

    // ---- main loop over all tiles but the last: no padded rows, every block has a successor
    int slot = 0;                                    // t % NBUF
    const bf16_t *prev1 = y1s, *prev2 = y2s;         // block whose output contractions are still due
    for (int t = 0; t + 1 < ntiles; ++t) {
        const int slot_next = (slot + 1) & (C::NBUF - 1);
        const bf16_t *t1 = y1s + slot * BN * LD1;
        const bf16_t *t2 = y2s + slot * BN * LD2;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
            const bf16_t *n1 = (nb + 1 < C::NB) ? t1 + (nb + 1) * 32 * LD1 : y1s + slot_next * BN * LD1;
            const bf16_t *n2 = (nb + 1 < C::NB) ? t2 + (nb + 1) * 32 * LD2 : y2s + slot_next * BN * LD2;
            const int srow0 = t * BN + nb * 32 + 4 * g;
            if (nb & 1) step(std_false{}, std_true{}, IntC<1>{}, n1, n2, prev1, prev2, srow0);
            else        step(std_false{}, std_true{}, IntC<0>{}, n1, n2, prev1, prev2, srow0);
            prev1 = t1 + nb * 32 * LD1;
            prev2 = t2 + nb * 32 * LD2;
        }
        // tile t + 2 goes to slot (t + 2) % 4 = (t - 2) % 4, last read during tile t - 1 (as the previous
        // block of its first step); every wave passed the barrier that ended tile t - 1.  It becomes
        // visible at this barrier, a full tile before its first read at the end of tile t + 1.
        // (Past the end these are harmless: the registers then hold zeros and the slot is not live.)
        store_tile((slot + 2) & (C::NBUF - 1));
        __syncthreads();
        load_tile(t + 3);
        slot = slot_next;
    }

    // ---- last tile: rows >= n masked, the final block has no successor
    {
        const int t = ntiles - 1;
        const bf16_t *t1 = y1s + slot * BN * LD1;
        const bf16_t *t2 = y2s + slot * BN * LD2;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
            const bf16_t *n1 = t1 + (nb + 1) * 32 * LD1;
            const bf16_t *n2 = t2 + (nb + 1) * 32 * LD2;
            const int srow0 = t * BN + nb * 32 + 4 * g;
            if (nb + 1 < C::NB) {
                if (nb & 1) step(std_true{}, std_true{}, IntC<1>{}, n1, n2, prev1, prev2, srow0);
                else        step(std_true{}, std_true{}, IntC<0>{}, n1, n2, prev1, prev2, srow0);
            } else {
                if (nb & 1) step(std_true{}, std_false{}, IntC<1>{}, n1, n2, prev1, prev2, srow0);
                else        step(std_true{}, std_false{}, IntC<0>{}, n1, n2, prev1, prev2, srow0);
            }
            prev1 = t1 + nb * 32 * LD1;
            prev2 = t2 + nb * 32 * LD2;
        }
        stage_outputs(prev1, prev2, pbuf[(C::NB - 1) & 1], dsbuf[(C::NB - 1) & 1]);
    }

    // ---- epilogue: transposed fp32 accumulators -> bf16 rows.  Lane holds owner row c of each block,
    // register i holds head-dim column 32 mb + 8 (i/4) + 4 g + (i%4): four consecutive columns per store.
    const float oscale = (MODE == FWD) ? 1.0f : p.scale;            // dQ and dK carry the factor `scale`
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int r = wrow0 + 32 * qb + c;
        if (r >= p.N) continue;
        const bool ok = r < n;                                       // padded owner rows are written as zero
        const size_t off = slice + (size_t)r * row_stride + 4 * g;
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w0 = {0u, 0u};
                if (ok) {
                    w0[0] = pack_bf16(acc0[qb][mb][4 * q4 + 0] * oscale, acc0[qb][mb][4 * q4 + 1] * oscale);
                    w0[1] = pack_bf16(acc0[qb][mb][4 * q4 + 2] * oscale, acc0[qb][mb][4 * q4 + 3] * oscale);
                }
                *reinterpret_cast<u32x2 *>(p.out0 + off + 32 * mb + 8 * q4) = w0;
                if (MODE == DKDV) {
                    u32x2 w1 = {0u, 0u};
                    if (ok) {
                        w1[0] = pack_bf16(acc1[qb][mb][4 * q4 + 0], acc1[qb][mb][4 * q4 + 1]);
                        w1[1] = pack_bf16(acc1[qb][mb][4 * q4 + 2], acc1[qb][mb][4 * q4 + 3]);
                    }
                    *reinterpret_cast<u32x2 *>(p.out1 + off + 32 * mb + 8 * q4) = w1;
                }
            }
        }
    }
}

}  // namespace sigattn
