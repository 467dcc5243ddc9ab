// Device code for padded bidirectional sigmoid attention on gfx950 (CDNA4).
//
// One kernel template serves the three passes of the method (paper appendix Alg. 1-3):
//
//   FWD   (Alg. 1): owner = a tile of queries,  streamed = key/value tiles.   Out = O
//   DQ    (Alg. 2): owner = a tile of queries,  streamed = key/value tiles.   Out = dQ
//   DKDV  (Alg. 3): owner = a tile of keys,     streamed = query/dO tiles.    Out = dK, dV
//
// "Owner" rows are held in registers for the whole kernel as MFMA B operands; "streamed" tiles go
// HBM -> registers -> LDS (a ring of four tiles) and are read from LDS as MFMA A operands, either row-wise
// (contraction over the head dimension) or through the transposing LDS read (contraction over tokens).
// Every score tile is computed transposed, streamed x owner, so that the fp32 accumulator of one lane
// holds one owner column and several streamed rows: after the fused sigmoid those registers are, without
// any shuffle, the bf16 B operand of the next contraction over streamed tokens.
//
// The inner loop is a software pipeline over 32-row blocks of the streamed tensors.  One step holds, for
// block b, the score contractions of block b + 1, the sigmoid of block b and the output contractions of
// block b - 1.  A step is cut into slots of one MFMA each; every slot also carries an equal share of the
// step's VALU work and, at most, the LDS read of one later A operand.  A operands travel through a small
// ring of registers and are requested RING - 1 operands before their first use, so that no MFMA waits for
// the LDS.  The order inside a step is pinned with scheduling fences; nothing is left to reorder.
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
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum Mode { FWD = 0, DQ = 1, DKDV = 2 };

template <int V>
struct IntC {
    static constexpr int value = V;
    __device__ __forceinline__ constexpr int get() const { return V; }
};
struct DynInt {   // same interface as IntC for a value only known at run time
    int v;
    __device__ __forceinline__ int get() const { return v; }
};

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for<I + 1, N>(f);
    }
}

// Owner side = the tensors whose rows a workgroup keeps (queries in FWD and DQ, keys in DKDV); streamed side
// = the other one.  The two sides have padded lengths and valid lengths of their own (appendix Alg. 1-3:
// L_q, L_k, n_q, n_k); self-attention passes the same numbers twice.
struct Params {
    const bf16_t *q, *k, *v, *d_o;   // inputs: q, d_o [B, L_q, H, D];  k, v [B, L_k, H, D]
    bf16_t *out0;                    // FWD: O;  DQ: dQ;  DKDV: dK
    bf16_t *out1;                    // DKDV: dV
    const int32_t *seqlens;          // [B] valid lengths of the owner side
    const int32_t *seqlens_str;      // [B] valid lengths of the streamed side
    const float *bias;               // [B]
    float scale;
    int B, N, H;                     // N: padded length of the owner side
    int N_str;                       // padded length of the streamed side
    float *db_part;                  // DQ with bias gradient: per-workgroup partial sums [gridDim.x]
    int32_t *db_seq;                 //   and the sequence each workgroup belongs to [gridDim.x]
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

// a * b under the rule 0 * x = 0 for every x, also +-inf and NaN (v_mul_legacy_f32).
__device__ __forceinline__ float mul_zero_wins(float a, float b) {
    float r;
    asm("v_mul_legacy_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(unsigned, h);
}

// Shape of one pipeline step and of the two instruction streams that are woven into it.
template <int MODE, int D, int QB, int NW, int BN, int LD1, int LD2, int RING>
struct Cfg {
    static constexpr bool HAS2 = (MODE != FWD);    // a second owner tensor and a second score tile (dP)
    static constexpr int BM = NW * 32 * QB;        // owner rows per workgroup
    static constexpr int THREADS = NW * 64;
    static constexpr int KS = D / 16;              // MFMA steps over the head dimension
    static constexpr int MB = D / 32;              // 32-row blocks of a transposed [D x 32] output
    static constexpr int NB = BN / 32;             // 32-row blocks of a streamed tile
    static constexpr int CH = D / 8;               // 16-byte chunks per row
    static constexpr int PER = (BN * CH) / THREADS;  // chunks per thread per streamed tensor
    static constexpr int NBUF = 4;                 // LDS ring: tile t lives in slot t % 4
    static constexpr size_t LDS_BYTES = (size_t)NBUF * BN * (LD1 + LD2) * sizeof(bf16_t);
    // A operands of one step, in the order they are used: first the row-wise ones of the score
    // contractions (block b + 1), then the transposed ones of the output contractions (block b - 1).
    static constexpr int NT = HAS2 ? 2 : 1;        // score tiles per block (S, dP)
    static constexpr int NO = (MODE == DKDV) ? 2 : 1;   // output tensors
    static constexpr int NA = KS * NT;
    static constexpr int NC = 2 * MB * NO;
    static constexpr int NOPS = NA + NC;
    static constexpr int SLOTS = NOPS * QB;        // one MFMA per slot
    // VALU work: units of two score elements (one packed bf16 register of the next B operand).
    static constexpr int UNITS = QB * 8;
    // LDS placement of a streamed row t: element offset t * LD + lds_shift(t).  Mode 0 is the plain padded
    // layout (row stride 16 bytes modulo 32): conflict-free for the 16-byte row-wise reads of 16 consecutive
    // rows.  The transposing 8-byte reads of a half-wave touch four consecutive rows; at D = 64 that layout
    // costs them nothing measurable, at D = 128 (272-byte rows) it quarters their rate.  Mode 2, for D = 128
    // tensors that are read transposed: 288-byte rows (32 bytes modulo the 256 bytes of the banks), the 32
    // output rows of one MFMA taken as two groups of 16 head-dim columns that lie 128 bytes apart, so that
    // the four rows of a read fall into disjoint banks; every second group of eight rows is shifted by a
    // further 16 bytes, which keeps the row-wise reads conflict-free under that stride.
    static constexpr int lds_mode(int LD) { return ((2 * LD) % 256 == 32 && D == 128) ? 2 : 0; }
    static constexpr int LM1 = lds_mode(LD1), LM2 = lds_mode(LD2);
    static_assert(LM1 != 2 || LD1 >= D + 8, "mode 2 shifts a row by up to 16 bytes");
    static_assert(LM2 != 2 || LD2 >= D + 8, "mode 2 shifts a row by up to 16 bytes");
    static_assert((BN * CH) % THREADS == 0, "tile does not split evenly over the workgroup");
    static_assert(D % 32 == 0 && BN % 64 == 0, "tile shape (an even number of 32-row blocks per tile)");
    static_assert(LD1 % 8 == 0 && LD2 % 8 == 0 && LD1 >= D && LD2 >= D, "LDS row stride");
    static_assert((NB * NOPS) % RING == 0 && RING >= 2 && RING <= NOPS, "operand ring does not close over a tile");
};

// Element offset added to row `row` of a streamed tile in LDS (see Cfg::lds_mode), the extra offset of the
// second transposing read (eight rows further on), and the column layout of the transposed operand.
template <int LM>
__device__ __forceinline__ constexpr int lds_shift(int row) {
    return LM == 2 ? 8 * ((row >> 3) & 1) : 0;
}
template <int LM>
struct TrLayout {
    static constexpr int HI_EXTRA = LM == 2 ? 8 : 0;                    // lds_shift(row + 8) - lds_shift(row), row % 8 < 4
    static constexpr int GROUP_COLS = LM == 2 ? 64 : 16;                // column distance of the two 16-lane groups
    static constexpr int MB_COLS = LM == 2 ? 16 : 32;                   // column step from one output block to the next
    // head-dim column of accumulator registers 4 q4 .. 4 q4 + 3 of output block mb (without the 4 g of the lane)
    static constexpr int out_col(int mb, int q4) {
        return LM == 2 ? 16 * mb + 64 * (q4 >> 1) + 8 * (q4 & 1) : 32 * mb + 8 * q4;
    }
};

// The VALU instructions of one step as a flat list.  Each unit (two score elements) runs through three
// stages -- exponentials | denominator and reciprocal | products and packing -- and the list is skewed by
// one unit per stage, so that an instruction never follows directly on the one that feeds it.
template <int UNITS, int OPU, int S0, int S1>
struct ValuOrder {
    static constexpr int LEN = UNITS * OPU;
    int unit[LEN];
    int op[LEN];
    constexpr ValuOrder() : unit{}, op{} {
        int n = 0;
        for (int tau = 0; tau < UNITS + 2; ++tau) {
            if (tau < UNITS)
                for (int o = 0; o < S0; ++o) { unit[n] = tau; op[n] = o; ++n; }
            if (tau >= 1 && tau - 1 < UNITS)
                for (int o = S0; o < S1; ++o) { unit[n] = tau - 1; op[n] = o; ++n; }
            if (tau >= 2 && tau - 2 < UNITS)
                for (int o = S1; o < OPU; ++o) { unit[n] = tau - 2; op[n] = o; ++n; }
        }
    }
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

// Longest-first work mapping.  The launch is a 1-D grid with one workgroup per owner tile of every
// (z, h); hardware hands consecutive workgroup ids to the 8 XCDs round-robin and to free CUs in order.
// Ids are therefore mapped so that the tiles of the LONGEST sequences come first (their cost is
// proportional to the sequence's valid length), every XCD receives every 8th id of that sorted list, and
// within one sequence the ids of one XCD are consecutive tiles of the same head; wholly padded tiles,
// which only write zeros, come last.  Sequences are ranked inside the kernel from seqlens, so the host
// never needs the lengths: up to MAP_MAX_B sequences by their exact length (every thread ranks one
// sequence against all others in LDS); larger batches by their number of owner tiles (at most
// MAP_CLASSES of them: the host refuses longer paddings for such batches), with a histogram and
// block-wide prefix sums (work per thread grows with B / THREADS, not with B).  Ties keep batch order
// in both forms.
constexpr int MAP_MAX_B = 256;
constexpr int MAP_CLASSES = 1024;

// Ids [lo, lo + cnt) are the H * tiles valid ids of one sequence.  Hardware deals consecutive ids round-robin
// to the 8 XCDs, each with an L2 of its own; the ids of the range that land on one XCD take consecutive
// tiles of one head (then of the next), so a head's streamed slab is fetched by one or two XCDs only.
// Returns the position of `id` in that XCD-major order of the range.
__device__ __forceinline__ int xcd_major_index(int id, int lo, int cnt) {
    const int idx = id - lo, x = id & 7;
    int e = 0;                                      // ids of this range on XCDs below x
    for (int y = 0; y < x; ++y) {
        const int first = (y - lo) & 7;             // first index of the range that lands on XCD y
        e += (first < cnt) ? ((cnt - first + 7) >> 3) : 0;
    }
    return e + ((idx - ((x - lo) & 7)) >> 3);       // plus the position among the ids on XCD x
}

template <int BM, int THREADS>
__device__ __forceinline__ void map_work(const Params &p, int &z, int &h, int &n, int &m0) {
    __shared__ int s_len[MAP_MAX_B];      // clamped valid length, by batch index
    __shared__ int s_res[4];              // z, n, h, m0 of this workgroup
    static_assert((BM & (BM - 1)) == 0, "owner tile rows: a power of two");
    const int T = (p.N + BM - 1) / BM;    // owner tiles per (z, h), padded ones included
    const int id = blockIdx.x;
    auto len_of = [&](int b) {
        const int v = p.seqlens[b];
        return v < 0 ? 0 : (v > p.N ? p.N : v);
    };
    if (p.B <= MAP_MAX_B) {
        // Id ranges: the valid tiles of every sequence, longest sequence first (ties in batch order), H ids
        // per tile; then the padded tiles in batch order.  One thread per sequence sums, in a single pass over
        // the lengths (uniform LDS reads, no dependent chain), the tiles in front of its own ranges, and the
        // thread whose range holds this workgroup's id publishes the answer.
        for (int t = threadIdx.x; t < p.B; t += THREADS) s_len[t] = len_of(t);
        __syncthreads();
        for (int t = threadIdx.x; t < p.B; t += THREADS) {
            const int mine = s_len[t], my_tiles = (mine + BM - 1) / BM;
            int before_valid = 0, before_padded = 0, all_valid = 0;
#pragma unroll 8
            for (int u = 0; u < p.B; ++u) {
                const int o = s_len[u], tiles = (o + BM - 1) / BM;
                const bool ahead = o > mine || (o == mine && u < t);
                before_valid += ahead ? tiles : 0;
                before_padded += (u < t) ? (T - tiles) : 0;
                all_valid += tiles;
            }
            {   // valid tiles of sequence t: ids lo .. lo + cnt - 1
                const int lo = before_valid * p.H, cnt = my_tiles * p.H;
                if (id >= lo && id < lo + cnt) {
                    const int e = xcd_major_index(id, lo, cnt);
                    s_res[0] = t; s_res[1] = mine; s_res[2] = e / my_tiles; s_res[3] = (e % my_tiles) * BM;
                }
            }
            {   // padded tiles of sequence t
                const int lo = (all_valid + before_padded) * p.H, cnt = (T - my_tiles) * p.H;
                if (id >= lo && id < lo + cnt) {
                    const int rest = id - lo;
                    s_res[0] = t; s_res[1] = mine; s_res[2] = rest % p.H; s_res[3] = (my_tiles + rest / p.H) * BM;
                }
            }
        }
        __syncthreads();
        z = s_res[0]; n = s_res[1]; h = s_res[2]; m0 = s_res[3];
        return;
    }

    // ---- more sequences than the pairwise ranking holds.  A sequence's class is its number of owner tiles
    // (class 0 = T tiles, the longest; T <= MAP_CLASSES is the host's check).
    // Id ranges: classes in ascending order, inside a class the sequences in batch order, H ids per tile;
    // then the padded tiles in batch order.  All positions are kept in tiles: a sequence whose tiles are
    // [tb, tb + tiles) of that list owns the ids [H tb, H (tb + tiles)).
    __shared__ int s_hist[MAP_CLASSES];   // owner tiles per class
    __shared__ int s_wave[THREADS / 64];  // wave totals of a block-wide prefix sum
    __shared__ int s_pick[4];             // class holding this id (-1: padded part) | tiles before it | all valid tiles | found
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto class_of = [&](int tiles) { return T - tiles; };      // tiles in [1, T]
    for (int i = tid; i < MAP_CLASSES; i += THREADS) s_hist[i] = 0;
    if (tid == 0) { s_pick[0] = -1; s_pick[3] = 0; }
    __syncthreads();
    for (int b = tid; b < p.B; b += THREADS) {
        const int tiles = (len_of(b) + BM - 1) / BM;
        if (tiles > 0) atomicAdd(&s_hist[class_of(tiles)], tiles);
    }
    __syncthreads();
    const int tgt = id / p.H;             // position of this id's tile in the list of all tiles
    if (wave == 0) {                      // prefix over the classes: each lane sums a run of them, lanes by shuffles
        constexpr int RUN = MAP_CLASSES / 64;
        int mine = 0;
        for (int i = 0; i < RUN; ++i) mine += s_hist[lane * RUN + i];
        int incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            incl += (lane >= off) ? up : 0;
        }
        if (lane == 63) s_pick[2] = incl;
        int before = incl - mine;
        if (tgt >= before && tgt < incl) {            // at most one lane
            int c = lane * RUN;
            while (tgt >= before + s_hist[c]) { before += s_hist[c]; ++c; }
            s_pick[0] = c; s_pick[1] = before;
        }
    }
    __syncthreads();
    const int cls = s_pick[0], all_valid = s_pick[2];
    const int base = cls >= 0 ? s_pick[1] : all_valid;      // tiles in front of the part that is searched
    const int rest = tgt - base;                            // position inside that part, in batch order
    int running = 0;
    for (int c0 = 0; c0 < p.B; c0 += THREADS) {
        const int b = c0 + tid;
        int len = 0, tiles = 0, v = 0;
        if (b < p.B) {
            len = len_of(b);
            tiles = (len + BM - 1) / BM;
            v = cls >= 0 ? ((tiles > 0 && class_of(tiles) == cls) ? tiles : 0) : T - tiles;
        }
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            incl += (lane >= off) ? up : 0;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int offset = 0, total = 0;
#pragma unroll
        for (int w = 0; w < THREADS / 64; ++w) {
            const int t = s_wave[w];
            offset += (w < wave) ? t : 0;
            total += t;
        }
        const int hi = running + offset + incl, lo_t = hi - v;
        if (v > 0 && rest >= lo_t && rest < hi) {           // exactly one thread of one chunk
            const int lo = (base + lo_t) * p.H;             // first id of this sequence's range
            if (cls >= 0) {
                const int e = xcd_major_index(id, lo, tiles * p.H);
                s_res[0] = b; s_res[1] = len; s_res[2] = e / tiles; s_res[3] = (e % tiles) * BM;
            } else {
                const int r = id - lo;
                s_res[0] = b; s_res[1] = len; s_res[2] = r % p.H; s_res[3] = (tiles + r / p.H) * BM;
            }
            s_pick[3] = 1;
        }
        __syncthreads();
        if (s_pick[3]) break;
        running += total;
    }
    z = s_res[0]; n = s_res[1]; h = s_res[2]; m0 = s_res[3];
}

template <int MODE, int D, int QB, int NW, int BN, int LD1, int LD2, int OCC, int RING, bool WITH_DB = false>
__global__ void __launch_bounds__(NW * 64, OCC) sigattn_kernel(const Params p) {
    static_assert(!WITH_DB || MODE == DQ, "the bias gradient rides on the dQ kernel");
    using C = Cfg<MODE, D, QB, NW, BN, LD1, LD2, RING>;
    constexpr bool HAS2 = C::HAS2;
    constexpr int Q2 = HAS2 ? QB : 1;
    constexpr int NB = C::NB, NA = C::NA, NOPS = C::NOPS, SLOTS = C::SLOTS, NT = C::NT, NO = C::NO, MB = C::MB;
    constexpr float LOG2E = 1.4426950408889634f;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ float s_db[WITH_DB ? NW : 1];                        // bias gradient: one partial per wave
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
    const size_t slice = ((size_t)z * p.N * p.H + h) * D;           // owner side: element offset of row 0 of (z, h)
    const size_t slice_s = ((size_t)z * p.N_str * p.H + h) * D;     // streamed side
    int ns = n;                                                     // valid rows of the streamed side
    if (p.seqlens_str != p.seqlens || p.N_str != p.N) {             // self-attention: the mapping already has it
        ns = p.seqlens_str[z];
        ns = ns < 0 ? 0 : (ns > p.N_str ? p.N_str : ns);
    }
    ns = __builtin_amdgcn_readfirstlane(ns);

    // Wholly padded owner tile, or nothing to stream: write zeros, do nothing else (block-sparse early exit).
    if (m0 >= n || ns == 0) {
        zero_rows<D, C::THREADS>(p.out0, slice, row_stride, m0, m1);
        if (MODE == DKDV) zero_rows<D, C::THREADS>(p.out1, slice, row_stride, m0, m1);
        if (WITH_DB && threadIdx.x == 0) {
            p.db_part[blockIdx.x] = 0.f;
            p.db_seq[blockIdx.x] = z;
        }
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
    // cb is finite and non-zero, so cb 2^t' is 0, finite or +inf but never NaN, and P lands in [0, 1].
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
            xa[qb][ks] = __builtin_bit_cast(bf16x8, t);      // scaled by c1 once the streamed tiles are requested
            if (HAS2) {
                u32x4 t2 = {0u, 0u, 0u, 0u};
                if (ok) t2 = *reinterpret_cast<const u32x4 *>(x2 + off + 16 * ks);
                xb[qb][ks] = __builtin_bit_cast(bf16x8, t2);
            }
        }
    }

    f32x16 acc0[QB][MB];                           // FWD: O^T;  DQ: dQ^T;  DKDV: dK^T
    f32x16 acc1[MODE == DKDV ? QB : 1][MODE == DKDV ? MB : 1];   // DKDV: dV^T
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc0[qb][mb][i] = 0.f;
            if (MODE == DKDV) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc1[qb][mb][i] = 0.f;
            }
        }

    // Bias gradient db = sum of dS over all valid pairs: one more (small) MFMA per 16 streamed rows with an
    // all-ones A operand sums the bf16 values that also feed dQ.  v_mfma_f32_16x16x32_bf16 reads the B operand
    // of the 32-wide shape as 16 columns x 32 contraction slots: column j of its result is the sum over the
    // lanes congruent to j modulo 16 -- which owner rows and streamed rows get mixed does not matter for a
    // total -- and every row of the result holds the same 16 sums.
    f32x4 accdb[WITH_DB ? QB : 1];
    bf16x8 ones;
    if (WITH_DB) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int i = 0; i < 4; ++i) accdb[qb][i] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) ones[i] = (bf16_t)1.0f;
    }

    // ---- streamed tile movement: HBM -> registers -> LDS ring slot
    const int ntiles = (ns + BN - 1) / BN;
    u32x4 st1[C::PER], st2[C::PER];
    // Thread tid moves chunk tid % CH of rows tid / CH + it * RPI, it = 0 .. PER - 1: one lane constant,
    // everything else is uniform (scalar registers) or a compile-time offset.
    constexpr int RPI = C::THREADS / C::CH;        // rows per pass of the workgroup over a tile
    static_assert(C::THREADS % C::CH == 0 && (C::PER == 1 || RPI % 16 == 0), "a pass must keep the LDS row shift");
    const int r0 = tid / C::CH, col0 = (tid % C::CH) * 8;
    const unsigned ld_off0 = (unsigned)r0 * (unsigned)row_stride + (unsigned)col0;
    auto load_tile = [&](int t) {   // branch-free: rows beyond the valid length read a clamped row, then become 0
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            const int r = t * BN + it * RPI + r0;
            const bool ok = r < ns;
            const size_t off = slice_s + (size_t)(ok ? r : ns - 1) * row_stride + col0;
            const u32x4 a = *reinterpret_cast<const u32x4 *>(y1 + off);
            const u32x4 b = *reinterpret_cast<const u32x4 *>(y2 + off);
            const u32x4 z4 = {0u, 0u, 0u, 0u};
            st1[it] = ok ? a : z4;
            st2[it] = ok ? b : z4;
        }
    };
    // Tiles that lie wholly below the valid length need neither the clamp nor the zero fill: their
    // addresses are a uniform base (scalar registers, advanced per tile and pass) plus the lane constant.
    auto load_full_tile = [&](int t) {
        const bf16_t *b1 = y1 + slice_s + (size_t)t * BN * row_stride;
        const bf16_t *b2 = y2 + slice_s + (size_t)t * BN * row_stride;
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            st1[it] = *reinterpret_cast<const u32x4 *>(b1 + (size_t)it * RPI * row_stride + ld_off0);
            st2[it] = *reinterpret_cast<const u32x4 *>(b2 + (size_t)it * RPI * row_stride + ld_off0);
        }
    };
    auto load_next = [&](int t) {   // t * BN + BN <= ns exactly when t < ntiles - 1
        if (t < ntiles - 1) load_full_tile(t);
        else load_tile(t);
    };
    bf16_t *const w1 = y1s + r0 * LD1 + lds_shift<C::LM1>(r0) + col0;   // LDS home of this thread's chunk, pass 0, slot 0
    bf16_t *const w2 = y2s + r0 * LD2 + lds_shift<C::LM2>(r0) + col0;
    auto store_tile = [&](int slot) {
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            *reinterpret_cast<u32x4 *>(w1 + (slot * BN + it * RPI) * LD1) = st1[it];
            *reinterpret_cast<u32x4 *>(w2 + (slot * BN + it * RPI) * LD2) = st2[it];
        }
    };

    // lane-constant pieces of the LDS addresses
    const int i16 = lane & 15, g16 = (lane >> 4) & 1;
    using TL1 = TrLayout<C::LM1>;
    using TL2 = TrLayout<C::LM2>;
    const int tr_row = 4 * g + (i16 >> 2);         // transposed A operand: rows 4 g + 0..3 (and + 8)
    // 16 output rows (head-dim columns) per 16-lane group; block and tile offsets are multiples of 16 rows and
    // leave the shift of a row unchanged, so every address stays a lane constant plus an immediate
    const bf16_t *rd1 = y1s + c * LD1 + lds_shift<C::LM1>(c) + 8 * g;     // row-wise A operand: row c, columns 16 ks + 8 g
    const bf16_t *rd2 = y2s + c * LD2 + lds_shift<C::LM2>(c) + 8 * g;
    const bf16_t *tr1 = y1s + tr_row * LD1 + lds_shift<C::LM1>(tr_row) + TL1::GROUP_COLS * g16 + 4 * (i16 & 3);
    const bf16_t *tr2 = y2s + tr_row * LD2 + lds_shift<C::LM2>(tr_row) + TL2::GROUP_COLS * g16 + 4 * (i16 & 3);

    // Score accumulators and bf16 operands, double buffered by block parity.
    f32x16 sbuf[2][QB], dbuf[2][Q2];
    u32x4 pbuf[2][QB][2], dsbuf[2][Q2][2];
    bf16x8 ring[RING];

    // First ring row of the block `delta` blocks after block nb of the tile in ring slot `slot`.
    auto block_row = [&](auto slot, int nb, int delta) {
        const int nbp = nb + delta + NB;                       // >= 0 for delta >= -NB
        const int sl = (slot.get() + nbp / NB + C::NBUF - 1) & (C::NBUF - 1);
        return sl * BN + (nbp % NB) * 32;
    };

    // The J-th A operand counted from the start of the step on block nb of `slot` (J >= NOPS runs into the
    // following step): row-wise operands belong to the block after the step's block, transposed ones to the
    // block before it.
    auto fetch = [&](auto J_, auto slot, int nb) -> bf16x8 {
        constexpr int J = decltype(J_)::value;
        constexpr int sstep = J / NOPS, j = J % NOPS;
        if constexpr (j < NA) {
            constexpr int ks = j / NT, which = j % NT;
            const int row = block_row(slot, nb, sstep + 1);
            if constexpr (which == 0) return lds_read_rows(rd1 + row * LD1 + 16 * ks);
            else return lds_read_rows(rd2 + row * LD2 + 16 * ks);
        } else {
            constexpr int jj = j - NA, which = jj % NO, idx = jj / NO, half = idx / MB, mb = idx % MB;
            const int row = block_row(slot, nb, sstep - 1) + 16 * half;
            // FWD contracts V^T (tensor 2); DQ contracts K^T (tensor 1); DKDV: Q^T (1) for dK, dO^T (2) for dV
            constexpr bool second = (MODE == FWD) || (MODE == DKDV && which == 1);
            if constexpr (second) {
                const bf16_t *a = tr2 + row * LD2 + TL2::MB_COLS * mb;
                return lds_read_tr(a, a + 8 * LD2 + TL2::HI_EXTRA);
            } else {
                const bf16_t *a = tr1 + row * LD1 + TL1::MB_COLS * mb;
                return lds_read_tr(a, a + 8 * LD1 + TL1::HI_EXTRA);
            }
        }
    };

    // VALU work of one step: see ValuOrder.  Per unit u (registers 2w, 2w + 1 of owner block qb = u / 8):
    //   0,1  e = 2^t'            2,3  y = 1 + cb e          4,5  P = 1 / y      [6,7  P = 0 on padded rows]
    //   FWD : pack P
    //   bwd : g = e P (2 ops), a = P dP (2 ops), dS / cb = g a (2 ops), pack it, DKDV also packs P
    // 1 - P = cb e P holds without cancellation however close P is to 1, so dS = P (1 - P) dP keeps its
    // relative accuracy on the saturated tail; the constant cb is applied once, to the finished sums.
    // e = +inf (score far below the bias) meets P = 0 there: the product must be 0, not NaN.
    constexpr int OPU_BASE = (MODE == FWD) ? 7 : (MODE == DQ ? 13 : 14);

    // One pipeline step on the block (slot, nb) of parity PAR (compile-time nb).  Slots run in program
    // order; a scheduling fence closes each of them.
    auto step = [&](auto masked_c, auto has_next_c, auto drain_c, auto nb_c, auto slot, const int srow0,
                    auto store_at_c, const int store_slot) {
        constexpr bool MASKED = decltype(masked_c)::value;
        constexpr int STORE_AT = decltype(store_at_c)::value;   // slot before which the staged tile goes to LDS (-1: never)
        constexpr bool HAS_NEXT = decltype(has_next_c)::value;
        constexpr bool DRAIN = decltype(drain_c)::value;
        constexpr int nb = decltype(nb_c)::value;
        constexpr int PAR = nb & 1;
        constexpr int G0 = (nb * NOPS) % RING;               // ring position of this step's first operand
        constexpr int MK = MASKED ? 2 : 0;
        constexpr int OPU = OPU_BASE + MK;
        constexpr ValuOrder<C::UNITS, OPU, 2, 6> order{};
        constexpr int LEN = DRAIN ? 0 : C::UNITS * OPU;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        float pv[HAS2 ? C::UNITS : 1][2];          // y, then P, of the units in flight (backward only)

        static_for<0, SLOTS>([&](auto k_) {
            constexpr int k = decltype(k_)::value;
            constexpr int j = k / QB, qb = k % QB;
            if constexpr (k == STORE_AT) {
                store_tile(store_slot);
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- the MFMA of this slot
            if constexpr (j < NA) {
                if constexpr (HAS_NEXT && !DRAIN) {
                    constexpr int ks = j / NT, which = j % NT;
                    if constexpr (which == 0)
                        sbuf[PAR ^ 1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            ring[(G0 + j) % RING], xa[qb][ks], ks == 0 ? zero : sbuf[PAR ^ 1][qb], 0, 0, 0);
                    else
                        dbuf[PAR ^ 1][HAS2 ? qb : 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            ring[(G0 + j) % RING], xb[HAS2 ? qb : 0][HAS2 ? ks : 0],
                            ks == 0 ? zero : dbuf[PAR ^ 1][HAS2 ? qb : 0], 0, 0, 0);
                }
            } else {
                constexpr int jj = j - NA, which = jj % NO, idx = jj / NO, half = idx / MB, mb = idx % MB;
                const bf16x8 a = ring[(G0 + j) % RING];
                if constexpr (MODE == FWD) {            // O^T += V^T P^T
                    acc0[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        a, __builtin_bit_cast(bf16x8, pbuf[PAR ^ 1][qb][half]), acc0[qb][mb], 0, 0, 0);
                } else if constexpr (which == 0) {      // dQ^T += K^T dS^T   |   dK^T += Q^T dS
                    acc0[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        a, __builtin_bit_cast(bf16x8, dsbuf[PAR ^ 1][HAS2 ? qb : 0][half]), acc0[qb][mb], 0, 0, 0);
                    if constexpr (WITH_DB && mb == MB - 1)
                        accdb[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            ones, __builtin_bit_cast(bf16x8, dsbuf[PAR ^ 1][HAS2 ? qb : 0][half]), accdb[qb], 0, 0, 0);
                } else {                                // dV^T += dO^T P
                    acc1[MODE == DKDV ? qb : 0][MODE == DKDV ? mb : 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        a, __builtin_bit_cast(bf16x8, pbuf[PAR ^ 1][qb][half]),
                        acc1[MODE == DKDV ? qb : 0][MODE == DKDV ? mb : 0], 0, 0, 0);
                }
            }
            // ---- the register of the previous operand is free now: request the operand RING - 1 ahead
            if constexpr (qb == 0 && (!DRAIN || j + RING - 1 < NOPS)) {
                ring[(G0 + j + RING - 1) % RING] = fetch(IntC<j + RING - 1>{}, slot, nb);
            }
            // ---- this slot's share of the sigmoid
            static_for<(k * LEN) / SLOTS, ((k + 1) * LEN) / SLOTS>([&](auto i_) {
                constexpr int i = decltype(i_)::value;
                constexpr int u = order.unit[i], o = order.op[i];
                constexpr int uq = u / 8, w = u % 8, ra = 2 * w, rb = 2 * w + 1;
                f32x16 &s = sbuf[PAR][uq];
                f32x16 &dp = dbuf[PAR][HAS2 ? uq : 0];
                // the forward pass turns the score register into y and P in place; the backward passes keep
                // e = 2^t' there and carry y, then P, in pv
                constexpr int pu = HAS2 ? u : 0;
                auto y_of = [&](auto which) -> float {
                    if constexpr (HAS2) return pv[pu][decltype(which)::value];
                    else return s[decltype(which)::value ? rb : ra];
                };
                auto set_y = [&](auto which, const float val) {
                    if constexpr (HAS2) pv[pu][decltype(which)::value] = val;
                    else s[decltype(which)::value ? rb : ra] = val;
                };
                constexpr IntC<0> A_{};
                constexpr IntC<1> B_{};
                if constexpr (o == 0) s[ra] = __builtin_amdgcn_exp2f(s[ra]);
                else if constexpr (o == 1) s[rb] = __builtin_amdgcn_exp2f(s[rb]);
                else if constexpr (o == 2) set_y(A_, __builtin_fmaf(cb, s[ra], 1.0f));
                else if constexpr (o == 3) set_y(B_, __builtin_fmaf(cb, s[rb], 1.0f));
                else if constexpr (o == 4) set_y(A_, __builtin_amdgcn_rcpf(y_of(A_)));
                else if constexpr (o == 5) set_y(B_, __builtin_amdgcn_rcpf(y_of(B_)));
                else if constexpr (MASKED && o == 6) set_y(A_, (srow0 + 8 * (ra >> 2) + (ra & 3) < ns) ? y_of(A_) : 0.f);
                else if constexpr (MASKED && o == 7) set_y(B_, (srow0 + 8 * (rb >> 2) + (rb & 3) < ns) ? y_of(B_) : 0.f);
                else {
                    constexpr int e = o - 6 - MK;     // position in the mode's tail of the unit
                    if constexpr (MODE == FWD) {
                        pbuf[PAR][uq][w / 4][w % 4] = pack_bf16(s[ra], s[rb]);
                    } else {
                        if constexpr (e == 0) s[ra] = mul_zero_wins(s[ra], y_of(A_));
                        else if constexpr (e == 1) s[rb] = mul_zero_wins(s[rb], y_of(B_));
                        else if constexpr (e == 2) dp[ra] = y_of(A_) * dp[ra];
                        else if constexpr (e == 3) dp[rb] = y_of(B_) * dp[rb];
                        else if constexpr (e == 4) dp[ra] = s[ra] * dp[ra];
                        else if constexpr (e == 5) dp[rb] = s[rb] * dp[rb];
                        else if constexpr (e == 6) dsbuf[PAR][HAS2 ? uq : 0][w / 4][w % 4] = pack_bf16(dp[ra], dp[rb]);
                        else pbuf[PAR][uq][w / 4][w % 4] = pack_bf16(y_of(A_), y_of(B_));
                    }
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using T_ = IntC<1>;
    using F_ = IntC<0>;

    // ---- prologue: tiles 0 and 1 into the ring, tile 2 into registers, scores of block 0 computed.
    // The step on block 0 contracts its (zero) "previous" operands with the last block of ring slot 3:
    // that block is cleared first, so that 0 x stale LDS bits can never be 0 x NaN.
    for (int cid = tid; cid < 32 * (LD1 / 8); cid += C::THREADS) {
        const u32x4 z4 = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(y1s + (C::NBUF * BN - 32) * LD1 + cid * 8) = z4;
    }
    for (int cid = tid; cid < 32 * (LD2 / 8); cid += C::THREADS) {
        const u32x4 z4 = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(y2s + (C::NBUF * BN - 32) * LD2 + cid * 8) = z4;
    }
    {   // the first three tiles are requested back to back, so their latencies overlap
        load_tile(0);
        u32x4 a1[C::PER], a2[C::PER];
#pragma unroll
        for (int it = 0; it < C::PER; ++it) { a1[it] = st1[it]; a2[it] = st2[it]; }
        load_tile(1);
        u32x4 b1[C::PER], b2[C::PER];
#pragma unroll
        for (int it = 0; it < C::PER; ++it) { b1[it] = st1[it]; b2[it] = st2[it]; }
        load_tile(2);
        // every request of the prologue is in flight now; the owner rows, requested first, arrive first
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) xa[qb][ks] = scale_bf16x8(xa[qb][ks], c1);
#pragma unroll
        for (int it = 0; it < C::PER; ++it) {
            *reinterpret_cast<u32x4 *>(w1 + (it * RPI) * LD1) = a1[it];
            *reinterpret_cast<u32x4 *>(w2 + (it * RPI) * LD2) = a2[it];
            *reinterpret_cast<u32x4 *>(w1 + (BN + it * RPI) * LD1) = b1[it];
            *reinterpret_cast<u32x4 *>(w2 + (BN + it * RPI) * LD2) = b2[it];
        }
    }
    __syncthreads();

    {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16x8 a1 = lds_read_rows(rd1 + 16 * ks);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                sbuf[0][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, xa[qb][ks], ks == 0 ? zero : sbuf[0][qb], 0, 0, 0);
            if (HAS2) {
                const bf16x8 a2 = lds_read_rows(rd2 + 16 * ks);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    dbuf[0][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, xb[qb][ks], ks == 0 ? zero : dbuf[0][qb], 0, 0, 0);
            }
        }
        const u32x4 z4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                pbuf[1][qb][half] = z4;
                if (HAS2) dsbuf[1][qb][half] = z4;
            }
    }
    // operands 0 .. RING - 2 of the first step
    static_for<0, RING - 1>([&](auto J_) { ring[decltype(J_)::value % RING] = fetch(J_, IntC<0>{}, 0); });

    // ---- main loop over all tiles but the last: no padded rows, every block has a successor.  The loop is
    // unrolled over the four ring slots so that every LDS address is a lane constant plus an immediate.
    // Tile t + 2 goes to slot (t + 2) % 4 = (t - 2) % 4, last read during the first step of tile t - 1 (as
    // the previous block); every wave passed the barrier that ended tile t - 1.  The staged registers are
    // written half-way through the last step of tile t, and the barrier that ends the tile waits only until
    // those writes have left the LDS queue: LDS operations of a wave complete in order, so it is enough to
    // let the READS_AFTER operand reads issued behind them stay in flight.  The tile becomes visible at
    // that barrier, most of a tile before its first read near the end of tile t + 1.
    // (Past the end the writes are harmless: the registers then hold zeros and the slot is not live.)
    constexpr auto reads_from = [](int first_slot) {
        int cnt = 0;
        for (int k = first_slot; k < SLOTS; k += QB) {
            const int j = (k / QB + RING - 1) % NOPS;
            cnt += (j < NA) ? 1 : 2;           // one 16-byte read, or two transposing 8-byte reads
        }
        return cnt;
    };
    constexpr int STORE_AT = [&] {             // about half-way, later if too many reads would follow
        int k = (SLOTS / 2 / QB) * QB;
        while (reads_from(k) > 12) k += QB;
        return k;
    }();
    constexpr int READS_AFTER = reads_from(STORE_AT);
    static_assert(READS_AFTER <= 15 && STORE_AT < SLOTS, "more reads behind the tile store than the LDS counter can express");
    auto tile_body = [&](auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        static_for<0, NB>([&](auto nb_) {
            if constexpr (decltype(nb_)::value + 1 < NB) step(F_{}, T_{}, F_{}, nb_, slot_c, 0, IntC<-1>{}, 0);
            else step(F_{}, T_{}, F_{}, nb_, slot_c, 0, IntC<STORE_AT>{}, (slot + 2) & (C::NBUF - 1));
        });
        asm volatile("s_waitcnt lgkmcnt(%0)\n\ts_barrier" ::"n"(READS_AFTER) : "memory");
    };
    int t = 0;
    const int last = ntiles - 1;
    int slot_rt = 0;
    while (true) {
        if (t >= last) { slot_rt = 0; break; }
        tile_body(IntC<0>{}); load_next(t + 3); ++t;
        if (t >= last) { slot_rt = 1; break; }
        tile_body(IntC<1>{}); load_next(t + 3); ++t;
        if (t >= last) { slot_rt = 2; break; }
        tile_body(IntC<2>{}); load_next(t + 3); ++t;
        if (t >= last) { slot_rt = 3; break; }
        tile_body(IntC<3>{}); load_next(t + 3); ++t;
    }

    // ---- last tile: rows >= n masked, its final block has no successor; then the output contractions
    // of that final block (a step that only drains).
    {
        const DynInt slot{slot_rt};
        static_for<0, NB>([&](auto nb_) {
            constexpr int nb = decltype(nb_)::value;
            const int srow0 = last * BN + nb * 32 + 4 * g;
            if constexpr (nb + 1 < NB) step(T_{}, T_{}, F_{}, nb_, slot, srow0, IntC<-1>{}, 0);
            else step(T_{}, F_{}, F_{}, nb_, slot, srow0, IntC<-1>{}, 0);
        });
        const DynInt slot_next{(slot_rt + 1) & (C::NBUF - 1)};
        step(F_{}, F_{}, T_{}, IntC<0>{}, slot_next, 0, IntC<-1>{}, 0);
    }


    if constexpr (WITH_DB) {
        // Row 0 of accdb (register 0 of lanes 0..15) holds 16 partial sums that together cover every dS of
        // this wave.  Owner rows beyond the valid length carry dO = 0, hence dS = 0.  Fixed-order sums: lanes
        // by butterfly, waves through LDS, workgroups in a second kernel.
        float v = 0.f;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) v += accdb[qb][0];
        v = (lane < 16) ? v : 0.f;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) s_db[wave] = v;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) t += s_db[w];
            p.db_part[blockIdx.x] = t * cb;                   // the summed values are dS / cb
            p.db_seq[blockIdx.x] = z;
        }
    }

    // ---- epilogue: transposed fp32 accumulators -> bf16 rows.  Lane (c, g) holds owner row c of each block;
    // registers 4 q4 .. 4 q4 + 3 of output block mb hold head-dim columns out_col(mb, q4) + 4 g + 0..3 of the
    // layout the transposed operand was read with (plain: 32 mb + 8 q4).  The two lanes of a row (32 apart)
    // exchange halves -- lane g = 0 takes the even q4, lane g = 1 the odd ones -- so that each lane stores
    // whole 16-byte chunks: a quarter of the store instructions and write requests of 8-byte stores.
    using TL_ACC0 = TrLayout<(MODE == FWD) ? C::LM2 : C::LM1>;      // FWD contracts V^T; DQ K^T; DKDV Q^T (acc0), dO^T (acc1)
    using TL_ACC1 = TrLayout<C::LM2>;
    const float oscale = (MODE == FWD) ? 1.0f : p.scale * cb;       // dQ and dK carry the factor `scale`; their sums are over dS / cb
    auto chunk = [&](const f32x16 &a, const int pr, const float f) {   // columns of q4 = 2 pr + g
        const unsigned e0 = pack_bf16(a[8 * pr + 0] * f, a[8 * pr + 1] * f), e1 = pack_bf16(a[8 * pr + 2] * f, a[8 * pr + 3] * f);
        const unsigned o0 = pack_bf16(a[8 * pr + 4] * f, a[8 * pr + 5] * f), o1 = pack_bf16(a[8 * pr + 6] * f, a[8 * pr + 7] * f);
        const auto s0 = __builtin_amdgcn_permlane32_swap(e0, o0, false, false);   // {lower half: e0 | o0 of g = 0, upper: of g = 1}
        const auto s1 = __builtin_amdgcn_permlane32_swap(e1, o1, false, false);
        const u32x4 w = {s0[0], s1[0], s0[1], s1[1]};
        return w;
    };
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int r = wrow0 + 32 * qb + c;
        const bool inside = r < p.N;                                 // both lanes of a row agree on these two
        const bool ok = r < n;                                       // padded owner rows are written as zero
        const size_t off = slice + (size_t)(inside ? r : 0) * row_stride + 8 * g;
        const u32x4 z4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                const u32x4 w0 = chunk(acc0[qb][mb], pr, oscale);
                if (inside) *reinterpret_cast<u32x4 *>(p.out0 + off + TL_ACC0::out_col(mb, 2 * pr)) = ok ? w0 : z4;
                if (MODE == DKDV) {
                    const u32x4 w1 = chunk(acc1[MODE == DKDV ? qb : 0][MODE == DKDV ? mb : 0], pr, 1.0f);
                    if (inside) *reinterpret_cast<u32x4 *>(p.out1 + off + TL_ACC1::out_col(mb, 2 * pr)) = ok ? w1 : z4;
                }
            }
        }
    }
}

// Second stage of the bias gradient: db[z] = sum of the partials of the workgroups of sequence z, in a
// fixed order (thread t takes workgroups t, t + 256, ...; then a tree in LDS), so the result is
// bitwise reproducible.  One workgroup per sequence.
__global__ void __launch_bounds__(256) sigattn_db_reduce(const float *part, const int32_t *seq, int nwg, float *db) {
    __shared__ float s[256];
    const int z = blockIdx.x;
    float t = 0.f;
    for (int i = threadIdx.x; i < nwg; i += 256) t += (seq[i] == z) ? part[i] : 0.f;
    s[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) db[z] = s[0];
}

}  // namespace sigattn
