// SoftmaxBalance (Alg. 2 of arXiv 2502.07861) on gfx950: Gram tiles on MFMA, kernel weights and
// the self-balancing walk on chip, strict halving, gather of the survivors.
//
// One workgroup (8 wavefronts) owns one block of b tokens; its keys are staged in LDS in chunks of as many 64-row
// panels as fit.  The walk is organised over 64-token panels.  sigma[l] (LDS) starts at minus the decision threshold
// of token l and accumulates sum_{i signed so far} eta_i g_il.  Wavefront 0 is the walker: for panel I it holds the
// strictly-upper part of the 64x64 diagonal tile of kernel weights as "one column per lane" registers and takes the 64
// sequential decisions of Alg. 2 (lane j tests the sign of its sigma; bit j of the compare mask becomes the +-1 that
// every later lane multiplies g_jl with).  Wavefronts 1..7 form tiles on MFMA while the walker walks.  There are no
// workgroup barriers inside the pipeline: the wavefronts hand data over through progress counters in LDS.
//
//   walker, panel I     take diagonal tile D(I) (registers), mark the buffer free, wait until column I is complete,
//                       take sigma of the panel, walk 64 steps, publish the signs of panel I
//   wave w = 1..7       owns column panel w (its keys stay in registers as the B operand): tiles (i, w), i = 0..w-1, in
//                       row order: weights first, then wait for the signs of panel i, signed column sum in a register;
//                       after tile (w-1, w) the sum goes into sigma[panel w] and column w is published.  Then the
//                       diagonal tile of panel w+2 (start-up tiles come from the wavefronts whose columns are due last),
//                       stored once the walker has taken the previous one.
//
// so the only work between two walks is one signed column sum and two hand-overs.  Rows of earlier chunks (b larger
// than one chunk) come back from global memory (L2) as the A operand against the resident chunk before its own panels
// are walked.
//
// Kernel weight: g_ij = exp((<k_i,k_j> - a_i - a_j + |mu|^2 - A)/sqrt(d) - ln c), a_i = <k_i,mu>
// (mu = block mean when keys are centred, else 0), A = r_key^2 or the largest centred squared norm:
// Alg. 2's y_i / (c R^2) with v = 1, never forming R^2.  The exponent is formed in one piece,
// alpha (<k_i,k_j> - a_i) + (rc - alpha a_j), alpha = log2(e)/sqrt(d), rc = alpha (|mu|^2 - A) - ln c log2(e): the row
// term -a_i is what the accumulators of the Gram start from (the C operand of the first MFMA of a tile), the column
// term is the addend of the one FMA in front of the exp2.  One FMA and one exp2 per entry, and no factor of the weight
// is ever formed on its own (a large common mean cannot overflow one factor and flush the other).
#include <utility>

#include "bkv_device.h"
#include "bkv_host.h"

namespace bkv {

template <typename T, int D> struct Geo {
    static constexpr int kRowBytes = D * (int)sizeof(T);
    static constexpr int kLdsRow = kRowBytes;               // rows are packed; 16-byte slices are permuted per row instead
    static constexpr int kGroups = kRowBytes / 32;          // k-groups of 32 bytes per row
    static constexpr int kSlices = kRowBytes / 16;          // 16-byte slices per row
    // Slice s of LDS row r is stored at slice position s ^ key(r).  Sixteen consecutive rows reading the same
    // logical slice (an MFMA operand fetch) then touch sixteen different groups of four banks, and so do the
    // slices of one row (staging, gathers): no padding bytes, no bank conflicts.  key(r) = key(r + 16).
    static __device__ __forceinline__ int key(int row) { return kRowBytes >= 256 ? (row & 15) : ((row >> 1) & (kSlices - 1)); }
    static __device__ __forceinline__ int slice_off(int row, int slice) { return (slice ^ key(row)) << 4; }
};

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kDiagStride = 68;                             // floats per column of the transposed diagonal tile (16-byte rows, conflict-free)
constexpr int kDiagFloats = 64 * kDiagStride;
constexpr int kLdsLimit = 160 * 1024;

static inline size_t lds_fixed_bytes(int b) {
    return (size_t)b * 4 * 2             // sigma, -a_i of every row
           + 16 * 8                      // eta of each panel as a 64-bit mask (bit j = 1 iff eta_j = +1)
           + 8 * 64 * 4                  // eta of the resident chunk's panels as +-1 floats, accumulator order
           + kDiagFloats * 4             // diagonal tile (also: mean partials, survivor list)
           + 64                          // scalars
           + 128;                        // progress counters of the panel pipeline
}
// rows of the block staged in LDS at a time: as many 64-row panels as fit, at most 8
// (with the value factor of Alg. 2 line 6 the value rows are staged next to the key rows: twice the bytes per row)
static inline int chunk_rows_for(int row_bytes, int b, bool value_gram = false) {
    const int rb = value_gram ? 2 * row_bytes : row_bytes;
    int rows = 512;
    while (rows > 64 && (size_t)rows * rb + lds_fixed_bytes(b) > (size_t)kLdsLimit) rows -= 64;
    return b < rows ? b : rows;
}

size_t compress_lds_bytes(int row_bytes, int b, bool value_gram) {
    return (size_t)chunk_rows_for(row_bytes, b, value_gram) * (value_gram ? 2 : 1) * row_bytes + lds_fixed_bytes(b);
}
// the value-factor variant keeps keys and values of the whole block in LDS
bool compress_value_gram_fits(int row_bytes, int b) { return chunk_rows_for(row_bytes, b, true) >= b; }
// does the launcher run such a block as one resident chunk (the instance without the multi-chunk code)?
bool compress_block_resident(int row_bytes, int b, bool value_gram) {
    const bool v_lds = value_gram && compress_value_gram_fits(row_bytes, b);
    return b <= chunk_rows_for(row_bytes, b, v_lds);
}

template <typename T, int D>
struct TileOps {
    typedef Geo<T, D> G;
    typedef typename Elem<T>::Frag Frag;

    // 64 rows starting at `base` (row stride in bytes) -> operand fragments of this lane.
    static __device__ __forceinline__ void load_frags(Frag (&F)[G::kGroups][2], const char* base,
                                                      int row_stride, int n, int h) {
#pragma unroll
        for (int g = 0; g < G::kGroups; ++g)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                F[g][rb] = *reinterpret_cast<const Frag*>(base + (size_t)(32 * rb + n) * row_stride + 32 * g + 16 * h);
    }

    // The same from 64 LDS rows (packed rows, permuted slices: foff[g] is this lane's byte offset of k-group g).
    static __device__ __forceinline__ void load_panel(Frag (&F)[G::kGroups][2], const char* lds_panel,
                                                      const int (&foff)[G::kGroups], int n) {
#pragma unroll
        for (int g = 0; g < G::kGroups; ++g)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                F[g][rb] = *reinterpret_cast<const Frag*>(lds_panel + (size_t)(32 * rb + n) * G::kLdsRow + foff[g]);
    }
    // Accumulator layout (32x32 MFMA): register r of lane (n,h) is row 8*(r/4) + 4*h + r%4, column n.

    // Signs of a row panel for the accumulator layout: entry 16*rb + r of lane half h belongs to row
    // 32*rb + 8*(r/4) + 4*h + r%4.  From the panel's mask (bit j = 1 iff eta_j = +1) ...
    static __device__ __forceinline__ void signs_from_mask(float (&sg)[32], unsigned long long m, int h) {
        const unsigned long long mh = ~m >> (4 * h);                  // bit set = '-'
        const unsigned int w[2] = {(unsigned int)mh, (unsigned int)(mh >> 32)};
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const int bit = 8 * ((k & 15) >> 2) + (k & 3);
            sg[k] = __uint_as_float(((w[k >> 4] << (31 - bit)) & 0x80000000u) | 0x3f800000u);   // +1 or -1
        }
    }
    // cs0 / cs1: per-lane partial sums for columns n / 32+n over this lane half's rows.  Returns, in lane (n, h), the
    // full sum of column 32*h + n: one half-wave swap (lanes 32..63 of cs0 <-> lanes 0..31 of cs1) and one add.
    static __device__ __forceinline__ float halves_sum(float cs0, float cs1) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(cs0), __float_as_uint(cs1), false, false);
        return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    // ... or as +-1 floats from LDS: this lane's 32 entries start at sgn_h = base + 32*h
    static __device__ __forceinline__ void signs_from_lds(float (&sg)[32], const float* sgn_h) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const floatx4 t = *reinterpret_cast<const floatx4*>(sgn_h + 4 * q);
            sg[4 * q] = t[0]; sg[4 * q + 1] = t[1]; sg[4 * q + 2] = t[2]; sg[4 * q + 3] = t[3];
        }
    }
    // sum over the 64 rows of sign * weight, per column; returns this lane's column 32*h + n (before the column factor)
    static __device__ __forceinline__ float signed_colsum(const floatx16 (&v)[2][2], const float (&sg)[32], int h) {
        float cs0 = 0.f, cs1 = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) cs0 = fmaf(sg[16 * rb + r], v[rb][0][r], cs0);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) cs1 = fmaf(sg[16 * rb + r], v[rb][1][r], cs1);
        return halves_sum(cs0, cs1);
    }
    // One 64x64 tile in two row halves: Gram of rows 0..31, then the Gram of rows 32..63 while the vector unit
    // turns the first half into kernel weights (acc <- exp2(alpha * acc + rc)) and, with SUM, adds them up
    // per column with the row signs; then the same for the second half.  Per MFMA (32 cycles in the matrix pipe)
    // the vector unit gets two elements: 2 FMA + 2 exp2 (+ 2 FMA); the order is written out and fenced, B fragments
    // are requested one k-group ahead.  A fragments come from registers (AREG: the caller's A, reused over several
    // tiles) or from LDS rows ldsA[0..63], one half at a time; signs come from registers (sg) or, if sg is null,
    // from LDS (sgn_h: this lane half's 32 floats).  naA / naB: -a_i of the tile's 64 rows / -a_j of its 64 columns.
    // Returns this lane's column 32*h + n of the signed column sums.
    // With BREG the column panel's fragments come from the caller's registers too (Bq), e.g. a panel that a
    // wavefront keeps for all tiles of its column.
    // With DIAG (a diagonal tile, not dumped) the quadrant rows 32..63 x columns 0..31, which the walk never uses, is skipped.
    // With VG the weights carry the value factor of Alg. 2 line 6: the Gram of the value rows of the same two panels
    // is formed first, scaled by 1 / r_value^2, and multiplies every weight after its exp2.  VG = 1: the value rows are
    // in LDS in the layout of the keys (vA: the 64 rows that match the tile's rows, vB: those that match its columns).
    // VG = 2: they are read from global memory; vA / vA1 are THIS LANE's rows n and n + 32 of the row panel, vB / vB1 of
    // the column panel.
    template <bool SUM, bool AREG, bool BREG = false, bool DIAG = false, int VG = 0>
    static __device__ __forceinline__ float tile(floatx16 (&acc)[2][2], const Frag (*A)[2], const char* ldsA, const char* ldsB,
                                                 const float* naA, const float* naB, float alpha, float rc, const float* sg, const float* sgn_h,
                                                 const int (&foff)[G::kGroups], int n, int h, const Frag (*Bq)[2] = nullptr,
                                                 const char* vA = nullptr, const char* vB = nullptr, float inv_rv2 = 0.f,
                                                 const char* vA1 = nullptr, const char* vB1 = nullptr, float vg_bias = 0.f) {
        constexpr int KG = G::kGroups;
        constexpr int RPI = 16 / KG;                       // accumulator registers (per column half) finished per k-group
        constexpr int kAhead = KG < 4 ? KG : 4;              // k-groups between the request of a B fragment and its use
        static_assert(RPI >= 1 && KG >= 4, "4 to 16 k-groups per row");
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        float cs0 = 0.f, cs1 = 0.f;
        floatx16 vg[2][2];                                   // value Gram / r_value^2 (VG only)
        if constexpr (VG != 0) {
            const char* va = VG == 1 ? vA + (size_t)n * G::kLdsRow : vA;
            const char* vb = VG == 1 ? vB + (size_t)n * G::kLdsRow : vB;
            const char* va1 = VG == 1 ? va + (size_t)32 * G::kLdsRow : vA1;
            const char* vb1 = VG == 1 ? vb + (size_t)32 * G::kLdsRow : vB1;
            vg[0][0] = zero; vg[0][1] = zero; vg[1][0] = zero; vg[1][1] = zero;
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                const int off = VG == 1 ? foff[g] : 32 * g + 16 * h;
                const Frag a0 = *reinterpret_cast<const Frag*>(va + off);
                const Frag a1 = *reinterpret_cast<const Frag*>(va1 + off);
                const Frag b0 = *reinterpret_cast<const Frag*>(vb + off);
                const Frag b1 = *reinterpret_cast<const Frag*>(vb1 + off);
                Elem<T>::mma(vg[0][0], a0, b0);
                Elem<T>::mma(vg[0][1], a0, b1);
                if (!DIAG) Elem<T>::mma(vg[1][0], a1, b0);
                Elem<T>::mma(vg[1][1], a1, b1);
            }
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) vg[rb][cb][r] = fmaf(vg[rb][cb][r], inv_rv2, vg_bias);
            __builtin_amdgcn_sched_barrier(0);
        }
        const char* bp0 = BREG ? nullptr : ldsB + (size_t)n * G::kLdsRow;
        const char* bp1 = BREG ? nullptr : bp0 + (size_t)32 * G::kLdsRow;
        const char* ap = AREG ? nullptr : ldsA + (size_t)n * G::kLdsRow;
        Frag Ah[2][KG], B0[KG], B1[KG];
        floatx4 sq[2][4];
        // -a_i of this lane's 16 rows of each half, in accumulator order: where the Gram's accumulators start from
        floatx16 rinit[2];
        auto load_rinit = [&](int rb) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 t = *reinterpret_cast<const floatx4*>(naA + 32 * rb + 8 * q + 4 * h);
                rinit[rb][4 * q] = t[0]; rinit[rb][4 * q + 1] = t[1]; rinit[rb][4 * q + 2] = t[2]; rinit[rb][4 * q + 3] = t[3];
            }
        };
        // the column term of this lane's two columns: rc - alpha a_j
        const float cc0 = fmaf(alpha, naB[n], rc), cc1 = fmaf(alpha, naB[32 + n], rc);
        auto load_a = [&](int rb, int g) {
            Ah[rb][g] = AREG ? A[g][rb] : *reinterpret_cast<const Frag*>(ap + (size_t)(32 * rb) * G::kLdsRow + foff[g]);
        };
        auto load_b = [&](int g) {
            if (BREG) { B0[g] = Bq[g][0]; B1[g] = Bq[g][1]; return; }
            B0[g] = *reinterpret_cast<const Frag*>(bp0 + foff[g]);
            B1[g] = *reinterpret_cast<const Frag*>(bp1 + foff[g]);
        };
        auto load_rowterm = [&](int rb, int q) {
            if (SUM) {
                if (sg) { sq[rb][q][0] = sg[16 * rb + 4 * q]; sq[rb][q][1] = sg[16 * rb + 4 * q + 1]; sq[rb][q][2] = sg[16 * rb + 4 * q + 2]; sq[rb][q][3] = sg[16 * rb + 4 * q + 3]; }
                else sq[rb][q] = *reinterpret_cast<const floatx4*>(sgn_h + 16 * rb + 4 * q);
            }
        };
        auto finish = [&](int rb, int r) {
            if (!(DIAG && rb == 1)) acc[rb][0][r] = fast_exp2(fmaf(acc[rb][0][r], alpha, cc0));
            acc[rb][1][r] = fast_exp2(fmaf(acc[rb][1][r], alpha, cc1));
            if constexpr (VG != 0) {
                if (!(DIAG && rb == 1)) acc[rb][0][r] *= vg[rb][0][r];
                acc[rb][1][r] *= vg[rb][1][r];
            }
            if (SUM) {
                cs0 = fmaf(sq[rb][r >> 2][r & 3], acc[rb][0][r], cs0);
                cs1 = fmaf(sq[rb][r >> 2][r & 3], acc[rb][1][r], cs1);
            }
        };
        // the same for registers r0 .. r0+RPI-1, one kind of instruction at a time (dependent instructions kept apart)
        auto finish_group = [&](int rb, int r0, int step) {
#pragma unroll
            for (int r = r0; r < r0 + RPI; ++r) {
                if (step == 0) {
                    acc[rb][0][r] = fmaf(acc[rb][0][r], alpha, cc0);
                    acc[rb][1][r] = fmaf(acc[rb][1][r], alpha, cc1);
                } else if (step == 1) {
                    acc[rb][0][r] = fast_exp2(acc[rb][0][r]);
                    acc[rb][1][r] = fast_exp2(acc[rb][1][r]);
                    if constexpr (VG != 0) { acc[rb][0][r] *= vg[rb][0][r]; acc[rb][1][r] *= vg[rb][1][r]; }
                } else if (SUM) {
                    cs0 = fmaf(sq[rb][r >> 2][r & 3], acc[rb][0][r], cs0);
                    cs1 = fmaf(sq[rb][r >> 2][r & 3], acc[rb][1][r], cs1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // rows 0..31 on the matrix pipe; requests for what the next stage needs ride along
#pragma unroll
        for (int g = 0; g < KG; ++g) load_a(0, g);
#pragma unroll
        for (int g = 0; g < kAhead; ++g) load_b(g);
        load_rinit(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            if (g + kAhead < KG) load_b(g + kAhead);
            if (g < 4) load_rowterm(0, g);
            if (g == 0) load_rinit(1);
            if (!AREG) load_a(1, g);
            if (g == 0) {                                  // both accumulators start from -a_i of their rows
                acc[0][0] = Elem<T>::mma_from(Ah[0][0], B0[0], rinit[0]);
                acc[0][1] = Elem<T>::mma_from(Ah[0][0], B1[0], rinit[0]);
            } else {
                Elem<T>::mma(acc[0][0], Ah[0][g], B0[g]);
                Elem<T>::mma(acc[0][1], Ah[0][g], B1[g]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // rows 32..63 on the matrix pipe, rows 0..31 on the vector unit
        if (AREG)
#pragma unroll
            for (int g = 0; g < KG; ++g) load_a(1, g);
        constexpr bool kKeepB = BREG || KG <= 8;           // up to 64 registers: the B fragments of the first half stay
        if (!kKeepB)
#pragma unroll
            for (int g = 0; g < kAhead; ++g) load_b(g);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            if (!kKeepB && g + kAhead < KG) load_b(g + kAhead);
            if (g >= KG - 4) load_rowterm(1, g - (KG - 4));
            if (g == 0) { if (!DIAG) acc[1][0] = Elem<T>::mma_from(Ah[1][0], B0[0], rinit[1]); }
            else if (!DIAG) Elem<T>::mma(acc[1][0], Ah[1][g], B0[g]);
            finish_group(0, g * RPI, 0);                   // scale-and-shift of this k-group's share of rows 0..31 ...
            if (g == 0) acc[1][1] = Elem<T>::mma_from(Ah[1][0], B1[0], rinit[1]);
            else Elem<T>::mma(acc[1][1], Ah[1][g], B1[g]);
            finish_group(0, g * RPI, 1);                   // ... their exponentials ...
            finish_group(0, g * RPI, 2);                   // ... and the signed sums
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) finish(1, r);
        if (!SUM) return 0.f;
        return halves_sum(cs0, cs1);
    }
    // One row panel (A in registers, signs in registers) against nJ consecutive 64-row column panels in LDS,
    // software-pipelined over half tiles: while the matrix pipe forms rows 0..31 of the next tile the vector unit
    // finishes rows 32..63 of the current one, and vice versa, so that neither unit waits for the other even when
    // two wavefronts share a SIMD.  emit(jj, cs) receives this lane's column 32*h + n of tile jj's signed column sums.
    template <typename Emit>
    static __device__ __forceinline__ void row_sweep(const Frag (&A)[G::kGroups][2], const char* ldsB, int nJ,
                                                     const float* naA, const float* naB, float alpha, float rc, unsigned long long eta_mask,
                                                     const int (&foff)[G::kGroups], int n, int h, Emit emit) {
        constexpr int KG = G::kGroups;
        constexpr int RPI = 16 / KG;
        constexpr int kAhead = KG < 3 ? KG : 3;
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        floatx16 acc[2][2];
        float cs0 = 0.f, cs1 = 0.f;
        // signs are formed where they are used (two cheap instructions per row) rather than held in 32 registers:
        // bit 8*(r/4) + r%4 of word rb is set iff the row of accumulator register r, row half rb, has eta = -1
        const unsigned long long mh = ~eta_mask >> (4 * h);
        const unsigned int nbw[2] = {(unsigned int)mh, (unsigned int)(mh >> 32)};
        auto sign_of = [&](int rb, int r) -> float {
            return __uint_as_float(((nbw[rb] << (31 - (8 * (r >> 2) + (r & 3)))) & 0x80000000u) | 0x3f800000u);
        };
        const char* bp0 = ldsB + (size_t)n * G::kLdsRow;
        Frag B0[KG], B1[KG];
        // -a_i of the row panel is where the accumulators start from (fetched anew for every half tile: 16 registers in
        // flight instead of 32 held), -a_j of the column panel at hand makes the FMA's addend (naB moves with bp0)
        float cc0 = 0.f, cc1 = 0.f;                      // rc - alpha a_j of this lane's two columns of the tile being finished
        auto load_b = [&](int g) {
            B0[g] = *reinterpret_cast<const Frag*>(bp0 + foff[g]);
            B1[g] = *reinterpret_cast<const Frag*>(bp0 + (size_t)32 * G::kLdsRow + foff[g]);
        };
        floatx16 rinit;
        auto load_rinit = [&](int rb) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 t = *reinterpret_cast<const floatx4*>(naA + 32 * rb + 8 * q + 4 * h);
                rinit[4 * q] = t[0]; rinit[4 * q + 1] = t[1]; rinit[4 * q + 2] = t[2]; rinit[4 * q + 3] = t[3];
            }
        };
        auto finish = [&](int rb, int r) {
            acc[rb][0][r] = fast_exp2(fmaf(acc[rb][0][r], alpha, cc0));
            acc[rb][1][r] = fast_exp2(fmaf(acc[rb][1][r], alpha, cc1));
            const float sr = sign_of(rb, r);
            cs0 = fmaf(sr, acc[rb][0][r], cs0);
            cs1 = fmaf(sr, acc[rb][1][r], cs1);
        };
        auto finish_group = [&](int rb, int r0, int step) {
#pragma unroll
            for (int r = r0; r < r0 + RPI; ++r) {
                if (step == 0) {
                    acc[rb][0][r] = fmaf(acc[rb][0][r], alpha, cc0);
                    acc[rb][1][r] = fmaf(acc[rb][1][r], alpha, cc1);
                } else if (step == 1) {
                    acc[rb][0][r] = fast_exp2(acc[rb][0][r]);
                    acc[rb][1][r] = fast_exp2(acc[rb][1][r]);
                } else {
                    const float sr = sign_of(rb, r);
                    cs0 = fmaf(sr, acc[rb][0][r], cs0);
                    cs1 = fmaf(sr, acc[rb][1][r], cs1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // the MFMAs of row half RBM of the tile at bp0; with FIN, the other half (of the previous product) is finished alongside
        auto stage = [&](auto rbm_c, auto fin_c) {
            constexpr int RBM = decltype(rbm_c)::value;
            constexpr bool FIN = decltype(fin_c)::value;
#pragma unroll
            for (int g = 0; g < kAhead; ++g) load_b(g);
            load_rinit(RBM);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                if (g + kAhead < KG) load_b(g + kAhead);
                if (g == 0) acc[RBM][0] = Elem<T>::mma_from(A[0][RBM], B0[0], rinit);
                else Elem<T>::mma(acc[RBM][0], A[g][RBM], B0[g]);
                if (FIN) finish_group(1 - RBM, g * RPI, 0);
                if (g == 0) acc[RBM][1] = Elem<T>::mma_from(A[0][RBM], B1[0], rinit);
                else Elem<T>::mma(acc[RBM][1], A[g][RBM], B1[g]);
                if (FIN) { finish_group(1 - RBM, g * RPI, 1); finish_group(1 - RBM, g * RPI, 2); }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        stage(std::integral_constant<int, 0>{}, std::false_type{});
#pragma unroll 1
        for (int jj = 0; jj < nJ; ++jj) {
            cs0 = 0.f; cs1 = 0.f;
            cc0 = fmaf(alpha, naB[(jj << 6) + n], rc); cc1 = fmaf(alpha, naB[(jj << 6) + 32 + n], rc);
            stage(std::integral_constant<int, 1>{}, std::true_type{});         // rows 32..63 of tile jj | finish rows 0..31
            if (jj + 1 < nJ) {
                bp0 += (size_t)64 * G::kLdsRow;
                stage(std::integral_constant<int, 0>{}, std::true_type{});     // rows 0..31 of tile jj+1 | finish rows 32..63
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) finish(1, r);
            }
            emit(jj, halves_sum(cs0, cs1));
        }
    }
    // Diagonal tile: zero everything that is not strictly above the diagonal
    // (the walk only ever adds eta_j * g_jl for l > j) ...
    // Quadrant by quadrant: rows 0..31 x columns 32..63 lie above the diagonal as a whole, rows 32..63 x columns
    // 0..31 below it as a whole; only the two diagonal quadrants need the per-entry test (local row < n in both).
    static __device__ __forceinline__ void mask_diag(floatx16 (&v)[2][2], int n, int h) {
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lrow = 8 * (r >> 2) + 4 * h + (r & 3);                  // row inside its half
            v[0][0][r] = (n > lrow) ? v[0][0][r] : 0.f;
            v[1][1][r] = (n > lrow) ? v[1][1][r] : 0.f;
        }
        v[1][0] = zero;
    }
    // ... and store it transposed, diag[col * kDiagStride + row]: four consecutive rows per 16-byte store.
    static __device__ __forceinline__ void store_diag(float* diag, const floatx16 (&v)[2][2], int n, int h) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    floatx4 t = {v[rb][cb][4 * q], v[rb][cb][4 * q + 1], v[rb][cb][4 * q + 2], v[rb][cb][4 * q + 3]};
                    *reinterpret_cast<floatx4*>(diag + (32 * cb + n) * kDiagStride + 32 * rb + 8 * q + 4 * h) = t;
                }
    }
    // One 32x32 quadrant (rows 32 QR.., columns 32 QC..) of a diagonal tile, from the panel's rows in LDS straight to
    // the transposed tile buffer: the same arithmetic, in the same order, as tile<DIAG> + mask_diag + store_diag give
    // that quadrant.  Three wavefronts on three SIMDs form the first tile of a chunk this way, so that the walk starts
    // after a third of the time one wavefront needs for the whole tile.  QR = QC = 0 also clears the quadrant below
    // the diagonal.
    template <int QR, int QC>
    static __device__ __forceinline__ void diag_quadrant(float* diag, const char* lds_panel, const float* naP, float alpha,
                                                         float rc, const int (&foff)[G::kGroups], int n, int h) {
        static_assert(QR <= QC, "quadrants on or above the diagonal");
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const char* ap = lds_panel + (size_t)(32 * QR + n) * G::kLdsRow;
        const char* bp = lds_panel + (size_t)(32 * QC + n) * G::kLdsRow;
        Frag A[G::kGroups], B[G::kGroups];
#pragma unroll
        for (int g = 0; g < G::kGroups; ++g) {
            A[g] = *reinterpret_cast<const Frag*>(ap + foff[g]);
            B[g] = *reinterpret_cast<const Frag*>(bp + foff[g]);
        }
        floatx16 acc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const floatx4 t = *reinterpret_cast<const floatx4*>(naP + 32 * QR + 8 * q + 4 * h);
            acc[4 * q] = t[0]; acc[4 * q + 1] = t[1]; acc[4 * q + 2] = t[2]; acc[4 * q + 3] = t[3];
        }
        const float cc = fmaf(alpha, naP[32 * QC + n], rc);
#pragma unroll
        for (int g = 0; g < G::kGroups; ++g) Elem<T>::mma(acc, A[g], B[g]);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lrow = 8 * (r >> 2) + 4 * h + (r & 3);
            const float w = fast_exp2(fmaf(acc[r], alpha, cc));
            acc[r] = (QR != QC || n > lrow) ? w : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const floatx4 t = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
            *reinterpret_cast<floatx4*>(diag + (32 * QC + n) * kDiagStride + 32 * QR + 8 * q + 4 * h) = t;
            if (QR == 0 && QC == 0) {
                const floatx4 z = {0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<floatx4*>(diag + n * kDiagStride + 32 + 8 * q + 4 * h) = z;
            }
        }
    }
};

// One decision of the walk (Alg. 2 lines 6-9 for token j of the panel).  Every lane tests the sign of its sigma
// (which carries the threshold, see the kernel); the compare mask is then read back as data by the vector unit:
// bit j of it, sign-extended, becomes the -1/+1 that multiplies row j of the diagonal tile.  No scalar-unit hop
// on the chain: four dependent vector instructions per step.  A vector instruction that reads a scalar register
// written by the vector instruction just before it needs two wait states on this hardware, hence the s_nop.
// Lanes <= j hold g[j] = 0, so their sigma stays at its decision-time value.
// Eight consecutive steps per asm statement, so that nothing is scheduled into the chain.
template <int B>
__device__ __forceinline__ void walk_steps8(float& sv, const float (&g)[64], unsigned int sign_bit) {
    int t;
    if constexpr (B < 32)
        asm volatile("v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %11, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %3\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %12, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %4\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %13, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %5\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %14, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %6\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %15, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %7\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %16, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %8\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %17, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %9\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_lo, %18, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %10"
                     : "+v"(sv), "=&v"(t)
                     : "s"(sign_bit), "v"(g[B]), "v"(g[B + 1]), "v"(g[B + 2]), "v"(g[B + 3]), "v"(g[B + 4]), "v"(g[B + 5]), "v"(g[B + 6]), "v"(g[B + 7]),
                       "n"(B), "n"(B + 1), "n"(B + 2), "n"(B + 3), "n"(B + 4), "n"(B + 5), "n"(B + 6), "n"(B + 7)
                     : "vcc");
    else
        asm volatile("v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %11, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %3\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %12, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %4\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %13, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %5\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %14, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %6\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %15, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %7\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %16, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %8\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %17, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %9\n\t"
                     "v_cmp_le_f32 vcc, 0, %0\n\ts_nop 1\n\tv_bfe_i32 %1, vcc_hi, %18, 1\n\tv_and_or_b32 %1, %1, %2, 1.0\n\tv_fmac_f32 %0, %1, %10"
                     : "+v"(sv), "=&v"(t)
                     : "s"(sign_bit), "v"(g[B]), "v"(g[B + 1]), "v"(g[B + 2]), "v"(g[B + 3]), "v"(g[B + 4]), "v"(g[B + 5]), "v"(g[B + 6]), "v"(g[B + 7]),
                       "n"(B - 32), "n"(B - 31), "n"(B - 30), "n"(B - 29), "n"(B - 28), "n"(B - 27), "n"(B - 26), "n"(B - 25)
                     : "vcc");
    // per step: sigma >= 0 -> bit set, factor -1 (eta = -1); sigma < 0 -> factor +1
}
__device__ __forceinline__ void walk_panel(float& sv, const float (&g)[64], unsigned int sign_bit) {
    walk_steps8<0>(sv, g, sign_bit);  walk_steps8<8>(sv, g, sign_bit);  walk_steps8<16>(sv, g, sign_bit); walk_steps8<24>(sv, g, sign_bit);
    walk_steps8<32>(sv, g, sign_bit); walk_steps8<40>(sv, g, sign_bit); walk_steps8<48>(sv, g, sign_bit); walk_steps8<56>(sv, g, sign_bit);
}

// Progress counters in LDS (one writer each, values only grow): a wavefront publishes with a release store and
// waits with a bounded poll.  Every wait is for an event that only depends on earlier events of the same block, and
// all eight wavefronts are resident, so the polls end; the bound turns a logic error into a status bit instead of
// a hang.
constexpr int kSpinLimit = 1 << 16;
// The fences name LDS only: a wavefront with global loads or stores in flight (look-ahead touches, dumps) must
// not wait for them here.
__device__ __forceinline__ void publish(int* counter, int value) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __hip_atomic_store(counter, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// The same for a hand-over on the walk's critical path, where counter and data are both in LDS and were written by
// this wavefront just before: LDS serves a wavefront's requests in order, so the counter cannot become visible before
// the data, and the wavefront need not wait for its own stores to finish first.  (The fence only keeps the compiler
// from moving the stores.)
__device__ __forceinline__ void publish_in_order(int* counter, int value) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __hip_atomic_store(counter, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
template <bool EAGER = false>
__device__ __forceinline__ void await(int* counter, int value, int* err) {
    for (int it = 0; it < kSpinLimit; ++it) {
        const int seen = __builtin_amdgcn_readfirstlane(__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
        if (seen >= value) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            return;
        }
        if (!EAGER) __builtin_amdgcn_s_sleep(1);          // waits on the walk's critical path poll back to back
    }
    __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// The walker's hand-overs: a counter and the data it guards are requested in one batch, counter first.  LDS serves a
// wavefront's requests in order, so data that arrives with a counter value >= the awaited one is current; this saves
// one LDS round trip per hand-over compared to "poll, then read".
__device__ __forceinline__ unsigned int lds_offset(const void* p) {
    return (unsigned int)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// the walker's column of the diagonal tile (16 x 16 bytes) once `counter` >= value
__device__ __forceinline__ void await_and_read_tile(int* counter, int value, const float* tile_col, float (&g)[64], int* err) {
    const unsigned int a0 = lds_offset(counter), a2 = lds_offset(tile_col);
    floatx4 q0, q1, q2, q3, q4, q5, q6, q7, q8, q9, q10, q11, q12, q13, q14, q15;
    bool ok = false;
    for (int it = 0; it < kSpinLimit && !ok; ++it) {
        int s0;
        asm volatile("ds_read_b32 %0, %17\n\t"
                     "ds_read_b128 %1, %18\n\tds_read_b128 %2, %18 offset:16\n\tds_read_b128 %3, %18 offset:32\n\tds_read_b128 %4, %18 offset:48\n\t"
                     "ds_read_b128 %5, %18 offset:64\n\tds_read_b128 %6, %18 offset:80\n\tds_read_b128 %7, %18 offset:96\n\tds_read_b128 %8, %18 offset:112\n\t"
                     "ds_read_b128 %9, %18 offset:128\n\tds_read_b128 %10, %18 offset:144\n\tds_read_b128 %11, %18 offset:160\n\tds_read_b128 %12, %18 offset:176\n\t"
                     "ds_read_b128 %13, %18 offset:192\n\tds_read_b128 %14, %18 offset:208\n\tds_read_b128 %15, %18 offset:224\n\tds_read_b128 %16, %18 offset:240\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(s0), "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3), "=&v"(q4), "=&v"(q5), "=&v"(q6), "=&v"(q7),
                       "=&v"(q8), "=&v"(q9), "=&v"(q10), "=&v"(q11), "=&v"(q12), "=&v"(q13), "=&v"(q14), "=&v"(q15)
                     : "v"(a0), "v"(a2) : "memory");
        ok = __builtin_amdgcn_readfirstlane(s0) >= value;
    }
    if (!ok) __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    const floatx4 q[16] = {q0, q1, q2, q3, q4, q5, q6, q7, q8, q9, q10, q11, q12, q13, q14, q15};
#pragma unroll
    for (int t = 0; t < 16; ++t) { g[4 * t] = q[t][0]; g[4 * t + 1] = q[t][1]; g[4 * t + 2] = q[t][2]; g[4 * t + 3] = q[t][3]; }
}
// one float once `counter` >= value
__device__ __forceinline__ float await_and_read(int* counter, int value, const float* data, int* err) {
    const unsigned int ca = lds_offset(counter), da = lds_offset(data);
    float x = 0.f;
    for (int it = 0; it < kSpinLimit; ++it) {
        int seen;
        asm volatile("ds_read_b32 %0, %2\n\tds_read_b32 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(seen), "=&v"(x) : "v"(ca), "v"(da) : "memory");
        if (__builtin_amdgcn_readfirstlane(seen) >= value) return x;
    }
    __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return x;
}

// MULTI = false: the launcher guarantees b <= chunk_rows (the block is resident in LDS as one chunk), and the
// multi-chunk code is compiled out.
// VG != 0: the kernel weights carry the value factor <v_i,v_j> / r_value^2 of Alg. 2 line 6.  VG = 1 (resident blocks
// whose values fit LDS too): the block's value rows are staged in LDS behind the key rows.  VG = 2 (any block): the
// value panels of every tile are read from global memory (L2) as they are needed.
template <typename T, int D, bool EMIT_G, bool MULTI, int VG = 0>
__global__ __launch_bounds__(kThreads) void compress_kernel(const CompressArgs a) {
    static_assert(VG == 0 || !EMIT_G, "the weight dump has no values");
    static_assert(VG != 1 || !MULTI, "values in LDS: resident blocks only");
    typedef Geo<T, D> G;
    typedef TileOps<T, D> Ops;
    typedef typename Elem<T>::Frag Frag;
    constexpr int EPL = Elem<T>::kPerFrag;
    constexpr int SL = G::kSlices;
    constexpr int RG = kThreads / SL;          // row groups: rows handled concurrently by the workgroup
    constexpr int GPW = 64 / SL;               // row groups per wavefront

    extern __shared__ __align__(16) char smem[];
    const int b = a.b, nP = b >> 6, CH = a.chunk_rows;
    char* ldsK = smem;
    char* ldsV = smem + (size_t)CH * G::kLdsRow;                   // value rows, same layout as the keys (VG only)
    float* sigma = reinterpret_cast<float*>(smem + (size_t)(VG == 1 ? 2 : 1) * CH * G::kLdsRow);
    float* narow = sigma + b;                                      // -a_i of every row (a_i = <k_i, mu>)
    unsigned long long* etaMask = reinterpret_cast<unsigned long long*>(narow + b);   // bit j of entry I: eta of token 64 I + j is +1
    float* etaF = reinterpret_cast<float*>(etaMask + 16);          // [8][2][32]: +-1 of the chunk's panel l, entry h*32 + 16*rb + r
    float* diag = etaF + 512;                                      // [64 columns][kDiagStride], transposed
    float* scal = diag + kDiagFloats;                              // [0] |mu|^2, [1] A, [2..2+kWaves) partial maxima
    int* prog = reinterpret_cast<int*>(scal + 16);                 // progress counters, see the panel pipeline below
    float* wpart = diag;                                           // [kWaves][D] column sums (statistics phase only)
    int* keptIdx = reinterpret_cast<int*>(diag);                   // [b/2]        (output phase only)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: roles branch on scalars
    const int n = lane & 31, h = lane >> 5;
    const int64_t inst = blockIdx.x;
    int64_t seq = inst / a.blocks_per_seq;
    const int blk = (int)(inst - seq * a.blocks_per_seq);
    int64_t in_tok0 = seq * a.in_seq_stride + (int64_t)blk * b;                // first input token
    int64_t out_tok0 = seq * a.out_seq_stride + (int64_t)blk * (b / 2);        // first output token
    int64_t idx_out0 = seq * a.idx_out_seq_stride + (int64_t)blk * (b / 2);    // first entry of idx_out
    int64_t signs0 = inst * b;                                                 // first entry of signs_out
    // generator stream and first counter of this instance
    uint64_t stream = a.tree_mode ? (uint64_t)(64 * (a.seq_base + seq) + a.round) : (uint64_t)inst;
    if (a.inst_ids) stream = a.inst_ids[inst];
    uint64_t ctr0 = a.tree_mode ? (uint64_t)(a.blk_base + blk) * (uint64_t)b : 0ull;
    float rvalue2 = a.rvalue2;
    if (a.desc) {                               // ragged launches: every coordinate of the instance comes from a table
        const InstDesc ds = a.desc[inst];
        if (!ds.valid) return;                  // the grid is an upper bound; uniform for the workgroup, before any barrier
        seq = ds.seq; in_tok0 = ds.in_tok; out_tok0 = ds.out_tok; idx_out0 = ds.out_tok; signs0 = ds.in_tok;
        stream = ds.stream; ctr0 = ds.ctr0;
        if (ds.rvalue2 > 0.f) rvalue2 = ds.rvalue2;
    }
    const char* Kin = a.K + in_tok0 * G::kRowBytes;
    // without idx_in a token's index within its sequence is its place in the input: by block number, or (ragged
    // launches, keys and values stored side by side) the instance's first token less the start of its sequence
    const int64_t tok_base = a.desc ? in_tok0 - seq * a.v_seq_stride : a.idx_base + (int64_t)blk * b;
    const int sl = tid % SL, rg = tid / SL;
    const bool center = (a.flags & BKV_CENTER_KEYS) != 0;
    const bool need_norm = !(a.rkey2 > 0.f);
    const bool single_chunk = MULTI ? (CH == b) : true;
    const float alpha = a.alpha;
    float* Gi = EMIT_G ? a.G_out + (size_t)inst * b * b : nullptr;

    // Every block of a launch takes the same time, so compute units that start together stay in lockstep and
    // would all hit HBM in the same phases.  The first wave of workgroups therefore starts spread over a good part
    // of one block's duration (a bounded wait on the clock; the launcher sets the step); later workgroups inherit the offsets.
    if (a.stagger_step > 0 && (int)blockIdx.x < a.stagger_blocks) {
        const long long wait = (long long)a.stagger_step * (long long)blockIdx.x;
        const long long t0 = __builtin_amdgcn_s_memtime();
        while (__builtin_amdgcn_s_memtime() - t0 < wait) __builtin_amdgcn_s_sleep(32);
    }

    const uint64_t key = stream_key(a.seed, stream);

    // decision threshold of token i: eta_i = +1 <=> u_i < 1/2 - s_i/2 <=> s_i < 1 - 2 u_i (exact in fp32)
    auto threshold = [&](int i) -> float {
        float u;
        if (a.uniforms) u = a.uniforms[(size_t)inst * b + i];
        else u = (float)draw_bits_keyed(key, ctr0 + (uint64_t)i) * (1.0f / 16777216.0f);
        return 1.f - 2.f * u;
    };

    // First byte of LDS row `r` of the resident chunk.  The row number passes through an empty asm so that the
    // compiler forms tile addresses where they are used (scalar base + per-lane fragment offset) instead of
    // carrying one induction register per fragment across the panel loops.
    auto lds_rows = [&](int r) -> const char* {
        asm volatile("" : "+s"(r));
        return ldsK + (size_t)r * G::kLdsRow;
    };

    // sigma starts at minus the threshold: the walk tests (sum of signed weights - threshold) < 0.  Integer work,
    // done first so that it overlaps the latency of the loads below.
    for (int i = tid; i < b; i += kThreads) sigma[i] = 0.f - threshold(i);      // never -0: the sign bit alone decides

    // column sums for the block mean, accumulated while rows pass through the registers
    float part[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) part[e] = 0.f;

    const int n_chunks = MULTI ? (b + CH - 1) / CH : 1;
    // Rows [row0, row0 + rows_here) of the block -> LDS, many rows in flight per thread; the first rows_sum rows
    // from row0 (possibly more than are staged) also enter the column sums of the mean.
    auto stage_chunk = [&](int row0, int rows_here, int rows_sum) {
        constexpr int U = 16;
        const int rows_all = max(rows_here, rows_sum);
        for (int i0 = rg; i0 < rows_all; i0 += RG * U) {
            uintx4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * RG;
                if (i < rows_all) {
                    const char* src = Kin + (size_t)(row0 + i) * G::kRowBytes;
                    if (!MULTI && a.k_by_idx)      // ragged first round: the block's rows lie scattered in the original tensor
                        src = a.K + ((size_t)seq * a.v_seq_stride + (size_t)a.idx_in[in_tok0 + row0 + i]) * G::kRowBytes;
                    raw[u] = *reinterpret_cast<const uintx4*>(src + sl * 16);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * RG;
                if (i < rows_here) *reinterpret_cast<uintx4*>(ldsK + (size_t)i * G::kLdsRow + G::slice_off(i, sl)) = raw[u];
                if (i < rows_sum) Elem<T>::accumulate(part, raw[u]);
            }
        }
    };
    // Blocks of several chunks, where registers allow: the whole block is requested in one batch (32 slices per thread),
    // and the slices of the rows beyond the first chunk stay in registers until the second statistics pass has used
    // them, so that those rows are read once here and once when their chunk is staged.
    constexpr int kU2 = 32;                                     // slices in flight per thread in the first pass
    constexpr int kCHm = G::kRowBytes <= 256 ? 512 : 256;       // chunk rows of a block that does not fit LDS
    constexpr int kU0 = kCHm / RG;                              // slices of a thread that belong to the first chunk
    constexpr int kUK = kU2 > kU0 ? (kU2 - kU0 < 16 ? kU2 - kU0 : 16) : 1;
    uintx4 keep[MULTI ? kUK : 1];
    bool kept = false;
    if constexpr (MULTI) {
        kept = CH == kCHm && b > CH && b <= RG * kU2 && b - CH <= RG * kUK && kU2 > kU0 && (center || need_norm);
    }
    if (MULTI && kept) {
        uintx4 raw[kU2];
#pragma unroll
        for (int u = 0; u < kU2; ++u) {
            const int i = rg + u * RG;
            if (i < b) raw[u] = *reinterpret_cast<const uintx4*>(Kin + (size_t)i * G::kRowBytes + sl * 16);
            else raw[u] = uintx4{0u, 0u, 0u, 0u};                // (rows past the block's end: defined, never counted)
        }
#pragma unroll
        for (int u = 0; u < kU2; ++u) {
            const int i = rg + u * RG;
            if (u < kU0) *reinterpret_cast<uintx4*>(ldsK + (size_t)i * G::kLdsRow + G::slice_off(i, sl)) = raw[u];    // i < CH <= b
            else if (u - kU0 < kUK) keep[u - kU0 < kUK ? u - kU0 : 0] = raw[u];
            if (center && i < b) Elem<T>::accumulate(part, raw[u]);
        }
    } else {
        stage_chunk(0, min(CH, b), center ? b : 0);
    }
    // Value factor: the value row of every token of the block -> LDS (the row of token i is the ORIGINAL row of that
    // token, as in the gather at the end); |v_i|^2 on the way when r_value has to be measured.
    float vmax = 0.f;
    // this lane's value row of token i of the block (VG = 2: the operand fetches go through these)
    const char* Vseq = VG != 0 ? a.V + (size_t)seq * a.v_seq_stride * G::kRowBytes : nullptr;
    auto vrow = [&](int i) -> const char* {
        const int64_t tok = a.idx_in ? (int64_t)a.idx_in[in_tok0 + i] : tok_base + i;
        return Vseq + (size_t)tok * G::kRowBytes;
    };
    if (VG == 1 || (VG == 2 && !(rvalue2 > 0.f))) {      // VG = 2 with a given radius: nothing to do here
        constexpr int U = 16;
        for (int i0 = rg; i0 < b; i0 += RG * U) {
            uintx4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * RG;
                if (i < b) raw[u] = *reinterpret_cast<const uintx4*>(vrow(i) + sl * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * RG;
                if (i < b) {
                    if constexpr (VG == 1) *reinterpret_cast<uintx4*>(ldsV + (size_t)i * G::kLdsRow + G::slice_off(i, sl)) = raw[u];
                    vmax = fmaxf(vmax, group_sum<SL>(Elem<T>::dot(raw[u], raw[u])));
                }
            }
        }
        vmax = wave_max(vmax);
        if (lane == 0) diag[kDiagFloats - 64 + wave] = vmax;   // the tail of the buffer: beyond the mean partials
    }
    if (center) {                        // column sums of every wavefront -> LDS
#pragma unroll
        for (int o = SL; o < 64; o <<= 1)
#pragma unroll
            for (int e = 0; e < EPL; ++e) part[e] += __shfl_xor(part[e], o);
        if (lane < SL)
#pragma unroll
            for (int q = 0; q < EPL / 4; ++q) {
                const floatx4 t = {part[4 * q], part[4 * q + 1], part[4 * q + 2], part[4 * q + 3]};
                *reinterpret_cast<floatx4*>(wpart + wave * D + sl * EPL + 4 * q) = t;
            }
    }
    __syncthreads();
    float inv_rv2 = 0.f, vg_bias = 0.f;       // the value factor is <v_i,v_j> * inv_rv2 + vg_bias
    {
        // ---------------------------------------------------------- block statistics
        // mu = mean key (fp32), a_i = <k_i, mu>, A = largest centred squared norm (or r_key^2)
        // Lane l of every wavefront holds columns l, 64 + l, ... of mu; |mu|^2 is the same value in all threads.
        constexpr int MH = D / 64;
        float mcol[MH];
        float mumu = 0.f;
        if constexpr (!MULTI) {
#pragma unroll
            for (int hh = 0; hh < MH; ++hh) {
                float s0 = 0.f;
                if (center)
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) s0 += wpart[w * D + 64 * hh + lane];
                mcol[hh] = s0 * (1.f / (float)b);
                mumu = fmaf(mcol[hh], mcol[hh], mumu);
            }
            mumu = wave_sum(mumu);
            // mu goes back to LDS, one copy per wavefront (no barrier needed): the row pass below reads it at uniform
            // addresses (broadcast reads), which costs the vector unit nothing, unlike a cross-lane read per column
            float* mu_w = wpart + kWaves * D + wave * D;
#pragma unroll
            for (int hh = 0; hh < MH; ++hh) mu_w[64 * hh + lane] = mcol[hh];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        }
        // general path: every thread forms its own 16-byte slice of mu
        float mloc[MULTI ? EPL : 1];
        if constexpr (MULTI) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) mloc[e] = 0.f;
            if (center) {
                floatx4 wp[kWaves][EPL / 4];
#pragma unroll
                for (int w = 0; w < kWaves; ++w)
#pragma unroll
                    for (int q = 0; q < EPL / 4; ++q)
                        wp[w][q] = *reinterpret_cast<const floatx4*>(wpart + w * D + sl * EPL + 4 * q);
#pragma unroll
                for (int w = 0; w < kWaves; ++w)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) mloc[e] += wp[w][e >> 2][e & 3];
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    mloc[e] *= 1.f / (float)b;
                    mumu = fmaf(mloc[e], mloc[e], mumu);
                }
                mumu = group_sum<SL>(mumu);
            }
            // mu also goes to LDS, one copy per wavefront behind the partials (its first SL lanes hold all of it; no
            // barrier): the rows that are resident in LDS are taken one per thread below, against mu at uniform addresses
            if (lane < SL) {
                float* mu_w = wpart + kWaves * D + wave * D;
#pragma unroll
                for (int q = 0; q < EPL / 4; ++q) {
                    const floatx4 t = {mloc[4 * q], mloc[4 * q + 1], mloc[4 * q + 2], mloc[4 * q + 3]};
                    *reinterpret_cast<floatx4*>(mu_w + sl * EPL + 4 * q) = t;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        }
        // Resident blocks take one row per thread (at most kThreads rows are ever resident); the general path
        // streams every row as 16-byte slices.
        const int nres = MULTI ? 0 : b;
        const bool has_row = tid < nres;
        float pa_row = 0.f;
        if (center || need_norm) {
            float amax = -3.0e38f;
            // One row per thread: mu comes through scalar registers, MC columns at a time, so the dot products need
            // no cross-lane step; |k|^2 from exact bf16 products (v_dot2c_f32_bf16).
            if constexpr (!MULTI) {
                constexpr int MC = 16;                          // columns of mu held in scalar registers at a time
                constexpr int SLQ = MC * (int)sizeof(T) / 16;   // 16-byte slices per MC columns
                float pn = 0.f;
#pragma unroll
                for (int qc = 0; qc < D / MC; ++qc) {
                    float sm[MC];
                    const float* mu_w = wpart + kWaves * D + wave * D;
#pragma unroll
                    for (int jj = 0; jj < MC / 4; ++jj) {
                        const floatx4 t = *reinterpret_cast<const floatx4*>(mu_w + qc * MC + 4 * jj);
                        sm[4 * jj] = t[0]; sm[4 * jj + 1] = t[1]; sm[4 * jj + 2] = t[2]; sm[4 * jj + 3] = t[3];
                    }
                    if (has_row) {
#pragma unroll
                        for (int ss = 0; ss < SLQ; ++ss) {
                            const uintx4 raw = *reinterpret_cast<const uintx4*>(ldsK + (size_t)tid * G::kLdsRow + G::slice_off(tid, qc * SLQ + ss));
                            float f[EPL];
                            Elem<T>::unpack(raw, f);
#pragma unroll
                            for (int e = 0; e < EPL; ++e) pa_row = fmaf(f[e], sm[ss * EPL + e], pa_row);
                            pn += Elem<T>::dot(raw, raw);
                        }
                    }
                }
                if (has_row) amax = pn - 2.f * pa_row + mumu;
            }
            if constexpr (MULTI) {
                // a 16-byte slice per thread, DPP sums per row.  Rows of the first chunk come from LDS, the others from
                // global memory (L2: the staging pass has just read them); the first batch of those is requested
                // before the resident rows are worked on, so that its latency is hidden.
                constexpr int U = 8;
                auto row_terms = [&](const uintx4& raw, int i) {
                    float f[EPL];
                    Elem<T>::unpack(raw, f);
                    float pa = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) pa = fmaf(f[e], mloc[e], pa);
                    float pn = Elem<T>::dot(raw, raw);
                    pa = group_sum<SL>(pa);
                    pn = group_sum<SL>(pn);
                    if (i < b) {
                        if (sl == 0) narow[i] = -pa;
                        amax = fmaxf(amax, pn - 2.f * pa + mumu);
                    }
                };
                auto load_global = [&](uintx4 (&raw)[U], int ib0) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = min(ib0 + u * RG + rg, b - 1);
                        raw[u] = *reinterpret_cast<const uintx4*>(Kin + (size_t)i * G::kRowBytes + sl * 16);
                    }
                };
                const int n_lds = min(CH, b);                    // b and CH are multiples of 64 and of RG
                uintx4 ahead[U];
                if (n_lds < b && !kept) load_global(ahead, n_lds);
                // resident rows: one row per thread (a chunk has at most kThreads rows), mu MC columns at a time from this
                // wavefront's copy (uniform addresses): no cross-lane step
                for (int i = tid; i < n_lds; i += kThreads) {
                    constexpr int MC = 16;
                    constexpr int SLQ = MC * (int)sizeof(T) / 16;
                    const float* mu_w = wpart + kWaves * D + wave * D;
                    float pa = 0.f, pn = 0.f;
#pragma unroll
                    for (int qc = 0; qc < D / MC; ++qc) {
                        float sm[MC];
#pragma unroll
                        for (int jj = 0; jj < MC / 4; ++jj) {
                            const floatx4 t = *reinterpret_cast<const floatx4*>(mu_w + qc * MC + 4 * jj);
                            sm[4 * jj] = t[0]; sm[4 * jj + 1] = t[1]; sm[4 * jj + 2] = t[2]; sm[4 * jj + 3] = t[3];
                        }
#pragma unroll
                        for (int ss = 0; ss < SLQ; ++ss) {
                            const uintx4 raw = *reinterpret_cast<const uintx4*>(ldsK + (size_t)i * G::kLdsRow + G::slice_off(i, qc * SLQ + ss));
                            float f[EPL];
                            Elem<T>::unpack(raw, f);
#pragma unroll
                            for (int e = 0; e < EPL; ++e) pa = fmaf(f[e], sm[ss * EPL + e], pa);
                            pn += Elem<T>::dot(raw, raw);
                        }
                    }
                    narow[i] = -pa;
                    amax = fmaxf(amax, pn - 2.f * pa + mumu);
                }
                if (kept) {                                     // the rows beyond the first chunk are still in registers
                    if constexpr (SL == 16 && kUK == 16) {
                        // sixteen rows per thread, sixteen slices per row: the partial sums change hands so that lane sl
                        // ends up with the totals of the thread's row number sl
                        float pa16[16], pn16[16];
#pragma unroll
                        for (int k = 0; k < 16; ++k) {
                            float f[EPL];
                            Elem<T>::unpack(keep[k], f);
                            float pa = 0.f;
#pragma unroll
                            for (int e = 0; e < EPL; ++e) pa = fmaf(f[e], mloc[e], pa);
                            pa16[k] = pa;
                            pn16[k] = Elem<T>::dot(keep[k], keep[k]);
                        }
                        const float pa = row16_transpose_sum(pa16, sl), pn = row16_transpose_sum(pn16, sl);
                        const int i = (kU0 + sl) * RG + rg;
                        if (i < b) {
                            narow[i] = -pa;
                            amax = fmaxf(amax, pn - 2.f * pa + mumu);
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < kUK; ++k) {
                            const int i = (kU0 + k) * RG + rg;
                            row_terms(keep[k], i < b ? i : b);
                        }
                    }
                }
                for (int ib0 = n_lds; ib0 < b && !kept; ib0 += RG * U) {
                    uintx4 raw[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) raw[u] = ahead[u];
                    if (ib0 + RG * U < b) load_global(ahead, ib0 + RG * U);
#pragma unroll
                    for (int u = 0; u < U; ++u) row_terms(raw[u], ib0 + u * RG + rg);
                }
            }
            amax = wave_max(amax);
            if (lane == 0) scal[2 + wave] = amax;
        } else {
            for (int i = nres + tid; i < b; i += kThreads) narow[i] = 0.f;
        }
        if constexpr (VG != 0) {                                // 1 / r_value^2: given, or the largest |v_i|^2 of the block
            float r2 = rvalue2;
            if (!(r2 > 0.f)) {
                r2 = diag[kDiagFloats - 64];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) r2 = fmaxf(r2, diag[kDiagFloats - 64 + w]);
            }
            inv_rv2 = r2 > 0.f ? 1.f / r2 : 0.f;               // all values zero: every weight is zero
            if (a.flags & BKV_VALUE_AUGMENT) {                  // value [v / r ; 1], radius^2 = 2 (or 1 when all values are zero)
                vg_bias = r2 > 0.f ? 0.5f : 1.f;
                inv_rv2 *= 0.5f;
            }
        }
        __syncthreads();                                        // wpart (aliasing diag) is dead from here
        {
            float A = a.rkey2;
            if (need_norm) {
                A = scal[2];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) A = fmaxf(A, scal[2 + w]);
            }
            const float rc = alpha * (mumu - A + a.cterm);       // row constant of the exponent
            if (has_row) narow[tid] = -pa_row;
            if (tid == 0) scal[1] = rc;
            if (tid < 32) prog[tid] = 0;                        // progress counters of the first chunk's pipeline
        }
        __syncthreads();
    }

    // Blocks of several full chunks of eight panels, plain instances with rows of 256 bytes: the rows of the NEXT chunk
    // are brought in during the panel pipeline by column owners whose duties are over (they would idle through the last
    // walks of the chunk): a panel through the registers of such a wavefront into the slot of a row panel that every
    // column owner has passed (rowp[w]: row tiles whose operands wavefront w has read).  Slot q by the owner of column
    // q+1 (q = 0..5), slot 7 by wavefront 5, which formed the last diagonal tile, slot 6 by wavefront 3 once the owner
    // of column 7 has read it.  The read's latency hides behind the walk; nothing stays in registers across a barrier.
    constexpr bool kPre = MULTI && !EMIT_G && VG == 0 && G::kRowBytes == 256;
    const bool pre_on = kPre && CH == 512;
    int foff[G::kGroups];                      // byte offset, inside an LDS row, of this lane's fragment of k-group g
#pragma unroll
    for (int g = 0; g < G::kGroups; ++g) foff[g] = G::slice_off(n, 2 * g + h);

    for (int c = 0; c < n_chunks; ++c) {
        const int row0 = c * CH;                       // first row of the chunk
        const int rows_here = min(CH, b - row0);
        const int p0 = row0 >> 6, p1 = (row0 + rows_here) >> 6;
        if (c > 0) {
            __syncthreads();                           // previous users of ldsK are done
            if (!pre_on) stage_chunk(row0, rows_here, 0);      // (else the previous pipeline has brought the rows in already)
            if (tid < 32 && tid != 3) prog[tid] = 0;   // progress counters of this chunk's pipeline (the error flag is sticky)
            __syncthreads();
        }
        const float row_const = scal[1];

        // ---------------------------------------------------------- rows of earlier chunks
        // Every earlier row panel I (all signs known) meets every column panel J of the resident chunk.
        // A wavefront takes row panels I = wave, wave + 8, ...: it loads them once from global memory (L2) as
        // the A operand and sweeps all J of the chunk; per-wavefront column sums go through LDS and are added
        // to sigma in a fixed order, so the result does not depend on timing.
        if (c > 0) {
            const int nJ = p1 - p0;                       // <= 8
            float* partial = diag;                        // [kWaves][8][64], the diagonal-tile buffer is idle here
            bool first = true;
            for (int I = wave; I < p0; I += kWaves) {
                Frag A[G::kGroups][2];
                Ops::load_frags(A, Kin + (size_t)(I << 6) * G::kRowBytes, G::kRowBytes, n, h);
                if constexpr (!EMIT_G && VG == 0) {
                    const bool first_panel = first;
                    Ops::row_sweep(A, ldsK, nJ, narow + (I << 6), narow + (p0 << 6), alpha, row_const, etaMask[I], foff, n, h, [&](int jj, float cs) {
                        float* slot = partial + (wave * 8 + jj) * 64 + lane;          // this wavefront's own slot
                        *slot = first_panel ? cs : *slot + cs;
                    });
                } else {
                float sg[32];
                Ops::signs_from_mask(sg, etaMask[I], h);
#pragma unroll 1
                for (int jj = 0; jj < nJ; ++jj) {
                    const int J = p0 + jj;
                    const char* ldsB = lds_rows(jj << 6);
                    floatx16 acc[2][2];
                    const float cs = Ops::template tile<true, true, false, false, VG>(
                        acc, A, nullptr, ldsB, narow + (I << 6), narow + (J << 6), alpha, row_const, sg, nullptr, foff, n, h, nullptr,
                        VG == 2 ? vrow((I << 6) + n) : nullptr, VG == 2 ? vrow((J << 6) + n) : nullptr, inv_rv2,
                        VG == 2 ? vrow((I << 6) + 32 + n) : nullptr, VG == 2 ? vrow((J << 6) + 32 + n) : nullptr, vg_bias);
                    if constexpr (EMIT_G) {
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int row = (I << 6) + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
                                Gi[(size_t)row * b + (J << 6) + n] = acc[rb][0][r];
                                Gi[(size_t)row * b + (J << 6) + 32 + n] = acc[rb][1][r];
                                Gi[(size_t)((J << 6) + n) * b + row] = acc[rb][0][r];
                                Gi[(size_t)((J << 6) + 32 + n) * b + row] = acc[rb][1][r];
                            }
                    }
                    float* slot = partial + (wave * 8 + jj) * 64 + lane;      // this wavefront's own slot
                    *slot = first ? cs : *slot + cs;
                }
                }
                first = false;
            }
            if (first)                                    // no row panel for this wavefront
                for (int jj = 0; jj < nJ; ++jj) partial[(wave * 8 + jj) * 64 + lane] = 0.f;
            __syncthreads();
            if (wave < nJ) {
                const int J = p0 + wave;
                float tot = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) tot += partial[(w * 8 + wave) * 64 + lane];
                sigma[(J << 6) + lane] += tot;
            }
            __syncthreads();                              // the buffer goes back to the diagonal tile
        }
        // ---------------------------------------------------------- panels of this chunk: a dataflow pipeline
        // No barriers in here.  Counters (all start at 0, local panel index l = I - p0):
        //   eta_done      panels walked so far (the walker publishes after writing the signs of panel l)
        //   diag_ready    diagonal tiles stored so far        diag_taken   diagonal tiles the walker has loaded so far
        //   col[l]        set to l by the owner of column panel l once sigma of that panel holds every earlier row panel
        //   rowp[w]       row panels whose LDS rows column owner w has read for the last time (only where the next chunk is
        //                 brought in during this pipeline, see kPre)
        // Wavefront w = 1..7 owns column panel w of the chunk: it keeps the panel's fragments in registers as the B
        // operand and forms, in row order, the tiles (i, w), i < w (weights need nothing; the signed column sum needs
        // eta_done > i and goes into a register copy of sigma); then, its column being complete just as the walk of
        // panel w starts, the diagonal tile of panel w+2, which it stores when the walker has taken the previous one
        // (at start-up the tile of panel 0 comes as three quadrants from wavefronts 1-3 -- as a whole from wavefront 7 in
        // the instances with a weight dump or the value factor --, that of panel 1 from wavefront 6, that of panel 2 from
        // wavefront 1).  Every sigma receives
        // its contributions in the same order on every run.  At most one tile per wavefront and walked panel is due,
        // so the walk (wavefront 0) only ever waits for the tile (l-1, l) that depends on its last signs.
        int* eta_done = prog;
        int* diag_ready = prog + 1;
        int* diag_taken = prog + 2;
        int* sync_err = prog + 3;
        int* first_parts = prog + 4;                  // quadrants of the chunk's first diagonal tile stored so far (three writers)
        int* col = prog + 8;
        int* rowp = prog + 16;                        // rowp[w]: row panels whose LDS rows column owner w needs no more
        constexpr bool kSplitFirst = !EMIT_G && VG == 0;   // the first tile comes in three quadrants from three wavefronts
        const int nPc = p1 - p0;
        const int next0 = row0 + rows_here;                                           // first row of the next chunk
        const int nN = pre_on && c + 1 < n_chunks ? (min(CH, b - next0) >> 6) : 0;    // its panels (0: nothing to bring in)
        if (wave == 0) {
            unsigned int sign_bit = 0x80000000u;
            asm volatile("" : "+s"(sign_bit));             // stays in a scalar register
            __builtin_amdgcn_s_setprio(3);                    // the serial chain goes first on its SIMD
            for (int l = 0; l < nPc; ++l) {
                const int I = p0 + l;
                // ------------------------------------------------ the walk over panel I (Alg. 2 lines 4-11)
                // this lane's column of the diagonal tile: g[j] = g_{j,lane} for j < lane, else 0
                // sigma holds (sum of signed weights so far) - (1 - 2 u): eta = +1 <=> u < 1/2 - s/2 <=> sigma < 0; it is
                // complete when the owner of this column panel says so (col[l] == l)
                float g[64];
                if (kSplitFirst && l == 0) await_and_read_tile(first_parts, 3, diag + lane * kDiagStride, g, sync_err);
                else await_and_read_tile(diag_ready, l + 1, diag + lane * kDiagStride, g, sync_err);
                publish(diag_taken, l + 1);                   // the tile is in registers: the buffer may be overwritten
                float sv = await_and_read(col + l, l, sigma + (I << 6) + lane, sync_err);
                walk_panel(sv, g, sign_bit);
                const unsigned long long m = __ballot(sv < 0.f);
                if (lane == 0) etaMask[I] = m;
                {
                    const int k = lane & 31;
                    const int row = 32 * (k >> 4) + 8 * ((k & 15) >> 2) + 4 * h + (k & 3);
                    etaF[(l << 6) + lane] = ((m >> row) & 1ull) ? 1.f : -1.f;
                }
                publish_in_order(eta_done, l + 1);
                sigma[(I << 6) + lane] = sv;                  // decision-time values, read back for the statistics (nobody waits for it)
            }
            __builtin_amdgcn_s_setprio(0);
        } else {
            const int w = wave;                               // local column panel of this wavefront
            const bool owner = w < nPc;
            // While the chip is busy with the walk, each of these wavefronts also touches the keys of one panel of the
            // block that this compute unit is likely to receive next (one dword per 16 bytes: every cache line), so
            // that its staging pass finds them in L2 / MALL.  The values are only consumed at the end.
            constexpr int PF = G::kRowBytes / 16;                               // loads per panel
            const int64_t inst_pf = inst + a.prefetch_ahead;
            const bool do_pf = a.prefetch_ahead > 0 && inst_pf < (int64_t)gridDim.x;
            int pfv[PF], pfv0[PF], pfacc = 0;
#pragma unroll
            for (int j = 0; j < PF; ++j) { pfv[j] = 0; pfv0[j] = 0; }
            if (do_pf) {
                const int64_t seq_pf = inst_pf / a.blocks_per_seq;
                const int64_t blk_pf = inst_pf - seq_pf * a.blocks_per_seq;
                const char* Kpf = a.K + (seq_pf * a.in_seq_stride + blk_pf * b) * G::kRowBytes + lane * 16;
                const int pf_panel = (owner ? p0 + w : p0);   // wavefront 1 covers panel 0 as well when it owns no column
                if (owner) {
#pragma unroll
                    for (int j = 0; j < PF; ++j) pfv[j] = *reinterpret_cast<const int*>(Kpf + (size_t)(pf_panel << 6) * G::kRowBytes + j * 1024);
                }
                if (w == 1) {
#pragma unroll
                    for (int j = 0; j < PF; ++j) pfv0[j] = *reinterpret_cast<const int*>(Kpf + (size_t)(p0 << 6) * G::kRowBytes + j * 1024);
                }
            }
            // diagonal tile of local panel l from the panel's fragments P (both operands), stored in turn
            auto diagonal = [&](const Frag (&P)[G::kGroups][2], int l) {
                const int I = p0 + l;
                floatx16 dv[2][2];
                const char* vrows = VG == 1 ? ldsV + (size_t)(l << 6) * G::kLdsRow : VG == 2 ? vrow((I << 6) + n) : nullptr;
                const char* vrows1 = VG == 2 ? vrow((I << 6) + 32 + n) : nullptr;
                Ops::template tile<false, true, true, !EMIT_G, VG>(dv, P, nullptr, nullptr, narow + (I << 6), narow + (I << 6), alpha, row_const,
                                                                   nullptr, nullptr, foff, n, h, P, vrows, vrows, inv_rv2, vrows1, vrows1, vg_bias);
                if (EMIT_G) {
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
                            Gi[(size_t)((I << 6) + row) * b + (I << 6) + n] = dv[rb][0][r];
                            Gi[(size_t)((I << 6) + row) * b + (I << 6) + 32 + n] = dv[rb][1][r];
                        }
                }
                Ops::mask_diag(dv, n, h);
                // the tile is complete here: the compiler must not sink its arithmetic below the wait
                asm volatile("" : "+v"(dv[0][0]), "+v"(dv[0][1]), "+v"(dv[1][0]), "+v"(dv[1][1]));
                await(diag_taken, l, sync_err);               // the walker holds the previous tile in registers
                Ops::store_diag(diag, dv, n, h);
                publish(diag_ready, l + 1);
            };
            Frag Bq[G::kGroups][2];
            // Start-up: the diagonal tile of panel 1 (and, where it is not split, that of panel 0) comes from the
            // wavefronts whose own columns are needed last.
            if (kSplitFirst && w <= 3) {
                // the walk cannot start without the first tile: wavefronts 1, 2, 3 (three SIMDs) take a quadrant each
                __builtin_amdgcn_s_setprio(2);
                const float* ap0 = narow + (p0 << 6);
                if (w == 1) Ops::template diag_quadrant<0, 0>(diag, lds_rows(0), ap0, alpha, row_const, foff, n, h);
                else if (w == 2) Ops::template diag_quadrant<0, 1>(diag, lds_rows(0), ap0, alpha, row_const, foff, n, h);
                else Ops::template diag_quadrant<1, 1>(diag, lds_rows(0), ap0, alpha, row_const, foff, n, h);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                if (lane == 0) __hip_atomic_fetch_add(first_parts, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __builtin_amdgcn_s_setprio(0);
            }
            if (w >= kWaves - 2 && kWaves - 1 - w < nPc && !(kSplitFirst && w == kWaves - 1)) {
                if (w == kWaves - 1) __builtin_amdgcn_s_setprio(2);       // the walk cannot start without the first tile
                Ops::load_panel(Bq, lds_rows((kWaves - 1 - w) << 6), foff, n);
                diagonal(Bq, kWaves - 1 - w);
                __builtin_amdgcn_s_setprio(0);
            }
            if (owner) {
                const int J = p0 + w;
                Ops::load_panel(Bq, lds_rows(w << 6), foff, n);
                float sig = sigma[(J << 6) + lane];           // minus the threshold, plus what earlier chunks added
                for (int i = 0; i < w; ++i) {
                    const int Ii = p0 + i;
                    floatx16 acc[2][2];
                    Ops::template tile<false, false, true, false, VG>(acc, nullptr, lds_rows(i << 6), nullptr, narow + (Ii << 6), narow + (J << 6), alpha, row_const,
                                                                      nullptr, nullptr, foff, n, h, Bq,
                                                                      VG == 1 ? ldsV + (size_t)(i << 6) * G::kLdsRow : VG == 2 ? vrow((Ii << 6) + n) : nullptr,
                                                                      VG == 1 ? ldsV + (size_t)(w << 6) * G::kLdsRow : VG == 2 ? vrow((J << 6) + n) : nullptr, inv_rv2,
                                                                      VG == 2 ? vrow((Ii << 6) + 32 + n) : nullptr, VG == 2 ? vrow((J << 6) + 32 + n) : nullptr, vg_bias);
                    if (EMIT_G) {
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int row = (Ii << 6) + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
                                Gi[(size_t)row * b + (J << 6) + n] = acc[rb][0][r];
                                Gi[(size_t)row * b + (J << 6) + 32 + n] = acc[rb][1][r];
                                Gi[(size_t)((J << 6) + n) * b + row] = acc[rb][0][r];
                                Gi[(size_t)((J << 6) + 32 + n) * b + row] = acc[rb][1][r];
                            }
                    }
                    // the weights are complete here: the compiler must not sink their arithmetic below the wait
                    asm volatile("" : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]));
                    // this wavefront has read row panel i for the last time: its operands were in registers before the tile's
                    // matrix instructions could issue, so a plain store says so
                    if (kPre && nN > 0) publish_in_order(rowp + w, i + 1);
                    // signs of row panel i (once the walker has published them), signed column sums
                    const bool urgent = i == w - 1;            // the walker is waiting for this one
                    float sg[32];
                    if (urgent) { __builtin_amdgcn_s_setprio(3); await<true>(eta_done, i + 1, sync_err); }
                    else await(eta_done, i + 1, sync_err);
                    Ops::signs_from_lds(sg, etaF + (i << 6) + 32 * h);
                    sig += Ops::signed_colsum(acc, sg, h);
                    if (urgent) {
                        sigma[(J << 6) + lane] = sig;
                        publish_in_order(col + w, w);
                        __builtin_amdgcn_s_setprio(0);
                    }
                }
                // This column is complete (the walk of panel w is starting): form the diagonal tile that is due two
                // walks from now.  Wavefront 1, which has no predecessor, also supplies the tile of panel 2.
                for (int l = (w == 1 ? 2 : w + 2); l <= w + 2 && l < nPc; ++l) {     // wavefront 1 also supplies panel 2's
                    Ops::load_panel(Bq, lds_rows(l << 6), foff, n);
                    diagonal(Bq, l);
                }
            }
#pragma unroll
            for (int j = 0; j < PF; ++j) pfacc ^= pfv[j] ^ pfv0[j];
            asm volatile("" :: "v"(pfacc));                   // the touches must not be optimised away
            if constexpr (kPre) {
                if (nN > 0 && nPc == 8 && w <= 6) {
                    int ln = lane;
                    asm volatile("" : "+v"(ln));              // the lane's offsets are formed here, not kept across the chunks
                    const int r_w = ln >> 4, s_w = ln & 15;  // 16 slices per row: a load covers four rows
                    // first job: slot w-1; second job of wavefronts 5 and 3: slots 7 and 6
                    for (int job = 0; job < 2; ++job) {
                        const int q = job == 0 ? w - 1 : (w == 5 ? 7 : w == 3 ? 6 : -1);
                        if (q < 0 || q >= nN) continue;
                        // The slot's readers are through: every column owner behind row panel q has taken its tile of it
                        // (slot 7: owner 7 its own fragments), owner q holds its fragments, and the diagonal tile of panel q is
                        // formed (stored, or for panel 0 its three quadrants; that of panel 7 this wavefront formed itself).
                        const int need = q == 7 ? 1 : q + 1;
                        for (int v = (q == 7 ? 7 : q + 1); v < 8; ++v)
                            if (v != w) await(rowp + v, need, sync_err);
                        if (q >= 1 && q != 7) await(rowp + q, 1, sync_err);
                        if (q == 0) await(first_parts, 3, sync_err);
                        else if (q != 7) await(diag_ready, q + 1, sync_err);
                        uintx4 t[16];
                        const char* src = Kin + (size_t)(next0 + (q << 6) + r_w) * G::kRowBytes + s_w * 16;
#pragma unroll
                        for (int u = 0; u < 16; ++u) t[u] = *reinterpret_cast<const uintx4*>(src + (size_t)u * 4 * G::kRowBytes);
#pragma unroll
                        for (int u = 0; u < 16; ++u) {
                            const int row = (q << 6) + 4 * u + r_w;
                            *reinterpret_cast<uintx4*>(ldsK + (size_t)row * G::kLdsRow + G::slice_off(row, s_w)) = t[u];
                        }
                    }
                }
            }
        }
        __syncthreads();                                   // the chunk is done: LDS rows, counters and tile buffer are free
    }

    // ------------------------------------------------------------------ output step (Alg. 2 lines 12-16 + strict n/2)
    // Every wavefront handles the panels p = wave, wave + 8, ...: minority sign ('+' on ties), then exactly
    // b/2 survivors = the minority class plus the lowest-index majority tokens, ascending.
    {
        // lane q < nP (nP <= 16) carries the counts of panel q; prefix sums run over the first row of 16 lanes
        auto row_scan = [](int x) -> int {                                // inclusive prefix sum inside a row of 16 lanes
            x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);   // row_shr:1, zero fill
            x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);   // row_shr:2
            x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);   // row_shr:4
            x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);   // row_shr:8
            return x;
        };
        int plus_q = 0;
        if (lane < nP) plus_q = __popcll(etaMask[lane]);
        const int n_plus = __builtin_amdgcn_readlane(row_scan(plus_q), 15);
        const bool plus_is_minority = n_plus <= b - n_plus;               // tie -> '+'
        const int n_min = plus_is_minority ? n_plus : b - n_plus;
        const int need = b / 2 - n_min;                                   // majority tokens to add, lowest index first
        const int min_q = (lane < nP) ? (plus_is_minority ? plus_q : 64 - plus_q) : 0;
        const int maj_q = (lane < nP) ? 64 - min_q : 0;
        const int maj_before_q = row_scan(maj_q) - maj_q;
        const int kept_q = min_q + max(0, min(maj_q, need - maj_before_q));
        const int kept_before_q = row_scan(kept_q) - kept_q;
        const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        for (int p = wave; p < nP; p += kWaves) {
            const int maj_before = __builtin_amdgcn_readlane(maj_before_q, p);
            const int kept_before = __builtin_amdgcn_readlane(kept_before_q, p);
            const unsigned long long mv = etaMask[p];
            const unsigned long long m = ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned int)(mv >> 32)) << 32) |
                                         (unsigned int)__builtin_amdgcn_readfirstlane((unsigned int)mv);
            const unsigned long long minm = plus_is_minority ? m : ~m;
            const unsigned long long majm = ~minm;
            const int my_rank = maj_before + __popcll(majm & lt);
            const bool keep = ((minm >> lane) & 1ull) || (my_rank < need);
            const unsigned long long km = __ballot(keep);
            if (keep) keptIdx[kept_before + __popcll(km & lt)] = (p << 6) + lane;
        }
    }
    __syncthreads();
    if (wave == 0) {      // side outputs: issued after the barrier so that nobody waits for these stores
        if (a.signs_out)
            for (int p = 0; p < nP; ++p)
                a.signs_out[(size_t)signs0 + (p << 6) + lane] = ((etaMask[p] >> lane) & 1ull) ? 1 : -1;
    } else if (wave == 2 && (a.status_out || a.stats_out)) {
        // walk statistics from the decision-time values: FAIL events (Alg. 2 line 7), near-tie decisions
        int n_margin = 0, any_fail = 0;
        float min_margin = 3.0e38f, max_sigma = 0.f;
        for (int p = 0; p < nP; ++p) {
            const float tau = threshold((p << 6) + lane);
            const float sg = sigma[(p << 6) + lane] + tau;                        // y^T eta / (c R^2) at decision time
            any_fail |= (__ballot(fabsf(sg) > 1.f) != 0ull);
            const float margin = 0.5f * fabsf(fminf(fmaxf(sg, -1.f), 1.f) - tau);  // |u - clamp(p)|
            n_margin += __popcll(__ballot(margin < 1e-4f));
            min_margin = fminf(min_margin, margin);
            max_sigma = fmaxf(max_sigma, fabsf(sg));
        }
        min_margin = wave_min(min_margin);
        max_sigma = wave_max(max_sigma);
        if (lane == 0) {
            const int sync_failed = prog[3];
            const int word = (any_fail ? BKV_STATUS_FAIL : 0) | (sync_failed ? BKV_STATUS_INTERNAL : 0) | (n_margin << 8);
            if (a.status_out) {
                if (a.tree_mode) {
                    int* dst = a.status_out + seq * a.status_stride + a.round;
                    if (any_fail) atomicOr(dst, BKV_STATUS_FAIL);
                    if (sync_failed) atomicOr(dst, BKV_STATUS_INTERNAL);
                    if (n_margin) {
                        // the count lives in bits 8..30 and saturates there: bit 31 is never set.  Margin decisions
                        // are rare, so the compare-and-swap loop (it ends when no other block updates the word in
                        // between) is next to never entered twice.
                        int seen = __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        for (;;) {
                            const int cnt = min((seen >> 8) + n_margin, 0x7fffff);
                            const int want = (seen & 0xff) | (cnt << 8);
                            const int prev = atomicCAS(dst, seen, want);
                            if (prev == seen) break;
                            seen = prev;
                        }
                    }
                } else {
                    a.status_out[inst] = word;
                }
            }
            if (a.stats_out) {
                a.stats_out[2 * inst] = min_margin;
                a.stats_out[2 * inst + 1] = max_sigma;
            }
        }
    }
    // a pipeline time-out also goes to the caller's sticky word (a streaming cache has one), whether or not a status
    // array was passed
    if (a.sticky_err && tid == 0 && prog[3]) atomicOr(a.sticky_err, BKV_STATUS_INTERNAL);
    const int half = b >> 1;
    // survivors: rows of the ORIGINAL keys / values, ascending index (16-byte slices, several rows in flight)
    auto src_token = [&](int r) -> int64_t {      // token of survivor r within its sequence, in the value tensor's frame
        const int kept = keptIdx[r];
        return a.idx_in ? (int64_t)a.idx_in[in_tok0 + kept] : tok_base + kept;
    };
    {
        // Keys come from LDS when the whole block is still resident, else from global memory (L2); value rows
        // always come from global memory.  All loads of a pass are issued before its first store.
        char* Ko = a.K_out ? a.K_out + out_tok0 * G::kRowBytes : nullptr;
        const bool do_v = a.V_out && a.V;
        const char* Vseq = do_v ? a.V + (size_t)seq * a.v_seq_stride * G::kRowBytes : nullptr;
        char* Vo = do_v ? a.V_out + out_tok0 * G::kRowBytes : nullptr;
        const bool k_global = Ko && !single_chunk;
        constexpr int U = 16;
        for (int r0 = rg; r0 < half; r0 += RG * U) {
            uintx4 kraw[U], vraw[U];
            if (do_v) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RG;
                    if (r < half) vraw[u] = *reinterpret_cast<const uintx4*>(Vseq + (size_t)src_token(r) * G::kRowBytes + sl * 16);
                }
            }
            if (k_global) {
                const int res0 = (n_chunks - 1) * CH;          // rows from here on are still resident (last chunk)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RG;
                    if (r < half) {
                        const int kr = keptIdx[r];
                        if (kr >= res0)
                            kraw[u] = *reinterpret_cast<const uintx4*>(ldsK + (size_t)(kr - res0) * G::kLdsRow + G::slice_off(kr - res0, sl));
                        else
                            kraw[u] = *reinterpret_cast<const uintx4*>(Kin + (size_t)kr * G::kRowBytes + sl * 16);
                    }
                }
            } else if (Ko) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RG;
                    if (r < half) {
                        const int kr = keptIdx[r];
                        kraw[u] = *reinterpret_cast<const uintx4*>(ldsK + (size_t)kr * G::kLdsRow + G::slice_off(kr, sl));
                    }
                }
            }
            if (Ko) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RG;
                    // (streamed past the caches: a later pass over the survivors then finds no write-backs in its way)
                    if (r < half) __builtin_nontemporal_store(kraw[u], reinterpret_cast<uintx4*>(Ko + (size_t)r * G::kRowBytes + sl * 16));
                }
            }
            if (do_v) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RG;
                    if (r < half) __builtin_nontemporal_store(vraw[u], reinterpret_cast<uintx4*>(Vo + (size_t)r * G::kRowBytes + sl * 16));
                }
            }
        }
    }
    for (int r = tid; r < half; r += kThreads) {
        if (a.w_out) a.w_out[out_tok0 + r] = a.w_out_val;
        if (a.idx_out) a.idx_out[idx_out0 + r] = (int32_t)src_token(r);
    }
}

// ------------------------------------------------------------------------------------------------
template <typename T, int D, bool EMIT_G, bool MULTI, int VG = 0>
static hipError_t launch_one(const CompressArgs& a, int64_t n_inst, hipStream_t st) {
    const size_t lds = compress_lds_bytes(Geo<T, D>::kRowBytes, a.b, VG == 1);
    auto kern = compress_kernel<T, D, EMIT_G, MULTI, VG>;
    static thread_local size_t configured = 0;
    if (lds > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = lds;
    }
    return launch_timed(kProfCompress, n_inst * a.b, kern, dim3((unsigned)n_inst), dim3(kThreads), lds, st, a);
}

hipError_t launch_compress(int dtype, int d, bool emit_g, CompressArgs& a, int64_t n_inst, hipStream_t st) {
    const int row_bytes = d * (dtype == BKV_BF16 ? 2 : 4);
    const bool vgram = (a.flags & BKV_VALUE_GRAM) != 0;
    // value factor: no Gram dump, value rows required; the values are staged in LDS when they fit next to the keys
    if (vgram && (emit_g || !a.V)) return hipErrorInvalidValue;
    if (a.k_by_idx && (!a.idx_in || emit_g)) return hipErrorInvalidValue;
    const bool v_lds = vgram && compress_value_gram_fits(row_bytes, a.b);
    a.chunk_rows = chunk_rows_for(row_bytes, a.b, v_lds);
    if (n_inst <= 0) return hipSuccess;
    {
        // one workgroup per compute unit is resident (LDS); with at least two rounds of workgroups, spread the first
        static thread_local int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0;
            hipDeviceProp_t prop;
            if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorUnknown;
            n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
        }
        a.stagger_blocks = 0; a.stagger_step = 0; a.prefetch_ahead = 0;
        if (n_inst >= 2 * (int64_t)n_cu && !a.desc) {   // (a ragged grid has unused slots: neighbours in the grid are not neighbours in memory)
            // The first workgroups start spread over about two thirds of one block's duration: 100k clock ticks for 1024
            // bf16 tokens, whose blocks take about 145k (a spread over the whole duration keeps the compute units idle
            // longer at both ends of a launch than the better interleaving gives back: 2 % on a launch of 32 blocks per
            // compute unit; a third of the duration interleaves too little).
            const double ticks = (20.0e3 + 0.075 * (double)a.b * (double)a.b) * (dtype == BKV_BF16 ? 1.0 : 1.5);
            a.stagger_blocks = n_cu;
            a.stagger_step = (int)(ticks / n_cu);
            // Look-ahead touches pay where they are the only second read of a row (blocks resident as one chunk: 2-4 %);
            // a block of several chunks already reads its rows about three times over and is limited by the traffic
            // between L2 and the fabric, where one more pass costs 6 %.
            a.prefetch_ahead = a.b <= a.chunk_rows ? n_cu : 0;
        }
    }
    // grids are one-dimensional; split very large launches
    const int64_t kMaxGrid = 1ll << 30;
    if (n_inst > kMaxGrid) return hipErrorInvalidValue;
    const bool multi = a.b > a.chunk_rows;       // the Gram-emitting (test) variant always takes the general code
    if (a.k_by_idx && multi) return hipErrorInvalidValue;      // scattered key rows: resident blocks only
#define BKV_DISPATCH(TT, DD)                                                                \
    return v_lds ? launch_one<TT, DD, false, false, 1>(a, n_inst, st)                       \
         : vgram ? (multi ? launch_one<TT, DD, false, true, 2>(a, n_inst, st)               \
                          : launch_one<TT, DD, false, false, 2>(a, n_inst, st))             \
         : emit_g ? launch_one<TT, DD, true, true>(a, n_inst, st)                           \
                  : multi ? launch_one<TT, DD, false, true>(a, n_inst, st)                  \
                          : launch_one<TT, DD, false, false>(a, n_inst, st)
    if (dtype == BKV_BF16 && d == 128) { BKV_DISPATCH(__bf16, 128); }
    if (dtype == BKV_BF16 && d == 64) { BKV_DISPATCH(__bf16, 64); }
    if (dtype == BKV_F32 && d == 128) { BKV_DISPATCH(float, 128); }
    if (dtype == BKV_F32 && d == 64) { BKV_DISPATCH(float, 64); }
#undef BKV_DISPATCH
    return hipErrorInvalidValue;
}

// Fill / copy helpers (plain kernels: safe under graph capture, unlike memset nodes).
__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (int64_t)gridDim.x * blockDim.x)
        p[t] = v;
}
hipError_t launch_fill_u32(void* p, uint32_t v, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t*)p, v, n);
    return hipGetLastError();
}

// Strided 16-byte copy: dst[seq, dst_off + r, :] = src[seq, src_off + r, :] for r < rows.
__global__ void copy_rows_kernel(const char* src, char* dst, int64_t src_seq_stride, int64_t dst_seq_stride,
                                 int64_t rows, int row_bytes, int64_t total_slices) {
    const int slices = row_bytes >> 4;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total_slices;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = t / slices;
        const int s = (int)(t - row * slices);
        const int64_t seq = row / rows;
        const int64_t r = row - seq * rows;
        *reinterpret_cast<uintx4*>(dst + (size_t)(seq * dst_seq_stride + r) * row_bytes + s * 16) =
            *reinterpret_cast<const uintx4*>(src + (size_t)(seq * src_seq_stride + r) * row_bytes + s * 16);
    }
}
hipError_t launch_copy_rows(const void* src, void* dst, int64_t n_seq, int64_t src_seq_stride,
                            int64_t dst_seq_stride, int64_t rows, int row_bytes, hipStream_t st) {
    const int64_t total = n_seq * rows * (row_bytes >> 4);
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const char*)src, (char*)dst,
                       src_seq_stride, dst_seq_stride, rows, row_bytes, total);
    return hipGetLastError();
}

// dst[seq, r] = src[seq, r] for r < rows (fp32, strided per sequence)
__global__ void copy_f32_kernel(const float* src, float* dst, int64_t src_seq_stride, int64_t dst_seq_stride,
                                int64_t rows, int64_t total) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t seq = t / rows;
        const int64_t r = t - seq * rows;
        dst[seq * dst_seq_stride + r] = src[seq * src_seq_stride + r];
    }
}
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n_seq, int64_t src_seq_stride,
                           int64_t dst_seq_stride, int64_t rows, hipStream_t st) {
    const int64_t total = n_seq * rows;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, src_seq_stride,
                       dst_seq_stride, rows, total);
    return hipGetLastError();
}

// One streamed token per sequence: K[seq, pos, :] = k[seq, :], V likewise, w[seq, pos] = 1 (Alg. 3: C^0 gets the new pair).
__global__ void append_kernel(const char* k, const char* v, char* K, char* V, float* w, int64_t seq_stride, int64_t pos,
                              int row_bytes, int64_t n_seq) {
    const int slices = row_bytes >> 4;
    const int64_t total = n_seq * slices;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t seq = t / slices;
        const int s = (int)(t - seq * slices);
        const size_t dst = (size_t)(seq * seq_stride + pos) * row_bytes + s * 16;
        *reinterpret_cast<uintx4*>(K + dst) = *reinterpret_cast<const uintx4*>(k + (size_t)seq * row_bytes + s * 16);
        *reinterpret_cast<uintx4*>(V + dst) = *reinterpret_cast<const uintx4*>(v + (size_t)seq * row_bytes + s * 16);
        if (s == 0) w[seq * seq_stride + pos] = 1.f;
    }
}
hipError_t launch_append(const void* k, const void* v, void* K, void* V, float* w, int64_t n_seq, int64_t seq_stride,
                         int64_t pos, int row_bytes, hipStream_t st) {
    const int64_t total = n_seq * (row_bytes >> 4);
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const char*)k, (const char*)v, (char*)K,
                       (char*)V, w, seq_stride, pos, row_bytes, n_seq);
    return hipGetLastError();
}

// w[seq, off + r] = val for r < rows
__global__ void fill_w_kernel(float* w, int64_t seq_stride, int64_t off, int64_t rows, float val, int64_t total) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t seq = t / rows;
        w[seq * seq_stride + off + (t - seq * rows)] = val;
    }
}
hipError_t launch_fill_w(float* w, int64_t n_seq, int64_t seq_stride, int64_t off, int64_t rows, float val,
                         hipStream_t st) {
    const int64_t total = n_seq * rows;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_w_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w, seq_stride, off, rows, val, total);
    return hipGetLastError();
}

// idx[seq, off + r] = first + r for r < rows
__global__ void fill_iota_kernel(int32_t* idx, int64_t seq_stride, int64_t off, int64_t rows, int32_t first, int64_t total) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t seq = t / rows;
        const int64_t r = t - seq * rows;
        idx[seq * seq_stride + off + r] = first + (int32_t)r;
    }
}
hipError_t launch_fill_iota(int32_t* idx, int64_t n_seq, int64_t seq_stride, int64_t off, int64_t rows, int32_t first,
                            hipStream_t st) {
    const int64_t total = n_seq * rows;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_iota_kernel, dim3((unsigned)blocks), dim3(256), 0, st, idx, seq_stride, off, rows, first, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Peak micro-benchmarks (diagnostics): what this GPU reaches on the two units the halving kernel is measured against,
// with nothing else in the way.  They give the denominators of "fraction of the measured peak" next to the vendor's.
// ------------------------------------------------------------------------------------------------
// (1) The matrix pipe alone: every wavefront issues 32x32x16 bf16 MFMAs on four independent accumulators.
__global__ __launch_bounds__(kThreads) void peak_mfma_kernel(float* out, int iters) {
    const int tid = threadIdx.x;
    bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((tid + e) & 3); b[e] = (__bf16)(float)((tid ^ e) & 1); }
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    floatx16 acc[4] = {zero, zero, zero, zero};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[u][r];
    out[(size_t)blockIdx.x * kThreads + tid] = sum;
}
// (2) The tile routine alone: one workgroup of 8 wavefronts keeps 512 bf16 rows of 128 columns in LDS; every wavefront
// takes one 64-row panel as the A operand (registers) and sweeps the 8 column panels, forming for each 64x64 tile the
// Gram, the kernel weights exp2(alpha S + row term) and the signed column sums, exactly as the halving kernel does for
// rows whose signs are known: no walk, no waiting, no HBM traffic after the first fill.  Repeated `iters` times.
__global__ __launch_bounds__(kThreads) void peak_tile_kernel(float* out, int iters) {
    typedef Geo<__bf16, 128> G;
    typedef TileOps<__bf16, 128> Ops;
    typedef typename Elem<__bf16>::Frag Frag;
    extern __shared__ __align__(16) char smem[];
    char* ldsK = smem;
    float* narow = reinterpret_cast<float*>(smem + (size_t)512 * G::kLdsRow);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, h = lane >> 5;
    for (int i = tid; i < 512 * G::kSlices; i += kThreads) {           // small integers: exact products, moderate exponents
        uintx4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned int x = (unsigned int)(i * 4 + e) * 2654435761u;
            const unsigned int lo = 0x3f80u | ((x >> 7) & 0x8000u), hi = 0x3f80u | ((x >> 9) & 0x8000u);   // +-1.0 in bf16
            v[e] = lo | (hi << 16);
        }
        const int row = i / G::kSlices, sl = i % G::kSlices;
        *reinterpret_cast<uintx4*>(ldsK + (size_t)row * G::kLdsRow + G::slice_off(row, sl)) = v;
    }
    for (int i = tid; i < 512; i += kThreads) narow[i] = -1.5f * (float)(i & 7);
    __syncthreads();
    int foff[G::kGroups];
#pragma unroll
    for (int g = 0; g < G::kGroups; ++g) foff[g] = G::slice_off(n, 2 * g + h);
    Frag A[G::kGroups][2];
    Ops::load_panel(A, ldsK + (size_t)(wave << 6) * G::kLdsRow, foff, n);
    float total = 0.f;
    for (int it = 0; it < iters; ++it)
        Ops::row_sweep(A, ldsK, 8, narow + (wave << 6), narow, 0.1275f, -20.f, 0x5a5a5a5a5a5a5a5aull + it, foff, n, h,
                       [&](int, float cs) { total += cs; });
    out[(size_t)blockIdx.x * kThreads + tid] = total;
}
// (3) Streaming: read `n16` 16-byte words once (XOR-folded into one word per thread), or copy them.  Every workgroup
// owns one contiguous range (as the attend pass does) and keeps eight 16-byte loads per lane in flight.
__global__ __launch_bounds__(256) void peak_read_kernel(const uintx4* src, unsigned int* out, int64_t n16) {
    unsigned int acc = 0;
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
    int64_t i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        uintx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < hi; i += 256) { const uintx4 a = src[i]; acc ^= a[0] ^ a[1] ^ a[2] ^ a[3]; }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}
__global__ __launch_bounds__(256) void peak_copy_kernel(const uintx4* src, uintx4* dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uintx4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// Runs one of the above `launches` times between two events and reports work per second (FLOP/s of executed MFMA work,
// or bytes/s moved).  Synchronises.  workspace: the streaming kernels use all of it (read: everything; copy: first half ->
// second half); the other kernels keep their per-thread results in its first 4 MiB.
hipError_t measure_peak(int kind, int launches, void* workspace, size_t ws_bytes, hipStream_t st, double* per_second, double* ms_per_launch) {
    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e;
    if ((e = hipGetDevice(&dev)) != hipSuccess || (e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    const int n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    hipEvent_t e0, e1;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    double work = 0.0;
    const int iters_mfma = 4096, iters_tile = 16;
    auto launch = [&]() {
        switch (kind) {
            case 0: {
                hipLaunchKernelGGL(peak_mfma_kernel, dim3(n_cu), dim3(kThreads), 0, st, (float*)workspace, iters_mfma);
                work = (double)n_cu * kWaves * iters_mfma * 4.0 * (2.0 * 32 * 32 * 16);
                break;
            }
            case 1: {
                const size_t lds = (size_t)512 * 256 + 512 * 4;
                hipLaunchKernelGGL(peak_tile_kernel, dim3(n_cu), dim3(kThreads), lds, st, (float*)workspace, iters_tile);
                work = (double)n_cu * kWaves * iters_tile * 8.0 * (2.0 * 64 * 64 * 128);
                break;
            }
            case 2: {
                const int64_t n16 = (int64_t)((ws_bytes - (4u << 20)) / 16);     // the first 4 MiB take the per-thread results
                hipLaunchKernelGGL(peak_read_kernel, dim3(n_cu * 8), dim3(256), 0, st, (const uintx4*)((char*)workspace + (4u << 20)),
                                   (unsigned int*)workspace, n16);
                work = (double)n16 * 16.0;
                break;
            }
            default: {
                const int64_t n16 = (int64_t)(ws_bytes / 32);
                hipLaunchKernelGGL(peak_copy_kernel, dim3(n_cu * 8), dim3(256), 0, st, (const uintx4*)workspace,
                                   (uintx4*)((char*)workspace + n16 * 16), n16);
                work = (double)n16 * 32.0;
                break;
            }
        }
    };
    if (kind == 1) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(peak_tile_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 512 * 256 + 512 * 4);
        if (e != hipSuccess) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return e; }
    }
    launch();                                            // warm-up
    (void)hipEventRecord(e0, st);
    for (int i = 0; i < launches; ++i) launch();
    (void)hipEventRecord(e1, st);
    e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    if ((e = hipGetLastError()) != hipSuccess) return e;
    *ms_per_launch = (double)ms / launches;
    *per_second = work * launches / ((double)ms * 1e-3);
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------------
// Opt-in per-launch timing (diagnostics): HIP events attached to the kernel launches themselves
// (start and end of the dispatch).  Disabled unless bkv_profile_enable(n > 0) was called.
// ------------------------------------------------------------------------------------------------
namespace {
struct ProfRec { hipEvent_t a, b; int kind; int64_t units; };
ProfRec* g_prof = nullptr;
int g_prof_cap = 0, g_prof_n = 0;
}  // namespace

int prof_enable(int n) {
    for (int i = 0; i < g_prof_cap; ++i) { (void)hipEventDestroy(g_prof[i].a); (void)hipEventDestroy(g_prof[i].b); }
    delete[] g_prof;
    g_prof = nullptr; g_prof_cap = 0; g_prof_n = 0;
    if (n <= 0) return 0;
    g_prof = new ProfRec[n];
    for (int i = 0; i < n; ++i) {
        if (hipEventCreate(&g_prof[i].a) != hipSuccess || hipEventCreate(&g_prof[i].b) != hipSuccess) return -1;
        g_prof_cap = i + 1;
    }
    return 0;
}
int prof_read(int32_t* kind, float* ms, int64_t* units, int cap) {
    int n = 0;
    for (int i = 0; i < g_prof_n && n < cap; ++i) {
        float t = 0.f;
        if (hipEventSynchronize(g_prof[i].b) != hipSuccess) break;
        if (hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess) break;
        kind[n] = g_prof[i].kind; ms[n] = t; units[n] = g_prof[i].units; ++n;
    }
    g_prof_n = 0;
    return n;
}
bool prof_slot(int kind, int64_t units, hipEvent_t* start, hipEvent_t* stop) {
    if (g_prof_n >= g_prof_cap) return false;
    ProfRec& r = g_prof[g_prof_n++];
    r.kind = kind; r.units = units;
    *start = r.a; *stop = r.b;
    return true;
}

}  // namespace bkv
