// SoftmaxBalance (Alg. 2 of arXiv 2502.07861) on gfx950: Gram tiles on MFMA, kernel weights and
// the self-balancing walk on chip, strict halving, gather of the survivors.
//
// One workgroup (8 wavefronts) owns one block of b tokens.  The block's keys are staged in LDS in
// chunks of up to kChunkRows rows.  The walk is organised right-looking over 64-row panels:
//
//   sigma[l] (LDS) holds sum_{i already signed} eta_i g_il for every column l of the block.
//   For panel I:  wavefront 0 forms the 64x64 diagonal tile of kernel weights, transposes it into
//                 "one column per lane" registers and runs the 64 sequential decisions
//                 (lane j compares sigma_j with 1 - 2 u_j; the outcome is broadcast with a ballot);
//                 then all wavefronts form the tiles (I, J), J > I, multiply row i by eta_i, sum
//                 over rows and add the column sums into sigma[J].
//   Rows of earlier chunks (b larger than one chunk) are streamed from global memory as the
//   A operand against the resident chunk before its own panels are walked.
//
// The kernel weight is g_ij = exp((<k_i,k_j> - a_i - a_j + |mu|^2 - A)/sqrt(d) - ln c) with
// a_i = <k_i, mu> (mu = block mean when keys are centred, else 0) and A = r_key^2 or the largest
// centred squared norm: Alg. 2's y_i / (c R^2), v = 1, never forming R^2.  The accumulator of each
// tile is initialised with t_i + t_j, t_i = -a_i + (|mu|^2 - A - sqrt(d) ln c)/2, so that the
// exponent is a single multiply of the MFMA result.
#include "bkv_device.h"
#include "bkv_host.h"

namespace bkv {

template <typename T, int D> struct Geo {
    static constexpr int kRowBytes = D * (int)sizeof(T);
    static constexpr int kLdsRow = kRowBytes + 16;          // +16 B: conflict-free 16-byte reads
    static constexpr int kGroups = kRowBytes / 32;          // k-groups of 32 bytes per row
    static constexpr int kSlices = kRowBytes / 16;          // 16-byte slices per row
    static constexpr int kChunkRows = kRowBytes == 128 ? 1024 : (kRowBytes == 256 ? 512 : 256);
};

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;

size_t compress_lds_bytes(int row_bytes, int b) {
    int chunk_max = row_bytes == 128 ? 1024 : (row_bytes == 256 ? 512 : 256);
    int ch = b < chunk_max ? b : chunk_max;
    size_t bytes = (size_t)ch * (row_bytes + 16);
    if (bytes < 16384) bytes = 16384;   // the chunk region doubles as scratch for the mean reduction
    bytes += (size_t)b * 4 * 2;      // sigma, t
    bytes += 16 * 8;                 // eta masks
    bytes += (size_t)(b / 2) * 4;    // survivor list
    bytes += (size_t)row_bytes * 4;  // mu (fp32, at most row_bytes/2 entries; generous)
    bytes += 256;                    // scalars / wave partials
    return bytes;
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

    // acc[rb][cb] = t_row + t_col, then += A_I * B_J^T with B read from LDS rows ldsB[0..63].
    // Accumulator layout (32x32 MFMA): register r of lane (n,h) is row 8*(r/4) + 4*h + r%4, column n.
    static __device__ __forceinline__ void gram(floatx16 (&acc)[2][2], const Frag (&A)[G::kGroups][2],
                                                const char* ldsB, const float* t_rows,
                                                const float* t_cols, int n, int h) {
        float tc[2] = {t_cols[n], t_cols[32 + n]};
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                floatx4 tr = *reinterpret_cast<const floatx4*>(t_rows + 32 * rb + 8 * q + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[rb][0][4 * q + e] = tr[e] + tc[0];
                    acc[rb][1][4 * q + e] = tr[e] + tc[1];
                }
            }
#pragma unroll
        for (int g = 0; g < G::kGroups; ++g) {
            Frag b0 = *reinterpret_cast<const Frag*>(ldsB + (size_t)n * G::kLdsRow + 32 * g + 16 * h);
            Frag b1 = *reinterpret_cast<const Frag*>(ldsB + (size_t)(32 + n) * G::kLdsRow + 32 * g + 16 * h);
            Elem<T>::mma(acc[0][0], A[g][0], b0);
            Elem<T>::mma(acc[0][1], A[g][0], b1);
            Elem<T>::mma(acc[1][0], A[g][1], b0);
            Elem<T>::mma(acc[1][1], A[g][1], b1);
        }
    }
};


template <typename T, int D, bool EMIT_G>
__global__ __launch_bounds__(kThreads) void compress_kernel(const CompressArgs a) {
    typedef Geo<T, D> G;
    typedef TileOps<T, D> Ops;
    typedef typename Elem<T>::Frag Frag;
    constexpr int EPL = Elem<T>::kPerFrag;
    constexpr int SL = G::kSlices;
    constexpr int RG = kThreads / SL;

    extern __shared__ __align__(16) char smem[];
    const int b = a.b, nP = b >> 6, CH = a.chunk_rows;
    char* ldsK = smem;
    const size_t chunk_bytes = (size_t)CH * G::kLdsRow < 16384 ? 16384 : (size_t)CH * G::kLdsRow;
    float* sigma = reinterpret_cast<float*>(smem + chunk_bytes);
    float* tterm = sigma + b;
    unsigned long long* etaMask = reinterpret_cast<unsigned long long*>(tterm + b);
    int* keptIdx = reinterpret_cast<int*>(etaMask + 16);
    float* mu = reinterpret_cast<float*>(keptIdx + b / 2);
    float* scal = mu + D;                       // [0] |mu|^2, [1] A, [8..8+kWaves) wave partials
    float* scratch = reinterpret_cast<float*>(ldsK);   // aliases the key chunk before it is loaded

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t inst = blockIdx.x;
    const int64_t seq = inst / a.blocks_per_seq;
    const int blk = (int)(inst - seq * a.blocks_per_seq);
    const int64_t in_tok0 = seq * a.in_seq_stride + (int64_t)blk * b;          // first input token
    const int64_t out_tok0 = seq * a.out_seq_stride + (int64_t)blk * (b / 2);  // first output token
    const char* Kin = a.K + in_tok0 * G::kRowBytes;
    const int sl = tid % SL, rg = tid / SL;
    const bool center = (a.flags & BKV_CENTER_KEYS) != 0;

    // ------------------------------------------------------------------ block statistics
    // mu = mean key (fp32), a_i = <k_i, mu>, |k_i|^2, A = max centred squared norm.
    if (center) {
        float part[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) part[e] = 0.f;
        for (int i = rg; i < b; i += RG) {
            uintx4 raw = *reinterpret_cast<const uintx4*>(Kin + (size_t)i * G::kRowBytes + sl * 16);
            float f[EPL];
            Elem<T>::unpack(raw, f);
#pragma unroll
            for (int e = 0; e < EPL; ++e) part[e] += f[e];
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) scratch[rg * D + sl * EPL + e] = part[e];
        __syncthreads();
        if (tid < D) {
            float s = 0.f;
            for (int r = 0; r < RG; ++r) s += scratch[r * D + tid];
            mu[tid] = s / (float)b;
        }
        __syncthreads();
        if (wave == 0) {
            float s = 0.f;
            for (int c = lane; c < D; c += 64) s += mu[c] * mu[c];
            s = wave_sum(s);
            if (lane == 0) scal[0] = s;
        }
    } else {
        if (tid < D) mu[tid] = 0.f;
        if (tid == 0) scal[0] = 0.f;
    }
    __syncthreads();
    const float mumu = scal[0];
    {
        float mloc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) mloc[e] = mu[sl * EPL + e];
        float amax = -3.0e38f;
        const bool need_norm = !(a.rkey2 > 0.f);
        if (center || need_norm) {
            for (int i = rg; i < b; i += RG) {
                uintx4 raw = *reinterpret_cast<const uintx4*>(Kin + (size_t)i * G::kRowBytes + sl * 16);
                float f[EPL];
                Elem<T>::unpack(raw, f);
                float pa = 0.f, pn = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) { pa += f[e] * mloc[e]; pn += f[e] * f[e]; }
#pragma unroll
                for (int o = SL / 2; o > 0; o >>= 1) { pa += __shfl_xor(pa, o); pn += __shfl_xor(pn, o); }
                if (sl == 0) tterm[i] = pa;                       // a_i for now
                amax = fmaxf(amax, pn - 2.f * pa + mumu);
            }
            amax = wave_max(amax);
            if (lane == 0) scal[8 + wave] = amax;
        } else {
            for (int i = tid; i < b; i += kThreads) tterm[i] = 0.f;
        }
        __syncthreads();
        if (tid == 0) {
            float A = a.rkey2;
            if (need_norm) {
                A = scal[8];
                for (int w = 1; w < kWaves; ++w) A = fmaxf(A, scal[8 + w]);
            }
            scal[1] = A;
        }
        __syncthreads();
        const float half_const = 0.5f * (mumu - scal[1] + a.cterm);
        for (int i = tid; i < b; i += kThreads) {
            tterm[i] = half_const - tterm[i];
            sigma[i] = 0.f;
        }
    }
    // generator stream of this instance
    uint64_t stream = a.tree_mode ? (uint64_t)(64 * (a.seq_base + seq) + a.round) : (uint64_t)inst;
    if (a.inst_ids) stream = a.inst_ids[inst];
    const uint64_t key = stream_key(a.seed, stream);
    const uint64_t ctr0 = a.tree_mode ? (uint64_t)(a.blk_base + blk) * (uint64_t)b : 0ull;

    // walk statistics (wave 0)
    int n_margin = 0, any_fail = 0;
    float min_margin = 3.0e38f, max_sigma = 0.f;

    const int n_chunks = (b + CH - 1) / CH;
    for (int c = 0; c < n_chunks; ++c) {
        const int row0 = c * CH;                       // first row of the chunk
        const int p0 = row0 >> 6, p1 = min(nP, (row0 + CH) >> 6);
        __syncthreads();                               // previous users of ldsK / scratch are done
        for (int i = rg; i < CH && row0 + i < b; i += RG) {
            uintx4 raw = *reinterpret_cast<const uintx4*>(Kin + (size_t)(row0 + i) * G::kRowBytes + sl * 16);
            *reinterpret_cast<uintx4*>(ldsK + (size_t)i * G::kLdsRow + sl * 16) = raw;
        }
        __syncthreads();

        // ---------------------------------------------------------- rows of earlier chunks
        if (c > 0) {
            for (int J = p0 + wave; J < p1; J += kWaves) {
                const char* ldsB = ldsK + (size_t)((J << 6) - row0) * G::kLdsRow;
                float csum = 0.f;
                for (int I = 0; I < p0; ++I) {
                    Frag A[G::kGroups][2];
                    Ops::load_frags(A, Kin + (size_t)(I << 6) * G::kRowBytes, G::kRowBytes, n, h);
                    floatx16 acc[2][2];
                    Ops::gram(acc, A, ldsB, tterm + (I << 6), tterm + (J << 6), n, h);
                    const unsigned long long em = etaMask[I] >> (4 * h);
                    float cs0 = 0.f, cs1 = 0.f;
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int bit = 32 * rb + 8 * (r >> 2) + (r & 3);
                            const float sg = ((em >> bit) & 1ull) ? 1.f : -1.f;
                            const float v0 = fast_exp2(a.alpha * acc[rb][0][r]);
                            const float v1 = fast_exp2(a.alpha * acc[rb][1][r]);
                            cs0 = fmaf(sg, v0, cs0);
                            cs1 = fmaf(sg, v1, cs1);
                            if (EMIT_G) {
                                const int row = (I << 6) + bit + 4 * h;
                                float* Gi = a.G_out + (size_t)inst * b * b;
                                Gi[(size_t)row * b + (J << 6) + n] = v0;
                                Gi[(size_t)row * b + (J << 6) + 32 + n] = v1;
                                Gi[(size_t)((J << 6) + n) * b + row] = v0;
                                Gi[(size_t)((J << 6) + 32 + n) * b + row] = v1;
                            }
                        }
                    cs0 += __shfl_xor(cs0, 32);
                    cs1 += __shfl_xor(cs1, 32);
                    csum += h ? cs1 : cs0;
                }
                sigma[(J << 6) + lane] += csum;
            }
            __syncthreads();
        }

        // ---------------------------------------------------------- panels of this chunk
        for (int I = p0; I < p1; ++I) {
            const char* ldsA = ldsK + (size_t)((I << 6) - row0) * G::kLdsRow;
            if (wave == 0) {
                // diagonal tile -> one column per lane
                Frag A[G::kGroups][2];
                Ops::load_frags(A, ldsA, G::kLdsRow, n, h);
                floatx16 acc[2][2];
                Ops::gram(acc, A, ldsA, tterm + (I << 6), tterm + (I << 6), n, h);
                float g[64];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v0 = fast_exp2(a.alpha * acc[rb][0][r]);
                        const float v1 = fast_exp2(a.alpha * acc[rb][1][r]);
                        if (EMIT_G) {
                            const int row = (I << 6) + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
                            float* Gi = a.G_out + (size_t)inst * b * b;
                            Gi[(size_t)row * b + (I << 6) + n] = v0;
                            Gi[(size_t)row * b + (I << 6) + 32 + n] = v1;
                        }
                        // my column is 32*h + n: rows of pattern h are mine, pattern 1-h sit in lane^32
                        const float mine = h ? v1 : v0;
                        const float send = h ? v0 : v1;
                        const float recv = __shfl_xor(send, 32);
                        const int j_same = 32 * rb + 8 * (r >> 2) + (r & 3);   // + 4*h
                        // rows j_same + 4*h (mine) and j_same + 4*(1-h) (received)
                        g[j_same] = h ? recv : mine;          // row j_same     has pattern 0
                        g[j_same + 4] = h ? mine : recv;      // row j_same + 4 has pattern 1
                    }
#pragma unroll
                for (int j = 0; j < 64; ++j) g[j] = (j < lane) ? g[j] : 0.f;   // strictly earlier rows only

                float sv = sigma[(I << 6) + lane];
                float u;
                if (a.uniforms) u = a.uniforms[(size_t)inst * b + (I << 6) + lane];
                else u = (float)draw_bits_keyed(key, ctr0 + (uint64_t)((I << 6) + lane)) * (1.0f / 16777216.0f);
                const float tau = 1.f - 2.f * u;              // eta = +1  <=>  u < 1/2 - sigma/2  <=>  sigma < tau
#pragma unroll
                for (int j = 0; j < 64; ++j) {
                    const unsigned long long m = __ballot(sv < tau);
                    const float sg = ((m >> j) & 1ull) ? 1.f : -1.f;
                    sv = fmaf(sg, g[j], sv);
                }
                const unsigned long long m = __ballot(sv < tau);
                if (lane == 0) etaMask[I] = m;
                any_fail |= (__ballot(fabsf(sv) > 1.f) != 0ull);
                const float margin = 0.5f * fabsf(fminf(fmaxf(sv, -1.f), 1.f) - tau);   // |u - clamp(p)|
                n_margin += __popcll(__ballot(margin < 1e-4f));
                min_margin = fminf(min_margin, margin);
                max_sigma = fmaxf(max_sigma, fabsf(sv));
            }
            __syncthreads();
            if (I + 1 + wave < p1) {
                Frag A[G::kGroups][2];
                Ops::load_frags(A, ldsA, G::kLdsRow, n, h);
                const unsigned long long em = etaMask[I] >> (4 * h);
                float sgn[2][16];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sgn[rb][r] = ((em >> (32 * rb + 8 * (r >> 2) + (r & 3))) & 1ull) ? 1.f : -1.f;
                for (int J = I + 1 + wave; J < p1; J += kWaves) {
                    const char* ldsB = ldsK + (size_t)((J << 6) - row0) * G::kLdsRow;
                    floatx16 acc[2][2];
                    Ops::gram(acc, A, ldsB, tterm + (I << 6), tterm + (J << 6), n, h);
                    float cs0 = 0.f, cs1 = 0.f;
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float v0 = fast_exp2(a.alpha * acc[rb][0][r]);
                            const float v1 = fast_exp2(a.alpha * acc[rb][1][r]);
                            cs0 = fmaf(sgn[rb][r], v0, cs0);
                            cs1 = fmaf(sgn[rb][r], v1, cs1);
                            if (EMIT_G) {
                                const int row = (I << 6) + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
                                float* Gi = a.G_out + (size_t)inst * b * b;
                                Gi[(size_t)row * b + (J << 6) + n] = v0;
                                Gi[(size_t)row * b + (J << 6) + 32 + n] = v1;
                                Gi[(size_t)((J << 6) + n) * b + row] = v0;
                                Gi[(size_t)((J << 6) + 32 + n) * b + row] = v1;
                            }
                        }
                    cs0 += __shfl_xor(cs0, 32);
                    cs1 += __shfl_xor(cs1, 32);
                    sigma[(J << 6) + lane] += h ? cs1 : cs0;
                }
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ output step (Alg. 2 lines 12-16 + strict n/2)
    if (wave == 0) {
        int n_plus = 0;
        for (int p = 0; p < nP; ++p) n_plus += __popcll(etaMask[p]);
        const bool plus_is_minority = n_plus <= b - n_plus;               // tie -> '+'
        const int n_min = plus_is_minority ? n_plus : b - n_plus;
        const int need = b / 2 - n_min;                                   // majority tokens to add, lowest index first
        int maj_before = 0, kept_before = 0;
        const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        for (int p = 0; p < nP; ++p) {
            const unsigned long long m = etaMask[p];
            const unsigned long long minm = plus_is_minority ? m : ~m;
            const unsigned long long majm = ~minm;
            const int my_rank = maj_before + __popcll(majm & lt);
            const bool keep = ((minm >> lane) & 1ull) || (my_rank < need);
            const unsigned long long km = __ballot(keep);
            if (keep) keptIdx[kept_before + __popcll(km & lt)] = (p << 6) + lane;
            maj_before += __popcll(majm);
            kept_before += __popcll(km);
            if (a.signs_out) a.signs_out[(size_t)inst * b + (p << 6) + lane] = ((m >> lane) & 1ull) ? 1 : -1;
        }
        min_margin = wave_min(min_margin);
        max_sigma = wave_max(max_sigma);
        if (lane == 0) {
            const int word = (any_fail ? BKV_STATUS_FAIL : 0) | (n_margin << 8);
            if (a.status_out) {
                if (a.tree_mode) {
                    int* dst = a.status_out + seq * a.status_stride + a.round;
                    if (any_fail) atomicOr(dst, BKV_STATUS_FAIL);
                    if (n_margin) atomicAdd(dst, n_margin << 8);
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
    __syncthreads();
    const int half = b >> 1;
    if (a.K_out) {
        char* Ko = a.K_out + out_tok0 * G::kRowBytes;
        for (int r = rg; r < half; r += RG)
            *reinterpret_cast<uintx4*>(Ko + (size_t)r * G::kRowBytes + sl * 16) =
                *reinterpret_cast<const uintx4*>(Kin + (size_t)keptIdx[r] * G::kRowBytes + sl * 16);
    }
    if (a.V_out && a.V) {
        const char* Vin = a.V + in_tok0 * G::kRowBytes;
        char* Vo = a.V_out + out_tok0 * G::kRowBytes;
        for (int r = rg; r < half; r += RG)
            *reinterpret_cast<uintx4*>(Vo + (size_t)r * G::kRowBytes + sl * 16) =
                *reinterpret_cast<const uintx4*>(Vin + (size_t)keptIdx[r] * G::kRowBytes + sl * 16);
    }
    for (int r = tid; r < half; r += kThreads) {
        if (a.w_out) a.w_out[out_tok0 + r] = a.w_out_val;
        if (a.idx_out) {
            const int src = keptIdx[r];
            a.idx_out[seq * a.idx_out_seq_stride + (int64_t)blk * half + r] = a.idx_in ? a.idx_in[in_tok0 + src] : blk * b + src;
        }
    }
}

// ------------------------------------------------------------------------------------------------
template <typename T, int D, bool EMIT_G>
static hipError_t launch_one(const CompressArgs& a, int64_t n_inst, hipStream_t st) {
    const size_t lds = compress_lds_bytes(Geo<T, D>::kRowBytes, a.b);
    auto kern = compress_kernel<T, D, EMIT_G>;
    static thread_local size_t configured = 0;
    if (lds > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = lds;
    }
    ProfScope prof(kProfCompress, n_inst * a.b, st);
    hipLaunchKernelGGL(kern, dim3((unsigned)n_inst), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_compress(int dtype, int d, bool emit_g, CompressArgs& a, int64_t n_inst, hipStream_t st) {
    const int row_bytes = d * (dtype == BKV_BF16 ? 2 : 4);
    const int chunk_max = row_bytes == 128 ? 1024 : (row_bytes == 256 ? 512 : 256);
    a.chunk_rows = a.b < chunk_max ? a.b : chunk_max;
    if (n_inst <= 0) return hipSuccess;
    // grids are one-dimensional; split very large launches
    const int64_t kMaxGrid = 1ll << 30;
    if (n_inst > kMaxGrid) return hipErrorInvalidValue;
#define BKV_DISPATCH(TT, DD)                                                  \
    return emit_g ? launch_one<TT, DD, true>(a, n_inst, st) : launch_one<TT, DD, false>(a, n_inst, st)
    if (dtype == BKV_BF16 && d == 128) { BKV_DISPATCH(__bf16, 128); }
    if (dtype == BKV_BF16 && d == 64) { BKV_DISPATCH(__bf16, 64); }
    if (dtype == BKV_F32 && d == 128) { BKV_DISPATCH(float, 128); }
    if (dtype == BKV_F32 && d == 64) { BKV_DISPATCH(float, 64); }
#undef BKV_DISPATCH
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------------
// Row gather: out[seq, r, :] = in[seq, idx[seq, r], :]  (values of the final survivors).
// ------------------------------------------------------------------------------------------------
__global__ void gather_rows_kernel(const char* in, const int32_t* idx, char* out, int64_t in_seq_stride,
                                   int64_t out_seq_stride, int64_t rows_out, int row_bytes, int64_t total_slices) {
    const int slices = row_bytes >> 4;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total_slices;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = t / slices;
        const int s = (int)(t - row * slices);
        const int64_t seq = row / rows_out;
        const int64_t src = seq * in_seq_stride + idx[row];
        const int64_t dst = seq * out_seq_stride + (row - seq * rows_out);
        *reinterpret_cast<uintx4*>(out + (size_t)dst * row_bytes + s * 16) =
            *reinterpret_cast<const uintx4*>(in + (size_t)src * row_bytes + s * 16);
    }
}

hipError_t launch_gather_rows(const void* in, const int32_t* idx, void* out, int64_t n_seq, int64_t in_seq_stride,
                              int64_t out_seq_stride, int64_t rows_out, int row_bytes, hipStream_t st) {
    const int64_t total = n_seq * rows_out * (row_bytes >> 4);
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    ProfScope prof(kProfGather, n_seq * rows_out, st);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const char*)in, idx,
                       (char*)out, in_seq_stride, out_seq_stride, rows_out, row_bytes, total);
    return hipGetLastError();
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

// ------------------------------------------------------------------------------------------------
// Opt-in per-launch timing (diagnostics): HIP events recorded around kernel launches on the
// caller's stream.  Disabled unless bkv_profile_enable(n > 0) was called.
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
ProfScope::ProfScope(int kind, int64_t units, hipStream_t st) : slot_(-1), st_(st) {
    if (g_prof_n < g_prof_cap) {
        slot_ = g_prof_n++;
        g_prof[slot_].kind = kind; g_prof[slot_].units = units;
        (void)hipEventRecord(g_prof[slot_].a, st_);
    }
}
ProfScope::~ProfScope() {
    if (slot_ >= 0) (void)hipEventRecord(g_prof[slot_].b, st_);
}

}  // namespace bkv
