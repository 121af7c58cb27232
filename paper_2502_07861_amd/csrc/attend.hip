// Decode attention against the compressed, weighted cache (Alg. 1 output line of arXiv 2502.07861):
//   z = sum_i w_i e^{<k_i,q>/sqrt d} v_i / sum_i w_i e^{<k_i,q>/sqrt d},  w_i = 2^level(i).
// w_i e^x = 2^{x log2(e) + log2 w_i}: a softmax with logit bias log2 w_i, evaluated with a running
// maximum.  The pass is one stream over K, V, w (HBM bound): every lane owns a 16-byte slice of a
// row, a group of kSlices lanes owns a row, each wavefront covers 64/kSlices rows per step, and up to
// QT query vectors that share the KV sequence (GQA) are served from the same loads.  The token range
// is split over workgroups; partial (max, denominator, numerator) triples are merged by a second
// small kernel, which also emits the log-denominator so callers can merge further partials.
#include "bkv_device.h"
#include "bkv_host.h"

namespace bkv {

constexpr int kQT = 4;           // query vectors per pass over the cache
constexpr int kAttWaves = 4;
constexpr int kUnroll = 4;       // rows in flight per lane group
constexpr int kTargetWGs = 512;    // workgroups of the streaming pass when the token range is split (two per compute unit:
                                   // more only lengthen the merge, measured from 8 to 256 sequences)
constexpr float kNeg = -1.0e30f; // "minus infinity" that stays finite under subtraction

// HASV = false: the normaliser alone (Alg. 1's denominator sum over a set of its own): no value row is read, the
// output columns are zero, lse_out carries the result.
template <typename T, int D, bool HASV = true>
__global__ __launch_bounds__(kAttWaves * 64) void attend_partial_kernel(const AttendArgs a) {
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int SL = ROWB / 16;              // lanes per row
    constexpr int RPW = 64 / SL;               // rows per wavefront per step
    constexpr int EPL = Elem<T>::kPerFrag;     // elements per lane
    constexpr int ROWS_IT = kAttWaves * RPW * kUnroll;

    __shared__ float red[kAttWaves][kQT][D + 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sl = lane % SL, lg = lane / SL;
    const int split = blockIdx.x, qg = blockIdx.y;
    const int64_t seq = blockIdx.z;
    const int64_t r_begin = (int64_t)split * a.rows_per_split;
    const int64_t r_end = min(a.count, r_begin + a.rows_per_split);

    const char* Kb = a.K + (size_t)seq * a.stride_tokens * ROWB;
    const char* Vb = HASV ? a.V + (size_t)seq * a.stride_tokens * ROWB : nullptr;
    const float* wb = a.w + (size_t)seq * a.stride_tokens;

    // queries of this pass: raw 16-byte slices (bf16 path: consumed by packed dot products) and, for
    // fp32, the unpacked values; the logit scale log2(e)/sqrt(d) is applied to the reduced dot product
    uintx4 qraw[kQT];
#pragma unroll
    for (int qi = 0; qi < kQT; ++qi) {
        const int q = qg * kQT + qi;
        qraw[qi] = (q < a.n_q) ? *reinterpret_cast<const uintx4*>(a.Q + ((size_t)seq * a.n_q + q) * ROWB + sl * 16)
                               : uintx4{0u, 0u, 0u, 0u};
    }
    float m[kQT], l[kQT], o[kQT][EPL];
#pragma unroll
    for (int qi = 0; qi < kQT; ++qi) {
        m[qi] = kNeg; l[qi] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[qi][e] = 0.f;
    }

    struct Batch { uintx4 k[kUnroll], v[kUnroll]; float w[kUnroll]; };
    auto issue = [&](Batch& t, int64_t base) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t row = base + (u * kAttWaves + wave) * RPW + lg;
            const int64_t rr = row < r_end ? row : r_end - 1;          // stay in bounds; masked in consume()
            t.k[u] = *reinterpret_cast<const uintx4*>(Kb + (size_t)rr * ROWB + sl * 16);
            if constexpr (HASV) t.v[u] = *reinterpret_cast<const uintx4*>(Vb + (size_t)rr * ROWB + sl * 16);
            t.w[u] = wb[rr];
        }
    };
    auto consume = [&](const Batch& t, int64_t base) {
        float lg2[kUnroll][kQT];
        float mb[kQT];
#pragma unroll
        for (int qi = 0; qi < kQT; ++qi) mb[qi] = kNeg;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t row = base + (u * kAttWaves + wave) * RPW + lg;
            const bool live = row < r_end && t.w[u] > 0.f;
            const float bias = live ? __builtin_amdgcn_logf(t.w[u]) : 0.f;    // v_log_f32 = log2
#pragma unroll
            for (int qi = 0; qi < kQT; ++qi) {
                float part = Elem<T>::dot(qraw[qi], t.k[u]);
                part = group_sum<SL>(part);
                lg2[u][qi] = live ? fmaf(part, a.scale_log2, bias) : 2.f * kNeg;   // below every running maximum: weight 0
                mb[qi] = fmaxf(mb[qi], lg2[u][qi]);
            }
        }
        // a new running maximum rescales what has been accumulated; once the maxima have settled this is rare, and
        // the whole wavefront skips it
        bool grew = false;
#pragma unroll
        for (int qi = 0; qi < kQT; ++qi) grew |= mb[qi] > m[qi];
        if (__builtin_amdgcn_ballot_w64(grew) != 0ull) {
#pragma unroll
            for (int qi = 0; qi < kQT; ++qi) {
                const float mnew = fmaxf(m[qi], mb[qi]);
                const float sc = fast_exp2(m[qi] - mnew);
                m[qi] = mnew;
                l[qi] *= sc;
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[qi][e] *= sc;
            }
        }
        if constexpr (sizeof(T) == 2) {
            // bf16 values: two rows at a time on the packed dot product.  The weights p of the two rows are rounded to
            // bf16 (to nearest even, both in one v_cvt_pk_bf16_f32) and the denominator adds the same rounded values,
            // so numerator and denominator stay one estimator and the rounding errors carry no bias; element e of rows
            // a and b is paired by byte permutes, and o[e] += p_a v_a[e] + p_b v_b[e] is one v_dot2c_f32_bf16 (exact
            // products, fp32 sum) instead of two conversions and two multiply-adds.
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            static_assert(kUnroll % 2 == 0, "rows are consumed in pairs");
            const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int u = 0; u < kUnroll; u += 2) {
                bf16x2_t vp[EPL];
                if constexpr (HASV)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned int wa = t.v[u][i], wb = t.v[u + 1][i];
                    vp[2 * i] = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(wb, wa, 0x05040100u));       // (a[2i], b[2i])
                    vp[2 * i + 1] = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(wb, wa, 0x07060302u));   // (a[2i+1], b[2i+1])
                }
#pragma unroll
                for (int qi = 0; qi < kQT; ++qi) {
                    const floatx2 pf = {fast_exp2(lg2[u][qi] - m[qi]),            // dead rows: 2^(2 kNeg - m) = 0, m >= kNeg
                                        fast_exp2(lg2[u + 1][qi] - m[qi])};
                    const bf16x2_t pp = __builtin_convertvector(pf, bf16x2_t);     // (p_a, p_b)
                    l[qi] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, l[qi], false);
                    if constexpr (HASV) {
#pragma unroll
                        for (int e = 0; e < EPL; ++e) o[qi][e] = __builtin_amdgcn_fdot2_f32_bf16(pp, vp[e], o[qi][e], false);
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float vf[EPL];
                if constexpr (HASV) Elem<T>::unpack(t.v[u], vf);
#pragma unroll
                for (int qi = 0; qi < kQT; ++qi) {
                    const float p = fast_exp2(lg2[u][qi] - m[qi]);        // dead rows: 2^(2 kNeg - m) = 0, m >= kNeg
                    l[qi] += p;
                    if constexpr (HASV)
#pragma unroll
                        for (int e = 0; e < EPL; ++e) o[qi][e] = fmaf(p, vf[e], o[qi][e]);
                }
            }
        }
    };

    // two batches of rows in flight: the loads of the next batch are issued before the current one is consumed
    if (r_begin < r_end) {
        Batch b0, b1;
        issue(b0, r_begin);
        for (int64_t base = r_begin; base < r_end; base += 2 * ROWS_IT) {
            if (base + ROWS_IT < r_end) issue(b1, base + ROWS_IT);
            consume(b0, base);
            if (base + ROWS_IT < r_end) {
                if (base + 2 * ROWS_IT < r_end) issue(b0, base + 2 * ROWS_IT);
                consume(b1, base + ROWS_IT);
            }
        }
    }

    // merge the lane groups of a wavefront (each saw different rows)
#pragma unroll
    for (int off = SL; off < 64; off <<= 1) {
#pragma unroll
        for (int qi = 0; qi < kQT; ++qi) {
            const float mo = __shfl_xor(m[qi], off);
            const float lo = __shfl_xor(l[qi], off);
            const float mn = fmaxf(m[qi], mo);
            const float s0 = fast_exp2(m[qi] - mn), s1 = fast_exp2(mo - mn);
            l[qi] = l[qi] * s0 + lo * s1;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[qi][e] = o[qi][e] * s0 + __shfl_xor(o[qi][e], off) * s1;
            m[qi] = mn;
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int qi = 0; qi < kQT; ++qi) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) red[wave][qi][sl * EPL + e] = o[qi][e];
            if (sl == 0) { red[wave][qi][D] = m[qi]; red[wave][qi][D + 1] = l[qi]; }
        }
    }
    __syncthreads();
    if (a.n_splits == 1) {
        // The whole token range was one split: normalise and store the result here (the same arithmetic as partial +
        // merge, which is not launched then).
        for (int t = tid; t < kQT * D; t += kAttWaves * 64) {
            const int qi = t / D, c = t - qi * D;
            const int q = qg * kQT + qi;
            if (q >= a.n_q) continue;
            float M = red[0][qi][D];
#pragma unroll
            for (int w = 1; w < kAttWaves; ++w) M = fmaxf(M, red[w][qi][D]);
            float val = 0.f, L = 0.f;
#pragma unroll
            for (int w = 0; w < kAttWaves; ++w) {
                const float sc = fast_exp2(red[w][qi][D] - M);
                val += red[w][qi][c] * sc;
                L += red[w][qi][D + 1] * sc;
            }
            const float z = val * (L > 0.f ? 1.f / L : 0.f);
            const size_t oi = ((size_t)seq * a.n_q + q) * D + c;
            if (sizeof(T) == 2) reinterpret_cast<unsigned short*>(a.out)[oi] = (unsigned short)f32_to_bf16_bits(z);
            else reinterpret_cast<float*>(a.out)[oi] = z;
            if (c == 0 && a.lse_out)
                a.lse_out[(size_t)seq * a.n_q + q] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : -INFINITY;
        }
        return;
    }
    // merge the wavefronts and store the partial: [seq][qg][split][qi][D + 2]
    float* dst = a.partial + ((((size_t)seq * gridDim.y + qg) * a.n_splits + split) * kQT) * (D + 2);
    for (int t = tid; t < kQT * (D + 2); t += kAttWaves * 64) {
        const int qi = t / (D + 2), c = t - qi * (D + 2);
        float M = red[0][qi][D];
#pragma unroll
        for (int w = 1; w < kAttWaves; ++w) M = fmaxf(M, red[w][qi][D]);
        float val;
        if (c == D) val = M;
        else {
            val = 0.f;
#pragma unroll
            for (int w = 0; w < kAttWaves; ++w) val += red[w][qi][c] * fast_exp2(red[w][qi][D] - M);
        }
        dst[qi * (D + 2) + c] = val;
    }
}

// One workgroup (4 wavefronts) per (sequence, query): merge the split partials, normalise, store.  The numerator
// pass spreads the splits over the threads (a thread owns two columns and every SR-th split, several loads in
// flight), so its latency does not grow with the number of splits; the partial sums meet in LDS in a fixed order.
constexpr int kMergeThreads = 256;
constexpr int kScaleCache = 512;
template <typename T, int D>
__global__ __launch_bounds__(kMergeThreads) void attend_merge_kernel(const AttendArgs a, int n_qgroups) {
    constexpr int NW = kMergeThreads / 64;
    constexpr int CG = D / 2;                        // column pairs (the rows of a partial are 8-byte aligned)
    constexpr int SR = kMergeThreads / CG;           // splits summed side by side
    __shared__ float red[2 * NW];
    __shared__ float scale[kScaleCache];
    __shared__ float part[SR][D];
    const int64_t seq = blockIdx.y;
    const int q = blockIdx.x, tid = threadIdx.x, ns = a.n_splits;
    const int qg = q / kQT, qi = q % kQT;
    const float* src = a.partial + ((((size_t)seq * n_qgroups + qg) * ns) * kQT + qi) * (D + 2);
    const size_t sstride = (size_t)kQT * (D + 2);                  // between consecutive splits
    // largest running maximum over the splits
    float m = kNeg;
    for (int s = tid; s < ns; s += kMergeThreads) m = fmaxf(m, src[s * sstride + D]);
    m = wave_max(m);
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();
    float M = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, red[w]);
    // denominators, rescaled; the per-split factors are kept for the numerator pass
    float l = 0.f;
    for (int s = tid; s < ns; s += kMergeThreads) {
        const float sc = fast_exp2(src[s * sstride + D] - M);
        l = fmaf(src[s * sstride + D + 1], sc, l);
        if (s < kScaleCache) scale[s] = sc;
    }
    l = wave_sum(l);
    if ((tid & 63) == 0) red[NW + (tid >> 6)] = l;
    __syncthreads();
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) L += red[NW + w];
    const float inv = L > 0.f ? 1.f / L : 0.f;
    // numerators
    const int cg = tid % CG, sg = tid / CG;
    auto factor = [&](int s) -> float { return s < kScaleCache ? scale[s] : fast_exp2(src[s * sstride + D] - M); };
    float acc0 = 0.f, acc1 = 0.f;
    int s = sg;
    for (; s + 3 * SR < ns; s += 4 * SR) {                         // four independent loads in flight
        const floatx2 p0 = *reinterpret_cast<const floatx2*>(src + (size_t)s * sstride + 2 * cg);
        const floatx2 p1 = *reinterpret_cast<const floatx2*>(src + (size_t)(s + SR) * sstride + 2 * cg);
        const floatx2 p2 = *reinterpret_cast<const floatx2*>(src + (size_t)(s + 2 * SR) * sstride + 2 * cg);
        const floatx2 p3 = *reinterpret_cast<const floatx2*>(src + (size_t)(s + 3 * SR) * sstride + 2 * cg);
        const float f0 = factor(s), f1 = factor(s + SR), f2 = factor(s + 2 * SR), f3 = factor(s + 3 * SR);
        acc0 = fmaf(p0[0], f0, acc0); acc1 = fmaf(p0[1], f0, acc1);
        acc0 = fmaf(p1[0], f1, acc0); acc1 = fmaf(p1[1], f1, acc1);
        acc0 = fmaf(p2[0], f2, acc0); acc1 = fmaf(p2[1], f2, acc1);
        acc0 = fmaf(p3[0], f3, acc0); acc1 = fmaf(p3[1], f3, acc1);
    }
    for (; s < ns; s += SR) {
        const floatx2 p0 = *reinterpret_cast<const floatx2*>(src + (size_t)s * sstride + 2 * cg);
        const float f0 = factor(s);
        acc0 = fmaf(p0[0], f0, acc0); acc1 = fmaf(p0[1], f0, acc1);
    }
    part[sg][2 * cg] = acc0; part[sg][2 * cg + 1] = acc1;
    __syncthreads();
    for (int c = tid; c < D; c += kMergeThreads) {
        float z = 0.f;
#pragma unroll
        for (int r = 0; r < SR; ++r) z += part[r][c];
        z *= inv;
        const size_t oi = ((size_t)seq * a.n_q + q) * D + c;
        if (sizeof(T) == 2) reinterpret_cast<unsigned short*>(a.out)[oi] = (unsigned short)f32_to_bf16_bits(z);
        else reinterpret_cast<float*>(a.out)[oi] = z;
    }
    if (a.lse_out && tid == 0)
        a.lse_out[(size_t)seq * a.n_q + q] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : -INFINITY;
}

static void attend_plan(int d, int dtype_bytes, int64_t n_seq, int64_t count, int n_q, int* n_qg, int* n_splits,
                        int* rows_per_split) {
    const int sl = d * dtype_bytes / 16;
    const int rows_it = kAttWaves * (64 / sl) * kUnroll;
    *n_qg = (n_q + kQT - 1) / kQT;
    int64_t wgs = n_seq * (*n_qg);
    int64_t want = wgs > 0 ? (kTargetWGs + wgs - 1) / wgs : 1;
    int64_t max_splits = (count + rows_it - 1) / rows_it;      // a split is at least one batch of rows
    if (max_splits < 1) max_splits = 1;
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    int64_t rps = (count + want - 1) / want;
    rps = (rps + rows_it - 1) / rows_it * rows_it;
    if (rps < rows_it) rps = rows_it;
    int64_t ns = (count + rps - 1) / rps;
    if (ns < 1) ns = 1;
    *n_splits = (int)ns;
    *rows_per_split = (int)rps;
}

size_t attend_workspace_bytes(int d, int64_t n_seq, int n_q) {
    // the split count never exceeds ceil(kTargetWGs / workgroups-without-splitting), whatever the token count
    const int64_t n_qg = (n_q + kQT - 1) / kQT;
    const int64_t wgs = n_seq * n_qg;
    const int64_t ns = wgs > 0 ? (kTargetWGs + wgs - 1) / wgs : 1;
    return (size_t)(wgs * ns) * kQT * (d + 2) * sizeof(float) + 256;
}

template <typename T, int D>
static hipError_t launch_attend_t(AttendArgs& a, int64_t n_seq, int n_qg, hipStream_t st) {
    const dim3 grid(a.n_splits, n_qg, (unsigned)n_seq);
    const hipError_t e = a.V ? launch_timed(kProfAttend, n_seq * a.count, attend_partial_kernel<T, D, true>, grid, dim3(kAttWaves * 64), 0, st, a)
                             : launch_timed(kProfAttend, n_seq * a.count, attend_partial_kernel<T, D, false>, grid, dim3(kAttWaves * 64), 0, st, a);
    if (e != hipSuccess || a.n_splits == 1) return e;          // a single split stores the final result itself
    return launch_timed(kProfAttendMerge, n_seq * a.n_q, attend_merge_kernel<T, D>, dim3(a.n_q, (unsigned)n_seq), dim3(kMergeThreads), 0, st,
                        a, n_qg);
}

// Bytes of split partials that a launch with this shape writes (0 when the token range is a single split: the
// streaming pass then stores the result itself).
size_t attend_partial_bytes(int dtype, int d, int64_t n_seq, int64_t count, int n_q) {
    if (n_seq <= 0 || n_q <= 0) return 0;
    int n_qg, ns, rps;
    attend_plan(d, dtype == BKV_BF16 ? 2 : 4, n_seq, count, n_q, &n_qg, &ns, &rps);
    if (ns <= 1) return 0;
    return (size_t)n_seq * n_qg * ns * kQT * (d + 2) * sizeof(float);
}

// Scratch of the entry point that allocates nothing: the split partials live in this array instead of a caller's
// workspace.  Every GPU holds its own copy at its own address; host code uses the address that
// hipGetSymbolAddress returns for the current device, never the array's name.
static __device__ __align__(256) unsigned char scratch[kAttendStaticScratchBytes];
namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];           // per device, filled at the first call on that device
}
hipError_t attend_static_scratch(void** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_attend(int dtype, int d, AttendArgs& a, int64_t n_seq, void* workspace, hipStream_t st) {
    if (n_seq <= 0 || a.n_q <= 0) return hipSuccess;
    if (n_seq > 65535) return hipErrorInvalidValue;
    int n_qg, ns, rps;
    attend_plan(d, dtype == BKV_BF16 ? 2 : 4, n_seq, a.count, a.n_q, &n_qg, &ns, &rps);
    if (n_qg > 65535) return hipErrorInvalidValue;
    a.n_splits = ns;
    a.rows_per_split = rps;
    a.partial = reinterpret_cast<float*>(workspace);
    if (dtype == BKV_BF16 && d == 128) return launch_attend_t<__bf16, 128>(a, n_seq, n_qg, st);
    if (dtype == BKV_BF16 && d == 64) return launch_attend_t<__bf16, 64>(a, n_seq, n_qg, st);
    if (dtype == BKV_F32 && d == 128) return launch_attend_t<float, 128>(a, n_seq, n_qg, st);
    if (dtype == BKV_F32 && d == 64) return launch_attend_t<float, 64>(a, n_seq, n_qg, st);
    return hipErrorInvalidValue;
}

}  // namespace bkv
