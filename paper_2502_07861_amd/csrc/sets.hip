// Alg. 1 of arXiv 2502.07861 around the halving kernel: the stream of one sequence is split into buckets by the
// norm of the value rows (line 5), every bucket is a MergeAndReduce instance of its own with the value factor and
// value radius 2^i (MR-Numerator_i), negligible buckets are erased (line 8); the keys alone form one more instance
// (MR-Denominator).  Offline form: all tokens are there, so each instance is brought to the state Alg. 3 would have
// reached after its last token -- full blocks halved level by level, at most one half block left over per level, a
// tail of fewer than `block` tokens at level 0.
//
// A "segment" is the set of tokens of one (sequence, slot); slot 0 is the denominator instance, slot 256 + i is
// bucket i, slot 511 collects the rows that take no part (zero or non-finite norm, erased buckets).  Tokens are
// brought into slot order by a stable partition; the segment that starts at position `start` of that order occupies
// positions from start >> l of the level-l buffers (lengths shrink at least as fast as the starts, so segments never
// overlap).  Every round is ONE launch of the halving kernel over a table of instances (InstDesc).
#include "bkv_device.h"
#include "bkv_host.h"

namespace bkv {

namespace {

constexpr int kSlots = 512;
constexpr int kDenSlot = 0;
constexpr int kNumSlot0 = 256;
constexpr int kDropSlot = 511;
constexpr int kBucketMin = -60, kBucketMax = 60;      // 4^i stays a normal fp32 number

// |v|^2 of every value row (fp32 accumulation) and, when asked for, the largest one per sequence (blockIdx.y =
// sequence; one atomic per workgroup: atomics on one address are served one after the other).
template <typename T, int D>
__global__ __launch_bounds__(256) void value_norm_kernel(const char* V, int64_t n, float* norm2, unsigned int* vmax2_bits) {
    constexpr int RB = D * (int)sizeof(T);
    constexpr int SL = RB / 16;
    const int sl = threadIdx.x % SL;
    const int64_t seq = blockIdx.y;
    float best = 0.f;
    for (int64_t row = (int64_t)blockIdx.x * (256 / SL) + threadIdx.x / SL; row < n; row += (int64_t)gridDim.x * (256 / SL)) {
        const uintx4 raw = *reinterpret_cast<const uintx4*>(V + (size_t)(seq * n + row) * RB + sl * 16);
        const float x = group_sum<SL>(Elem<T>::dot(raw, raw));
        if (sl == 0) norm2[seq * n + row] = x;
        if (x < __builtin_inff()) best = fmaxf(best, x);
    }
    if (!vmax2_bits) return;
    __shared__ float wbest[4];
    best = wave_max(best);
    if ((threadIdx.x & 63) == 0) wbest[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        best = fmaxf(fmaxf(wbest[0], wbest[1]), fmaxf(wbest[2], wbest[3]));
        if (best > 0.f) atomicMax(vmax2_bits + seq, __float_as_uint(best));   // order of positive floats = order of their bits
    }
}

// Bucket of a value row with |v|^2 = x: the smallest i with 2^i >= |v| (Alg. 1 line 5), from the exponent of x,
// clamped to [kBucketMin, kBucketMax].  False: the row belongs to no bucket (zero or non-finite norm).
__device__ __forceinline__ bool bucket_of(float x, int& i) {
    if (!(x > 0.f && x < __builtin_inff())) return false;
    int e;
    const float m = frexpf(x, &e);                    // x = m 2^e, 1/2 <= m < 1
    const int ee = (m == 0.5f) ? e - 1 : e;           // smallest integer with 2^ee >= x
    i = ee >= 0 ? (ee + 1) / 2 : ee / 2;              // ceil(ee / 2): smallest i with 4^i >= x
    i = min(max(i, kBucketMin), kBucketMax);
    return true;
}

// Slot of every token: its bucket (Alg. 1 line 5);
// erased (line 8) when 4^i <= erase2 * max |v|^2.  Counts per (sequence, slot): blockIdx.y = sequence, a histogram per
// workgroup in LDS, one global atomic per workgroup and occupied slot.
__global__ __launch_bounds__(256) void slot_kernel(const float* norm2, const unsigned int* vmax2_bits, int64_t n, float erase2,
                                                   int32_t* slot, int32_t* cnt) {
    __shared__ int hist[kSlots];
    const int64_t seq = blockIdx.y;
    for (int s = threadIdx.x; s < kSlots; s += 256) hist[s] = 0;
    __syncthreads();
    const float limit = erase2 > 0.f ? erase2 * __uint_as_float(vmax2_bits[seq]) : 0.f;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < n; t += (int64_t)gridDim.x * 256) {
        int s = kDropSlot;
        const float x = norm2[seq * n + t];
        int i;
        if (bucket_of(x, i)) s = (ldexpf(1.f, 2 * i) <= limit) ? kDropSlot : kNumSlot0 + i;
        slot[seq * n + t] = s;
        atomicAdd(&hist[s], 1);
    }
    __syncthreads();
    for (int s = threadIdx.x; s < kSlots; s += 256)
        if (hist[s]) atomicAdd(cnt + seq * kSlots + s, hist[s]);
}

// the keys-only instance: one segment per sequence (slot 0) with all n tokens (the other counts are cleared before)
__global__ void single_segment_kernel(int32_t* cnt, int64_t n_seq, int32_t n) {
    const int64_t seq = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (seq < n_seq) cnt[seq * kSlots + kDenSlot] = n;
}

// exclusive prefix sum over the 64 lanes of a wavefront
__device__ __forceinline__ int wave_exclusive_sum(int x, int lane) {
    int incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    return incl - x;
}

// start[seq][slot] = tokens of the sequence in earlier slots.  One wavefront per sequence, eight slots per lane.
__global__ __launch_bounds__(64) void segment_start_kernel(const int32_t* cnt, int32_t* start) {
    const int64_t seq = blockIdx.x;
    const int lane = threadIdx.x;
    int c[8], sum = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) { c[k] = cnt[seq * kSlots + lane * 8 + k]; sum += c[k]; }
    int run = wave_exclusive_sum(sum, lane);
#pragma unroll
    for (int k = 0; k < 8; ++k) { start[seq * kSlots + lane * 8 + k] = run; run += c[k]; }
}

// The non-empty segments of a sequence (the slot that takes no part left out), ascending slot, as a list in LDS.
// Called by one wavefront; returns the length of the list.
__device__ __forceinline__ int list_segments(const int32_t* cnt, const int32_t* start, int64_t seq, int lane, int* lslot, int* lcnt,
                                             int* lstart) {
    int c[8], st[8], ne = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int s = lane * 8 + k;
        c[k] = s == kDropSlot ? 0 : cnt[seq * kSlots + s];
        st[k] = start[seq * kSlots + s];
        ne += c[k] > 0;
    }
    int at = wave_exclusive_sum(ne, lane);
    const int total = __shfl(at + ne, 63);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (c[k] > 0) { lslot[at] = lane * 8 + k; lcnt[at] = c[k]; lstart[at] = st[k]; ++at; }
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): the list is in LDS before the wavefront reads it
    __builtin_amdgcn_wave_barrier();
    return total;
}

// Stable partition of the tokens of a sequence by slot: perm[seq][start[slot] + rank among the slot's tokens] = token.
// One workgroup of sixteen wavefronts per sequence, 1024 tokens at a time: every wavefront counts its tokens per slot,
// a token's place is its slot's running base + the counts of the wavefronts before its own + its rank in its wavefront.
constexpr int kPartThreads = 1024, kPartWaves = kPartThreads / 64, kPartIds = 128;   // at most 123 slots are ever in use
__global__ __launch_bounds__(kPartThreads) void partition_kernel(const int32_t* slot, const int32_t* cnt, const int32_t* start,
                                                                 int64_t n, int32_t* perm) {
    __shared__ int cid[kSlots];                   // slot -> dense id of the non-empty slots
    __shared__ int cbase[kPartIds];               // next free position of every dense id
    __shared__ int wcnt[kPartWaves][kPartIds];
    __shared__ int wtot[kSlots / 64];
    const int64_t seq = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int i = tid; i < kPartWaves * kPartIds; i += kPartThreads) (&wcnt[0][0])[i] = 0;
    bool mine = false;
    unsigned long long present = 0ull;
    if (tid < kSlots) {
        mine = cnt[seq * kSlots + tid] > 0;
        present = __ballot(mine);
        if (lane == 0) wtot[wave] = (int)__popcll(present);
    }
    __syncthreads();
    if (tid < kSlots) {
        int id = (int)__popcll(present & lt);
        for (int w = 0; w < wave; ++w) id += wtot[w];
        cid[tid] = mine ? id : -1;
        if (mine && id < kPartIds) cbase[id] = start[seq * kSlots + tid];
    }
    __syncthreads();
    for (int64_t c0 = 0; c0 < n; c0 += kPartThreads) {
        const int64_t t = c0 + tid;
        int c = -1;
        if (t < n) c = cid[slot[seq * n + t]];
        const bool live = c >= 0 && c < kPartIds;
        int rank = 0;
        unsigned long long rem = __ballot(live);
        while (rem) {
            const int leader = __ffsll((long long)rem) - 1;
            const int lc = __shfl(c, leader);
            const unsigned long long same = __ballot(live && c == lc);
            if (live && c == lc) rank = (int)__popcll(same & lt);
            if (lane == leader) wcnt[wave][lc] = (int)__popcll(same);
            rem &= ~same;
        }
        __syncthreads();
        if (live) {
            int before = 0;
            for (int w = 0; w < wave; ++w) before += wcnt[w][c];
            perm[seq * n + cbase[c] + before + rank] = (int32_t)t;
        }
        __syncthreads();
        if (tid < kPartIds) {
            int tot = 0;
            for (int w = 0; w < kPartWaves; ++w) { tot += wcnt[w][tid]; wcnt[w][tid] = 0; }
            cbase[tid] += tot;
        }
        __syncthreads();
    }
}

// dst[seq, j, :] = src[seq, idx[seq, j], :] for j < min(rows, count[seq]) (count null: rows), zeros up to rows.
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* src, const int32_t* idx, char* dst, int64_t n_seq,
                                                          int64_t src_stride, int64_t idx_stride, int64_t dst_stride,
                                                          int64_t rows, const int32_t* count, int row_bytes) {
    const int slices = row_bytes >> 4;
    const int64_t total = n_seq * rows * slices;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t row = t / slices;
        const int s = (int)(t - row * slices);
        const int64_t seq = row / rows, j = row - seq * rows;
        uintx4 v = {0u, 0u, 0u, 0u};
        if (!count || j < count[seq])
            v = *reinterpret_cast<const uintx4*>(src + (size_t)(seq * src_stride + idx[seq * idx_stride + j]) * row_bytes + s * 16);
        *reinterpret_cast<uintx4*>(dst + (size_t)(seq * dst_stride + j) * row_bytes + s * 16) = v;
    }
}

struct SegGeo {
    int64_t n;            // tokens per sequence
    int32_t b, T;
    int64_t seq_base;
    int32_t numerator;    // 1: slots 256 + i carry r_value = 2^i
};

// Instance table of round r: for every segment its (full blocks >> r) blocks of `b` tokens of the level-r buffer,
// survivors to the level-(r+1) buffer.  One wavefront per sequence; unused entries of the grid are marked.
__global__ __launch_bounds__(64) void build_desc_kernel(const int32_t* cnt, const int32_t* start, SegGeo g, int r, int64_t max_inst,
                                                        InstDesc* desc) {
    __shared__ int lslot[kSlots], lcnt[kSlots], lstart[kSlots];
    const int64_t seq = blockIdx.x;
    const int lane = threadIdx.x;
    const int64_t stride_in = g.n >> r, stride_out = g.n >> (r + 1);
    const int n_seg = list_segments(cnt, start, seq, lane, lslot, lcnt, lstart);
    int64_t base = 0;
    for (int e = 0; e < n_seg; ++e) {
        const int s = lslot[e], c = lcnt[e], st = lstart[e];
        const int nb = (c / g.b) >> r;
        if (nb == 0) continue;
        const int64_t in0 = seq * stride_in + (st >> r), out0 = seq * stride_out + (st >> (r + 1));
        const float rv2 = (g.numerator && s >= kNumSlot0) ? ldexpf(1.f, 2 * (s - kNumSlot0)) : 0.f;
        for (int j = lane; j < nb; j += 64) {
            if (base + j < max_inst) {
                InstDesc d;
                d.in_tok = in0 + (int64_t)j * g.b;
                d.out_tok = out0 + (int64_t)j * (g.b / 2);
                d.stream = 64ull * ((uint64_t)(g.seq_base + seq) * kSlots + (uint64_t)s) + (uint64_t)r;
                d.ctr0 = (uint64_t)j * (uint64_t)g.b;
                d.seq = (int32_t)seq; d.valid = 1; d.rvalue2 = rv2; d.pad = 0;
                desc[seq * max_inst + base + j] = d;
            }
        }
        base += nb;
    }
    for (int64_t j = base + lane; j < max_inst; j += 64) {
        InstDesc d;
        d.in_tok = d.out_tok = 0; d.stream = d.ctr0 = 0; d.seq = 0; d.valid = 0; d.rvalue2 = 0.f; d.pad = 0;
        desc[seq * max_inst + j] = d;
    }
}

struct LevelIdx {
    const int32_t* lvl[32];     // lvl[l]: original index of every token of the level-l buffer, [n_seq, n >> l]; lvl[0] = perm
};

// The state of Alg. 3 of every segment, flattened: per slot the level-T tokens (weight 2^T), then the half block left
// at level T-1 ... 1 (weight 2^l), then the tail at level 0 (weight 1).  One wavefront per sequence.
__global__ __launch_bounds__(64) void collect_kernel(const int32_t* cnt, const int32_t* start, SegGeo g, LevelIdx L, int64_t capacity,
                                                     int32_t* idx_out, float* w_out, int32_t* count_out) {
    __shared__ int lslot[kSlots], lcnt[kSlots], lstart[kSlots];
    const int64_t seq = blockIdx.x;
    const int lane = threadIdx.x;
    const int T = g.T, half = g.b / 2;
    const int n_seg = list_segments(cnt, start, seq, lane, lslot, lcnt, lstart);
    int64_t pos = 0;
    auto emit = [&](const int32_t* src, int64_t m, float w) {
        for (int64_t j = lane; j < m; j += 64)
            if (pos + j < capacity) {
                if (idx_out) idx_out[seq * capacity + pos + j] = src[j];
                if (w_out) w_out[seq * capacity + pos + j] = w;
            }
        pos += m;
    };
    for (int e = 0; e < n_seg; ++e) {
        const int c = lcnt[e], st = lstart[e];
        const int full = T > 0 ? c / g.b : 0;
        if (T > 0) emit(L.lvl[T] + seq * (g.n >> T) + (st >> T), (int64_t)(full >> (T - 1)) * half, ldexpf(1.f, T));
        for (int l = T - 1; l >= 1; --l)
            if ((full >> (l - 1)) & 1)
                emit(L.lvl[l] + seq * (g.n >> l) + (st >> l) + (int64_t)(full >> l) * g.b, half, ldexpf(1.f, l));
        emit(L.lvl[0] + seq * g.n + st + (int64_t)full * g.b, c - full * g.b, 1.f);
    }
    if (lane == 0 && count_out) count_out[seq] = (int32_t)pos;
    for (int64_t j = pos + lane; j < capacity; j += 64) {
        if (idx_out) idx_out[seq * capacity + j] = 0;
        if (w_out) w_out[seq * capacity + j] = 0.f;
    }
}

// out[seq, q, :] *= exp(lse_num - lse_den): the numerator sum over one set divided by the denominator sum over another
template <typename T>
__global__ __launch_bounds__(256) void rescale_kernel(char* out, const float* lse_num, const float* lse_den, int64_t rows, int d) {
    const int64_t total = rows * d;
    T* o = reinterpret_cast<T*>(out);
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t row = t / d;
        const float ln = lse_num[row], ld = lse_den[row];
        const float f = (ln == -__builtin_inff()) ? 0.f : __expf(ln - ld);
        o[t] = (T)((float)o[t] * f);
    }
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }
inline unsigned grid_for(int64_t items, int per_block) {
    int64_t blocks = (items + per_block - 1) / per_block;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

}  // namespace

size_t sets_workspace_bytes(int row_bytes, int b, int64_t n_seq, int64_t n) {
    size_t s = 0;
    s += up256((size_t)n_seq * n * 4);                    // |v|^2
    s += up256((size_t)n_seq * n * 4);                    // slot of every token
    s += up256((size_t)n_seq * 4);                        // max |v|^2
    s += 2 * up256((size_t)n_seq * kSlots * 4);           // counts, starts
    s += 2 * up256((size_t)n_seq * n * 4);                // perm; original indices of the levels 1..T
    s += up256((size_t)n_seq * n * row_bytes);            // keys in slot order
    s += up256((size_t)n_seq * (n / 2) * row_bytes);      // level buffers, used in turn
    s += up256((size_t)n_seq * (n / 4) * row_bytes);
    s += up256((size_t)n_seq * (size_t)(n / b > 0 ? n / b : 1) * sizeof(InstDesc));
    return s;
}

hipError_t run_sets(const SetsArgs& q, hipStream_t st) {
    const int64_t n_seq = q.n_seq, n = q.n;
    const int rb = q.row_bytes, b = q.b, T = q.T;
    char* ws = (char*)q.workspace;
    auto carve = [&](size_t bytes) { char* p = ws; ws += up256(bytes); return p; };
    float* norm2 = (float*)carve((size_t)n_seq * n * 4);
    int32_t* slot_ws = (int32_t*)carve((size_t)n_seq * n * 4);
    unsigned int* vmax2 = (unsigned int*)carve((size_t)n_seq * 4);
    int32_t* cnt = (int32_t*)carve((size_t)n_seq * kSlots * 4);
    int32_t* start = (int32_t*)carve((size_t)n_seq * kSlots * 4);
    int32_t* perm = (int32_t*)carve((size_t)n_seq * n * 4);
    int32_t* lvl_idx = (int32_t*)carve((size_t)n_seq * n * 4);
    char* k_sorted = carve((size_t)n_seq * n * rb);
    char* k_a = carve((size_t)n_seq * (n / 2) * rb);
    char* k_b = carve((size_t)n_seq * (n / 4) * rb);
    InstDesc* desc = (InstDesc*)carve((size_t)n_seq * (size_t)(n / b > 0 ? n / b : 1) * sizeof(InstDesc));
    int32_t* slot = q.slot_out ? q.slot_out : slot_ws;
    hipError_t e;

    // ---- segments
    if ((e = launch_fill_u32(cnt, 0u, n_seq * kSlots, st)) != hipSuccess) return e;
    const char* k0;                      // level-0 keys, slot order (or the original keys, read through perm)
    bool first_by_idx = false;

    if (q.numerator) {
        if ((e = launch_fill_u32(vmax2, 0u, n_seq, st)) != hipSuccess) return e;
        const dim3 g1(grid_for(n, 256 / (rb / 16)) > 256 ? 256 : grid_for(n, 256 / (rb / 16)), (unsigned)n_seq);
        unsigned int* vmax_arg = q.erase2 > 0.f ? vmax2 : nullptr;      // only the erase rule needs the largest norm
        if (q.dtype == BKV_BF16 && q.d == 128) hipLaunchKernelGGL((value_norm_kernel<__bf16, 128>), g1, dim3(256), 0, st, q.V, n, norm2, vmax_arg);
        else if (q.dtype == BKV_BF16 && q.d == 64) hipLaunchKernelGGL((value_norm_kernel<__bf16, 64>), g1, dim3(256), 0, st, q.V, n, norm2, vmax_arg);
        else if (q.dtype == BKV_F32 && q.d == 128) hipLaunchKernelGGL((value_norm_kernel<float, 128>), g1, dim3(256), 0, st, q.V, n, norm2, vmax_arg);
        else if (q.dtype == BKV_F32 && q.d == 64) hipLaunchKernelGGL((value_norm_kernel<float, 64>), g1, dim3(256), 0, st, q.V, n, norm2, vmax_arg);
        else return hipErrorInvalidValue;
        if ((e = hipGetLastError()) != hipSuccess) return e;
        const unsigned gs = grid_for(n, 4096) > 64 ? 64 : grid_for(n, 4096);
        hipLaunchKernelGGL(slot_kernel, dim3(gs, (unsigned)n_seq), dim3(256), 0, st, norm2, vmax2, n, q.erase2, slot, cnt);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(segment_start_kernel, dim3((unsigned)n_seq), dim3(64), 0, st, cnt, start);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(partition_kernel, dim3((unsigned)n_seq), dim3(kPartThreads), 0, st, slot, cnt, start, n, perm);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        // blocks resident as one chunk read their key rows through perm (no copy in slot order); larger blocks need the copy
        if (!compress_block_resident(rb, b, true)) {
            hipLaunchKernelGGL(gather_rows_kernel, dim3(grid_for(n_seq * n * (rb / 16), 256)), dim3(256), 0, st, q.K, perm, k_sorted, n_seq,
                               n, n, n, n, (const int32_t*)nullptr, rb);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            k0 = k_sorted;
        } else {
            k0 = q.K;
            first_by_idx = true;
        }
    } else {
        // one segment per sequence (slot 0), already in order
        hipLaunchKernelGGL(single_segment_kernel, dim3(grid_for(n_seq, 64)), dim3(64), 0, st, cnt, n_seq, (int32_t)n);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (q.slot_out && (e = launch_fill_u32(q.slot_out, (uint32_t)kDenSlot, n_seq * n, st)) != hipSuccess) return e;
        hipLaunchKernelGGL(segment_start_kernel, dim3((unsigned)n_seq), dim3(64), 0, st, cnt, start);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if ((e = launch_fill_iota(perm, n_seq, n, 0, n, 0, st)) != hipSuccess) return e;
        k0 = q.K;
    }

    // ---- rounds
    LevelIdx L;
    for (int l = 0; l < 32; ++l) L.lvl[l] = nullptr;
    L.lvl[0] = perm;
    {
        int32_t* p = lvl_idx;
        for (int l = 1; l <= T; ++l) { L.lvl[l] = p; p += n_seq * (n >> l); }
    }
    SegGeo g;
    g.n = n; g.b = b; g.T = T; g.seq_base = q.seq_base; g.numerator = q.numerator;
    const char* k_in = k0;
    int64_t signs_off = 0;
    for (int r = 0; r < T; ++r) {
        const int64_t max_inst = (n / b) >> r;
        if (max_inst == 0) break;                 // no segment has a block at this level any more
        hipLaunchKernelGGL(build_desc_kernel, dim3((unsigned)n_seq), dim3(64), 0, st, cnt, start, g, r, max_inst, desc);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        CompressArgs a = q.common;
        a.desc = desc;
        a.K = k_in;
        a.k_by_idx = (r == 0 && first_by_idx) ? 1 : 0;
        a.K_out = (r == T - 1) ? nullptr : ((r & 1) ? k_b : k_a);      // the last level's keys are gathered from the originals
        a.V = q.numerator ? q.V : nullptr;
        a.V_out = nullptr; a.w_out = nullptr;
        a.v_seq_stride = n;
        a.idx_in = L.lvl[r];
        a.idx_out = const_cast<int32_t*>(L.lvl[r + 1]);
        a.signs_out = q.signs_out ? q.signs_out + signs_off : nullptr;
        a.status_out = q.status_out; a.status_stride = T;
        a.tree_mode = 1; a.round = r;
        a.blocks_per_seq = 1;
        if ((e = launch_compress(q.dtype, q.d, false, a, n_seq * max_inst, st)) != hipSuccess) return e;
        k_in = a.K_out;
        signs_off += n_seq * (n >> r);
    }

    // ---- the kept sets
    hipLaunchKernelGGL(collect_kernel, dim3((unsigned)n_seq), dim3(64), 0, st, cnt, start, g, L, q.capacity, q.idx_ws, q.w_out, q.count_out);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (q.capacity > 0) {
        const unsigned gg = grid_for(n_seq * q.capacity * (rb / 16), 256);
        if (q.K_out) {
            hipLaunchKernelGGL(gather_rows_kernel, dim3(gg), dim3(256), 0, st, q.K, q.idx_ws, q.K_out, n_seq, n, q.capacity, q.capacity,
                               q.capacity, (const int32_t*)q.count_out, rb);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if (q.V_out) {
            hipLaunchKernelGGL(gather_rows_kernel, dim3(gg), dim3(256), 0, st, q.V, q.idx_ws, q.V_out, n_seq, n, q.capacity, q.capacity,
                               q.capacity, (const int32_t*)q.count_out, rb);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_rescale(int dtype, void* out, const float* lse_num, const float* lse_den, int64_t rows, int d, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    const unsigned gg = grid_for(rows * d, 256);
    if (dtype == BKV_BF16) hipLaunchKernelGGL(rescale_kernel<__bf16>, dim3(gg), dim3(256), 0, st, (char*)out, lse_num, lse_den, rows, d);
    else hipLaunchKernelGGL(rescale_kernel<float>, dim3(gg), dim3(256), 0, st, (char*)out, lse_num, lse_den, rows, d);
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------------ Alg. 1 token by token
namespace {

constexpr int kFreeRegion = INT32_MIN;

// Lines 4-12 of Alg. 1 for one token per sequence, up to the halvings themselves.  One wavefront per sequence:
//  * |v|^2, the running maximum and the erase limit (line 8): regions whose bucket has 4^i <= limit are given back;
//  * the token's bucket (line 5) -> its region (a free one on the bucket's first token) -> the row goes to the tail of
//    the region with weight 1 (line 7 feeds MR-Numerator_i); the key goes to the denominator region (line 11);
//  * the carry loop of Alg. 3 for both instances as a table: round r of this token halves the last `b` stored tokens
//    of the region as they will stand after the rounds before it (each takes b/2 away), draws from the instance's
//    stream at level r, block number = blocks that reached level r before.
// Lane l < regions looks after region l.
template <typename T, int D>
__global__ __launch_bounds__(64) void stream_route_kernel(StreamState s, const char* k, const char* v, int32_t j) {
    constexpr int RB = D * (int)sizeof(T);
    constexpr int SL = RB / 16;
    const int64_t seq = blockIdx.x;
    const int lane = threadIdx.x;
    const int R = s.regions, b = s.b, half = s.b / 2, Tn = s.T;
    uintx4 kraw = {0u, 0u, 0u, 0u}, vraw = {0u, 0u, 0u, 0u};
    if (lane < SL) {
        kraw = *reinterpret_cast<const uintx4*>(k + (size_t)seq * RB + lane * 16);
        vraw = *reinterpret_cast<const uintx4*>(v + (size_t)seq * RB + lane * 16);
    }
    const float x = __shfl(group_sum<SL>(Elem<T>::dot(vraw, vraw)), 0);          // |v|^2, fp32
    float vm = __uint_as_float(s.vmax2[seq]);
    if (x < __builtin_inff() && x > vm) {
        vm = x;
        if (lane == 0) s.vmax2[seq] = __float_as_uint(vm);
    }
    const float limit = s.erase2 > 0.f ? s.erase2 * vm : 0.f;

    // ---- line 8: erase the negligible buckets (lane l keeps region l's bucket and counters in registers; they are
    // written back once, at the end)
    int bk = lane < R ? s.bucket[seq * R + lane] : kFreeRegion;
    int my_cnt = lane < R ? s.cnt[seq * (R + 1) + lane] : 0;
    int my_jj = lane < R ? s.jj[seq * (R + 1) + lane] : 0;
    const bool gone = bk != kFreeRegion && ldexpf(1.f, 2 * bk) <= limit;
    unsigned long long erased = __ballot(gone);
    while (erased) {
        const int e = __ffsll((long long)erased) - 1;
        erased &= erased - 1;
        const int c = __shfl(my_cnt, e);
        float* w = s.wn + (size_t)(seq * R + e) * s.cap_n;
        for (int t = lane; t < c; t += 64) w[t] = 0.f;
    }
    if (gone) { bk = kFreeRegion; my_cnt = 0; my_jj = 0; }

    // ---- lines 5-7: the token's bucket and region
    int i = 0;
    int reg = 0;
    bool take = bucket_of(x, i) && !(ldexpf(1.f, 2 * i) <= limit);      // a token of a negligible bucket is dropped at once
    if (take) {
        const unsigned long long hit = __ballot(bk == i);
        if (hit) reg = __ffsll((long long)hit) - 1;
        else {
            const unsigned long long vacant = __ballot(lane < R && bk == kFreeRegion);
            if (vacant) {
                reg = __ffsll((long long)vacant) - 1;
                if (lane == reg) bk = i;                         // counters of a free region are 0
            } else {
                take = false;
                if (lane == 0) atomicOr(s.err, BKV_STREAM_NO_REGION);
            }
        }
    }
    int pos_n = __shfl(my_cnt, reg);
    if (take && pos_n >= s.cap_n) {
        take = false;
        if (lane == 0) atomicOr(s.err, BKV_STREAM_NUM_FULL);
    }
    int carries_n = 0, blocks_n = 0;
    if (take) {
        const size_t at = (size_t)(seq * R + reg) * s.cap_n + pos_n;
        if (lane < SL) {
            *reinterpret_cast<uintx4*>(s.Kn + at * RB + lane * 16) = kraw;
            *reinterpret_cast<uintx4*>(s.Vn + at * RB + lane * 16) = vraw;
        }
        if (lane == 0) { s.wn[at] = 1.f; s.on[at] = j; }
        const int seen = __shfl(my_jj, reg) + 1;
        pos_n += 1;
        if (lane == reg) { my_cnt = pos_n; my_jj = seen; }
        if (Tn > 0 && seen % b == 0) {
            blocks_n = seen / b;
            carries_n = min(Tn, __ffs(blocks_n));               // rounds r < T with blocks_n divisible by 2^r
        }
    }
    if (lane < R) {
        s.bucket[seq * R + lane] = bk;
        s.cnt[seq * (R + 1) + lane] = my_cnt;
        s.jj[seq * (R + 1) + lane] = my_jj;
    }

    // ---- line 11: the key alone goes to MR-Denominator
    int pos_d = s.cnt[seq * (R + 1) + R];
    int carries_d = 0, blocks_d = 0;
    if (pos_d >= s.cap_d) {
        if (lane == 0) atomicOr(s.err, BKV_STREAM_DEN_FULL);
    } else {
        const size_t at = (size_t)seq * s.cap_d + pos_d;
        if (lane < SL) *reinterpret_cast<uintx4*>(s.Kd + at * RB + lane * 16) = kraw;
        const int seen = s.jj[seq * (R + 1) + R] + 1;
        if (lane == 0) {
            s.wd[at] = 1.f; s.od[at] = j;
            s.cnt[seq * (R + 1) + R] = pos_d + 1;
            s.jj[seq * (R + 1) + R] = seen;
        }
        pos_d += 1;
        if (Tn > 0 && seen % b == 0) {
            blocks_d = seen / b;
            carries_d = min(Tn, __ffs(blocks_d));
        }
    }

    // ---- the carries of this token, round by round (lanes 0..T-1: numerator, 32..32+T-1: denominator)
    const int r = lane & 31, kind = lane >> 5;
    if (r < Tn) {
        InstDesc ds;
        ds.in_tok = ds.out_tok = 0; ds.stream = ds.ctr0 = 0; ds.seq = (int32_t)seq; ds.valid = 0; ds.rvalue2 = 0.f; ds.pad = 0;
        const int carries = kind ? carries_d : carries_n;
        if (r < carries) {
            const int64_t region0 = kind ? seq * s.cap_d : (seq * R + reg) * s.cap_n;
            const int64_t first = (kind ? pos_d : pos_n) - (int64_t)r * half - b;
            const uint64_t slot = kind ? (uint64_t)kDenSlot : (uint64_t)(kNumSlot0 + i);
            ds.in_tok = region0 + first;
            ds.out_tok = seq * half;
            ds.stream = 64ull * ((uint64_t)(s.seq_base + seq) * kSlots + slot) + (uint64_t)r;
            ds.ctr0 = (uint64_t)(((kind ? blocks_d : blocks_n) >> r) - 1) * (uint64_t)b;
            ds.valid = 1;
            ds.rvalue2 = kind ? 0.f : ldexpf(1.f, 2 * i);
            ds.pad = kind ? R : reg;
        }
        s.desc[((int64_t)r * 2 + kind) * s.n_seq + seq] = ds;
    }
}

// After the halvings of round r: the survivors (rows, original indices) go back to the front of the block they came
// from with weight 2^(r+1), the rest of the block is marked absent and the region shrinks by half a block.
__global__ __launch_bounds__(256) void stream_fixup_kernel(StreamState s, int r) {
    __shared__ int32_t so[512];
    const int64_t seq = blockIdx.x;
    const int kind = blockIdx.y, tid = threadIdx.x;
    const InstDesc ds = s.desc[((int64_t)r * 2 + kind) * s.n_seq + seq];
    if (!ds.valid) return;
    const int half = s.b / 2, rb = s.row_bytes, slices = rb >> 4;
    char* K = kind ? s.Kd : s.Kn;
    float* w = kind ? s.wd : s.wn;
    int32_t* o = kind ? s.od : s.on;
    const int64_t frame = kind ? seq * s.cap_d : seq * (int64_t)s.regions * s.cap_n;      // first place of the sequence
    const int64_t first = ds.in_tok;
    const size_t t0 = (size_t)(kind * s.n_seq + seq) * half;
    const int32_t* ti = s.tmpIdx + t0;
    for (int t = tid; t < half; t += 256) so[t] = o[frame + ti[t]];
    __syncthreads();
    const float wnew = ldexpf(1.f, r + 1);
    for (int t = tid; t < half; t += 256) {
        o[first + t] = so[t];
        w[first + t] = wnew;
        w[first + half + t] = 0.f;
    }
    for (int t = tid; t < half * slices; t += 256) {
        const int row = t / slices, sl = t - row * slices;
        const size_t src = (t0 + row) * rb + sl * 16, dst = (size_t)(first + row) * rb + sl * 16;
        *reinterpret_cast<uintx4*>(K + dst) = *reinterpret_cast<const uintx4*>(s.tmpK + src);
        if (!kind) *reinterpret_cast<uintx4*>(s.Vn + dst) = *reinterpret_cast<const uintx4*>(s.tmpV + src);
    }
    if (tid == 0) s.cnt[seq * (s.regions + 1) + ds.pad] -= half;
}

}  // namespace

hipError_t stream_route(const StreamState& s, const void* k, const void* v, int64_t j, hipStream_t st) {
    const dim3 grid((unsigned)s.n_seq), block(64);
    const char* kp = (const char*)k;
    const char* vp = (const char*)v;
    if (s.dtype == BKV_BF16 && s.d == 128) hipLaunchKernelGGL((stream_route_kernel<__bf16, 128>), grid, block, 0, st, s, kp, vp, (int32_t)j);
    else if (s.dtype == BKV_BF16 && s.d == 64) hipLaunchKernelGGL((stream_route_kernel<__bf16, 64>), grid, block, 0, st, s, kp, vp, (int32_t)j);
    else if (s.dtype == BKV_F32 && s.d == 128) hipLaunchKernelGGL((stream_route_kernel<float, 128>), grid, block, 0, st, s, kp, vp, (int32_t)j);
    else if (s.dtype == BKV_F32 && s.d == 64) hipLaunchKernelGGL((stream_route_kernel<float, 64>), grid, block, 0, st, s, kp, vp, (int32_t)j);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t stream_fixup(const StreamState& s, int round, hipStream_t st) {
    hipLaunchKernelGGL(stream_fixup_kernel, dim3((unsigned)s.n_seq, 2u), dim3(256), 0, st, s, round);
    return hipGetLastError();
}

}  // namespace bkv
