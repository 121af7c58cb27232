// C ABI of libbalancekv: argument validation, workspace carving, launch orchestration, and the
// host-side bookkeeping of Alg. 3 (arXiv 2502.07861).  Every step of the path runs in the kernels of
// compress.hip / attend.hip; nothing here touches tensor contents on the host.
#include <math.h>
#include <new>
#include <string.h>

#include "bkv_device.h"
#include "bkv_host.h"

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return BKV_EHIP;
}
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_params(const bkv_params* p) {
    if (!p) return BKV_EINVAL;
    if (p->reserved != 0) return BKV_EINVAL;
    if (p->d != 64 && p->d != 128) return BKV_ESHAPE;
    if (p->block < 64 || p->block > 1024 || (p->block & 63)) return BKV_ESHAPE;
    if (p->rounds < 0 || p->rounds > 30) return BKV_ESHAPE;
    if (p->dtype != BKV_F32 && p->dtype != BKV_BF16) return BKV_ESHAPE;
    if (p->flags & ~(BKV_CENTER_KEYS | BKV_STRICT_HALF | BKV_VALUE_GRAM | BKV_VALUE_AUGMENT)) return BKV_EINVAL;
    if ((p->flags & BKV_VALUE_AUGMENT) && !(p->flags & BKV_VALUE_GRAM)) return BKV_EINVAL;    // an option of the value factor
    if (!(p->flags & BKV_STRICT_HALF)) return BKV_ESHAPE;      // variable-size output not built
    if (isnan(p->log_c) && !(p->delta > 0.f && p->delta < (float)p->block)) return BKV_EINVAL;
    return BKV_OK;
}
inline int elem_bytes(const bkv_params* p) { return p->dtype == BKV_BF16 ? 2 : 4; }
inline int row_bytes(const bkv_params* p) { return p->d * elem_bytes(p); }

// ln c: given, or c = 30 ln(block/delta) (Alg. 2 line 3 with n = the block handed to the call)
inline float resolve_log_c(const bkv_params* p) {
    if (!isnan(p->log_c)) return p->log_c;
    return logf(30.0f * logf((float)p->block / p->delta));
}

void fill_common(bkv::CompressArgs& a, const bkv_params* p) {
    memset(&a, 0, sizeof(a));
    a.b = p->block;
    a.seed = p->seed;
    a.flags = p->flags;
    a.alpha = (float)(1.4426950408889634 / sqrt((double)p->d));
    a.cterm = (float)(-sqrt((double)p->d) * (double)resolve_log_c(p));
    a.rkey2 = p->r_key > 0.f ? p->r_key * p->r_key : 0.f;
    a.rvalue2 = p->r_value > 0.f ? p->r_value * p->r_value : 0.f;
}

}  // namespace

struct bkv_stream {
    bkv_params p;
    bkv::StreamState s;
    int64_t seen;         // tokens appended per sequence
};

struct bkv_cache {
    bkv_params p;
    int64_t n_seq, cap;
    char* K;
    char* V;
    float* w;
    int64_t count;        // stored tokens per sequence
    int64_t base_count;   // adopted survivors (never touched by carries)
    int64_t stream_j;     // tokens appended since init/load (the j of Alg. 3)
    int32_t* err;         // device word behind the weights: sticky BKV_STATUS_INTERNAL of every halving run for this cache
};

extern "C" {

const char* bkv_version(void) { return "balancekv-gfx950 0.1"; }

const char* bkv_error_string(int code) {
    switch (code) {
        case BKV_OK: return "ok";
        case BKV_EINVAL: return "invalid argument";
        case BKV_ESHAPE: return "unsupported shape, dtype or mode";
        case BKV_EWORKSPACE: return "workspace missing or too small";
        case BKV_EHIP: return "HIP error";
        case BKV_ECAPACITY: return "cache capacity exceeded";
        default: return "unknown";
    }
}

int bkv_last_hip_error(void) { return g_last_hip_error; }

uint32_t bkv_uniform_bits(uint64_t seed, uint64_t stream, uint64_t ctr) { return bkv::draw_bits(seed, stream, ctr); }

// ------------------------------------------------------------------------------------------ Alg. 2
size_t bkv_compress_workspace_bytes(const bkv_params* p, int64_t n_inst) {
    (void)p; (void)n_inst;
    return 0;
}

int bkv_compress_block(const bkv_params* p, const void* K, const void* V, int64_t n_inst,
                       const uint64_t* inst_ids, float w_in, const float* uniforms, void* K_out, void* V_out,
                       float* w_out, int32_t* idx_out, int8_t* signs_out, int32_t* status_out, float* stats_out,
                       void* workspace, size_t ws_bytes, void* hip_stream) {
    (void)workspace; (void)ws_bytes;
    int rc = check_params(p);
    if (rc) return rc;
    if (n_inst < 0) return BKV_EINVAL;
    if (n_inst == 0) return BKV_OK;
    if (!K || !aligned16(K) || (K_out && !aligned16(K_out))) return BKV_EINVAL;
    if (V_out && (!V || !aligned16(V) || !aligned16(V_out))) return BKV_EINVAL;
    if ((p->flags & BKV_VALUE_GRAM) && (!V || !aligned16(V))) return BKV_EINVAL;
    if (!(w_in > 0.f)) return BKV_EINVAL;
    bkv::CompressArgs a;
    fill_common(a, p);
    a.K = (const char*)K; a.V = (const char*)V; a.K_out = (char*)K_out; a.V_out = (char*)V_out;
    a.w_out = w_out; a.idx_out = idx_out; a.signs_out = signs_out; a.status_out = status_out; a.stats_out = stats_out;
    a.inst_ids = inst_ids; a.uniforms = uniforms;
    a.in_seq_stride = a.v_seq_stride = p->block; a.out_seq_stride = a.idx_out_seq_stride = p->block / 2;
    a.blocks_per_seq = 1; a.tree_mode = 0; a.w_out_val = 2.f * w_in;
    hipError_t e = bkv::launch_compress(p->dtype, p->d, false, a, n_inst, (hipStream_t)hip_stream);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

int bkv_kernel_weights(const bkv_params* p, const void* K, int64_t n_inst, float* G_out, void* hip_stream) {
    int rc = check_params(p);
    if (rc) return rc;
    if (n_inst < 0) return BKV_EINVAL;
    if (n_inst == 0) return BKV_OK;
    if (!K || !aligned16(K) || !G_out) return BKV_EINVAL;
    if (p->flags & BKV_VALUE_GRAM) return BKV_ESHAPE;          // the dump takes no values
    bkv::CompressArgs a;
    fill_common(a, p);
    a.K = (const char*)K; a.G_out = G_out;
    a.in_seq_stride = p->block; a.out_seq_stride = a.idx_out_seq_stride = p->block / 2; a.blocks_per_seq = 1;
    a.w_out_val = 2.f;
    hipError_t e = bkv::launch_compress(p->dtype, p->d, true, a, n_inst, (hipStream_t)hip_stream);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

// ------------------------------------------------------------------------------------------ Alg. 3 offline
// workspace: K ping [n_seq, n/2, d] | K pong [n_seq, n/4, d] | idx ping [n_seq, n/2] | idx pong [n_seq, n/4]
size_t bkv_merge_reduce_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t n) {
    if (check_params(p) || n_seq < 0 || n < 0) return 0;
    if (p->rounds <= 1) return align_up((size_t)n_seq * (n / 2) * 4, 256) + 256;   // survivor indices only
    const size_t rb = (size_t)row_bytes(p);
    size_t bytes = 0;
    bytes += align_up((size_t)n_seq * (n / 2) * rb, 256);
    bytes += align_up((size_t)n_seq * (n / 4) * rb, 256);
    bytes += align_up((size_t)n_seq * (n / 2) * 4, 256);
    bytes += align_up((size_t)n_seq * (n / 4) * 4, 256);
    return bytes + 256;
}

}  // extern "C"

// T rounds; the last round writes K_out / V_out / w_out with `out_stride` tokens between sequences
// (idx_out, if given, is always dense [n_seq, n >> T]).
// The n tokens halved may be a window of longer sequences: K points at the window's first row, rows of consecutive
// sequences are k_stride tokens apart (0: n); V points at token 0 of the first sequence, v_stride tokens apart (0: n),
// and the window starts at token idx_base; idx_out rows are idx_out_stride apart (0: n >> T).
struct TreeWindow { int64_t k_stride, v_stride, idx_base, idx_out_stride; };
static int merge_reduce_impl(const bkv_params* p, const void* K, const void* V, int64_t n_seq, int64_t n,
                             int64_t seq_base, void* K_out, void* V_out, float* w_out, int64_t out_stride,
                             int32_t* idx_out, int8_t* signs_out, int32_t* status_out, void* workspace,
                             size_t ws_bytes, void* hip_stream, const TreeWindow* win = nullptr,
                             int32_t* sticky_err = nullptr) {
    const int64_t k_stride = win && win->k_stride ? win->k_stride : n;
    const int64_t v_stride = win && win->v_stride ? win->v_stride : n;
    const int64_t idx_base = win ? win->idx_base : 0;
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq < 0 || n < 0 || seq_base < 0) return BKV_EINVAL;
    const int T = p->rounds, b = p->block;
    if (n % ((int64_t)b << T) != 0) return BKV_ESHAPE;
    if (n_seq == 0 || n == 0) return BKV_OK;
    if (n_seq * (n / b) > (1ll << 30) || n > (1ll << 31) - 1) return BKV_ESHAPE;
    if (!K || !V || !K_out || !V_out) return BKV_EINVAL;
    if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out)) return BKV_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t rb = (size_t)row_bytes(p);
    hipError_t e;
    if (T == 0) {   // nothing to halve: weights 1
        if (idx_out) return BKV_ESHAPE;   // identity indices are not materialised
        const char* Vwin = (const char*)V + (size_t)idx_base * rb;
        if ((e = bkv::launch_copy_rows(K, K_out, n_seq, k_stride, out_stride, n, (int)rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_rows(Vwin, V_out, n_seq, v_stride, out_stride, n, (int)rb, st)) != hipSuccess) return hip_fail(e);
        if (w_out && (e = bkv::launch_fill_w(w_out, n_seq, out_stride, 0, n, 1.f, st)) != hipSuccess) return hip_fail(e);
        return BKV_OK;
    }
    const size_t need = bkv_merge_reduce_workspace_bytes(p, n_seq, n);
    char* kbuf[2] = {nullptr, nullptr};
    int32_t* ibuf[2] = {nullptr, nullptr};
    int32_t* idx_final = idx_out;
    if (T > 1) {
        if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
        char* ws = (char*)workspace;
        kbuf[0] = ws; ws += align_up((size_t)n_seq * (n / 2) * rb, 256);
        kbuf[1] = ws; ws += align_up((size_t)n_seq * (n / 4) * rb, 256);
        ibuf[0] = (int32_t*)ws; ws += align_up((size_t)n_seq * (n / 2) * 4, 256);
        ibuf[1] = (int32_t*)ws;
    }
    if (!idx_final) {     // the value gather needs the survivor indices even if the caller does not
        if (T > 1) idx_final = ibuf[(T - 1) & 1];      // free at the last round (its input is the other one)
        else {                                         // T == 1: a small index buffer from the workspace
            if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
            idx_final = (int32_t*)workspace;
        }
    }
    if (status_out && (e = bkv::launch_fill_u32(status_out, 0u, n_seq * T, st)) != hipSuccess) return hip_fail(e);

    const char* k_in = (const char*)K;
    const int32_t* i_in = nullptr;
    int64_t m = n;
    for (int r = 0; r < T; ++r) {
        const bool last = (r == T - 1);
        bkv::CompressArgs a;
        fill_common(a, p);
        a.K = k_in;
        a.K_out = last ? (char*)K_out : kbuf[r & 1];
        // values are gathered once, from the original rows; the value factor reads them (by original index) in every round
        a.V = (last || (p->flags & BKV_VALUE_GRAM)) ? (const char*)V : nullptr;
        a.V_out = last ? (char*)V_out : nullptr;
        a.v_seq_stride = v_stride;
        a.idx_base = idx_base;
        a.w_out = last ? w_out : nullptr;
        a.idx_in = i_in;
        a.idx_out = last ? idx_final : ibuf[r & 1];
        a.signs_out = signs_out ? signs_out + (size_t)n_seq * (size_t)(2 * n - ((2 * n) >> r)) : nullptr;
        a.status_out = status_out; a.status_stride = T; a.sticky_err = sticky_err;
        a.in_seq_stride = r == 0 ? k_stride : m; a.out_seq_stride = last ? out_stride : m / 2;
        a.idx_out_seq_stride = (last && idx_out && win && win->idx_out_stride) ? win->idx_out_stride : m / 2;
        a.blocks_per_seq = (int32_t)(m / b);
        a.tree_mode = 1; a.round = r; a.seq_base = seq_base; a.blk_base = 0;
        a.w_out_val = (float)(1u << (r + 1));
        e = bkv::launch_compress(p->dtype, p->d, false, a, n_seq * (m / b), st);
        if (e != hipSuccess) return hip_fail(e);
        k_in = a.K_out; i_in = a.idx_out; m /= 2;
    }
    return BKV_OK;
}

extern "C" {

int bkv_merge_reduce(const bkv_params* p, const void* K, const void* V, int64_t n_seq, int64_t n,
                     int64_t seq_base, void* K_out, void* V_out, float* w_out, int32_t* idx_out,
                     int8_t* signs_out, int32_t* status_out, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!p) return BKV_EINVAL;
    return merge_reduce_impl(p, K, V, n_seq, n, seq_base, K_out, V_out, w_out, n >> (p->rounds & 31), idx_out,
                             signs_out, status_out, workspace, ws_bytes, hip_stream);
}

int bkv_merge_reduce_protected(const bkv_params* p, const void* K, const void* V, int64_t n_seq, int64_t n,
                               int64_t n_sink, int64_t n_recent, int64_t seq_base, void* K_out, void* V_out, float* w_out,
                               int32_t* idx_out, int32_t* status_out, void* workspace, size_t ws_bytes, void* hip_stream) {
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq < 0 || n < 0 || n_sink < 0 || n_recent < 0 || n_sink + n_recent > n || seq_base < 0) return BKV_EINVAL;
    const int T = p->rounds;
    const int64_t n_mid = n - n_sink - n_recent;
    if (n_mid % ((int64_t)p->block << T) != 0 || n > (1ll << 31) - 1) return BKV_ESHAPE;
    if (n_seq == 0 || n == 0) return BKV_OK;
    if (!K || !V || !K_out || !V_out || !aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out)) return BKV_EINVAL;
    const int64_t kept_mid = n_mid >> T, count = n_sink + kept_mid + n_recent;
    if (n_mid > 0 && (T > 1 || (T == 1 && !idx_out))) {      // what the tree will ask for, before anything is launched
        const size_t need = bkv_merge_reduce_workspace_bytes(p, n_seq, n_mid);
        if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
    }
    const size_t rb = (size_t)row_bytes(p);
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    // the two windows: copies of the original rows, weight 1, their own indices
    const int64_t from[2] = {0, n - n_recent}, to[2] = {0, count - n_recent}, rows[2] = {n_sink, n_recent};
    for (int k = 0; k < 2; ++k) {
        const char* Ks = (const char*)K + (size_t)from[k] * rb;
        const char* Vs = (const char*)V + (size_t)from[k] * rb;
        if ((e = bkv::launch_copy_rows(Ks, (char*)K_out + (size_t)to[k] * rb, n_seq, n, count, rows[k], (int)rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_rows(Vs, (char*)V_out + (size_t)to[k] * rb, n_seq, n, count, rows[k], (int)rb, st)) != hipSuccess) return hip_fail(e);
        if (w_out && (e = bkv::launch_fill_w(w_out, n_seq, count, to[k], rows[k], 1.f, st)) != hipSuccess) return hip_fail(e);
        if (idx_out && (e = bkv::launch_fill_iota(idx_out, n_seq, count, to[k], rows[k], (int32_t)from[k], st)) != hipSuccess) return hip_fail(e);
    }
    if (n_mid == 0) {   // nothing to halve: no events to report
        if (status_out && T > 0 && (e = bkv::launch_fill_u32(status_out, 0u, n_seq * T, st)) != hipSuccess) return hip_fail(e);
        return BKV_OK;
    }
    if (T == 0) {       // the rows in between are kept as they are too
        if (idx_out && (e = bkv::launch_fill_iota(idx_out, n_seq, count, n_sink, n_mid, (int32_t)n_sink, st)) != hipSuccess) return hip_fail(e);
        idx_out = nullptr;
    }
    const TreeWindow win = {n, n, n_sink, count};
    return merge_reduce_impl(p, (const char*)K + (size_t)n_sink * rb, V, n_seq, n_mid, seq_base, (char*)K_out + (size_t)n_sink * rb,
                             (char*)V_out + (size_t)n_sink * rb, w_out ? w_out + n_sink : nullptr, count,
                             idx_out ? idx_out + n_sink : nullptr, nullptr, status_out, workspace, ws_bytes, hip_stream, &win);
}

int bkv_profile_enable(int32_t max_records) { return bkv::prof_enable(max_records) == 0 ? BKV_OK : BKV_EHIP; }
int bkv_profile_read(int32_t* kind, float* ms, int64_t* units, int32_t cap) {
    if (!kind || !ms || !units || cap < 0) return BKV_EINVAL;
    return bkv::prof_read(kind, ms, units, cap);
}

int bkv_measure_peak(int32_t kind, int32_t launches, void* workspace, size_t ws_bytes, void* hip_stream,
                     double* per_second, double* ms_per_launch) {
    if (kind < BKV_PEAK_MFMA_BF16 || kind > BKV_PEAK_STREAM_COPY || launches <= 0 || !per_second || !ms_per_launch) return BKV_EINVAL;
    if (!workspace || !aligned16(workspace) || ws_bytes < ((size_t)8 << 20)) return BKV_EWORKSPACE;
    const hipError_t e = bkv::measure_peak(kind, launches, workspace, ws_bytes, (hipStream_t)hip_stream, per_second, ms_per_launch);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

// ------------------------------------------------------------------------------------------ estimator
size_t bkv_attend_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t count, int32_t g, int32_t nq) {
    if (check_params(p) || n_seq < 0 || count < 0 || g <= 0 || nq <= 0) return 0;
    return bkv::attend_workspace_bytes(p->d, n_seq, g * nq);
}

}  // extern "C"

// exact_need: the workspace need only hold what this very launch writes (else: the public, count-independent bound)
static int attend_kv_impl(const bkv_params* p, const void* K_c, const void* V_c, const float* w, int64_t n_seq,
                          int64_t count, int64_t stride_tokens, const void* Q, int32_t g, int32_t nq, void* out,
                          float* lse_out, void* workspace, size_t ws_bytes, bool exact_need, void* hip_stream) {
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq < 0 || count < 0 || stride_tokens < count || g <= 0 || nq <= 0) return BKV_EINVAL;
    if (n_seq == 0) return BKV_OK;
    if (n_seq > 65535 || (int64_t)g * nq > 4 * 65535) return BKV_ESHAPE;
    if (!Q || !out || !aligned16(Q) || !aligned16(out)) return BKV_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    const int n_q = g * nq;
    if (count == 0) {   // empty cache: zeros, lse = -inf
        const int64_t words = n_seq * n_q * (int64_t)row_bytes(p) / 4;
        if ((e = bkv::launch_fill_u32(out, 0u, words, st)) != hipSuccess) return hip_fail(e);
        if (lse_out && (e = bkv::launch_fill_u32(lse_out, 0xff800000u, n_seq * n_q, st)) != hipSuccess) return hip_fail(e);
        return BKV_OK;
    }
    if (!K_c || !V_c || !w || !aligned16(K_c) || !aligned16(V_c)) return BKV_EINVAL;
    const size_t need = exact_need ? bkv::attend_partial_bytes(p->dtype, p->d, n_seq, count, n_q)
                                   : bkv::attend_workspace_bytes(p->d, n_seq, n_q);
    if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
    bkv::AttendArgs a;
    memset(&a, 0, sizeof(a));
    a.K = (const char*)K_c; a.V = (const char*)V_c; a.w = w; a.Q = (const char*)Q; a.out = (char*)out;
    a.lse_out = lse_out; a.stride_tokens = stride_tokens; a.count = count; a.n_q = n_q;
    a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)p->d));
    e = bkv::launch_attend(p->dtype, p->d, a, n_seq, workspace, st);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

extern "C" {

int bkv_attend_kv(const bkv_params* p, const void* K_c, const void* V_c, const float* w, int64_t n_seq,
                  int64_t count, int64_t stride_tokens, const void* Q, int32_t g, int32_t nq, void* out,
                  float* lse_out, void* workspace, size_t ws_bytes, void* hip_stream) {
    return attend_kv_impl(p, K_c, V_c, w, n_seq, count, stride_tokens, Q, g, nq, out, lse_out, workspace, ws_bytes, false,
                          hip_stream);
}

size_t bkv_attend_kv_static_max_bytes(void) { return bkv::kAttendStaticScratchBytes; }

int bkv_attend_kv_static(const bkv_params* p, const void* K_c, const void* V_c, const float* w, int64_t n_seq,
                         int64_t count, int64_t stride_tokens, const void* Q, int32_t g, int32_t nq, void* out,
                         float* lse_out, void* hip_stream) {
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq < 0 || count < 0 || g <= 0 || nq <= 0) return BKV_EINVAL;
    if (n_seq > 65535 || (int64_t)g * nq > 4 * 65535) return BKV_ESHAPE;
    // what this launch would write into the partial buffer must fit the library's static array
    if (bkv::attend_partial_bytes(p->dtype, p->d, n_seq, count, g * nq) > bkv::kAttendStaticScratchBytes) return BKV_EWORKSPACE;
    void* ws = nullptr;
    const hipError_t e = bkv::attend_static_scratch(&ws);
    if (e != hipSuccess) return hip_fail(e);
    // The partials of a launch are written in full before its merge reads them, so nothing has to be cleared between
    // calls; two calls in flight on one GPU at the same time would share the array and race.
    return attend_kv_impl(p, K_c, V_c, w, n_seq, count, stride_tokens, Q, g, nq, out, lse_out, ws,
                          bkv::kAttendStaticScratchBytes, true, hip_stream);
}

// ------------------------------------------------------------------------------------------ Alg. 1: buckets, two instances
int64_t bkv_sets_capacity(const bkv_params* p, int64_t n, int32_t max_buckets) {
    if (check_params(p) || n < 0 || max_buckets < 1) return 0;
    // per instance: level-T survivors (at most its share of n >> T), one half block per level below, a tail < block
    const int64_t per = (int64_t)p->block + (int64_t)(p->rounds > 1 ? p->rounds - 1 : 0) * (p->block / 2);
    const int64_t cap = (n >> p->rounds) + (int64_t)max_buckets * per;
    return cap < n ? cap : n;
}

size_t bkv_balancekv_sets_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t n, int64_t capacity) {
    if (check_params(p) || n_seq < 0 || n < 0 || capacity < 0) return 0;
    return bkv::sets_workspace_bytes(row_bytes(p), p->block, n_seq, n) + align_up((size_t)n_seq * capacity * 4, 256) +
           align_up((size_t)n_seq * 4, 256) + 256;
}

int bkv_balancekv_sets(const bkv_params* p_in, int32_t which, const void* K, const void* V, int64_t n_seq, int64_t n,
                       int64_t seq_base, float eps, float r, void* K_out, void* V_out, float* w_out, int32_t* idx_out,
                       int64_t capacity, int32_t* count_out, int32_t* slot_out, int8_t* signs_out, int32_t* status_out,
                       void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!p_in) return BKV_EINVAL;
    if (which != BKV_SET_NUMERATOR && which != BKV_SET_DENOMINATOR) return BKV_EINVAL;
    bkv_params p = *p_in;
    p.flags = which == BKV_SET_NUMERATOR ? (p.flags | BKV_VALUE_GRAM) : (p.flags & ~(BKV_VALUE_GRAM | BKV_VALUE_AUGMENT));
    int rc = check_params(&p);
    if (rc) return rc;
    if (n_seq < 0 || n < 0 || seq_base < 0 || capacity < 0 || !(r >= 0.f)) return BKV_EINVAL;
    if (n > (1ll << 30) || n_seq > 65535 || n_seq * (n / p.block + 1) > (1ll << 30)) return BKV_ESHAPE;
    if (n_seq == 0) return BKV_OK;
    if (n > 0 && (!K || !aligned16(K))) return BKV_EINVAL;
    if (n > 0 && (which == BKV_SET_NUMERATOR || V_out) && (!V || !aligned16(V))) return BKV_EINVAL;
    if ((K_out && !aligned16(K_out)) || (V_out && !aligned16(V_out))) return BKV_EINVAL;
    const size_t need = bkv_balancekv_sets_workspace_bytes(&p, n_seq, n, capacity);
    if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    const int T = p.rounds;
    if (status_out && (e = bkv::launch_fill_u32(status_out, 0u, n_seq * (T > 0 ? T : 1), st)) != hipSuccess) return hip_fail(e);
    bkv::SetsArgs q;
    memset(&q, 0, sizeof(q));
    fill_common(q.common, &p);
    q.K = (const char*)K; q.V = (const char*)V;
    q.n_seq = n_seq; q.n = n; q.seq_base = seq_base; q.capacity = capacity;
    q.dtype = p.dtype; q.d = p.d; q.row_bytes = row_bytes(&p); q.b = p.block; q.T = T;
    q.numerator = which == BKV_SET_NUMERATOR;
    q.erase2 = 0.f;
    if (eps > 0.f && n > 0) {
        const double f = (double)eps / (2.0 * (double)n) * exp(-(double)r * (double)r / sqrt((double)p.d));
        q.erase2 = (float)(f * f);
    }
    q.K_out = (char*)K_out; q.V_out = (char*)V_out; q.w_out = w_out;
    char* ws = (char*)workspace;
    q.idx_ws = idx_out;
    if (!q.idx_ws) { q.idx_ws = (int32_t*)ws; }
    ws += align_up((size_t)n_seq * capacity * 4, 256);
    q.count_out = count_out;
    if (!q.count_out) { q.count_out = (int32_t*)ws; }
    ws += align_up((size_t)n_seq * 4, 256);
    q.slot_out = slot_out; q.signs_out = signs_out; q.status_out = status_out;
    q.workspace = ws;
    e = bkv::run_sets(q, st);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

size_t bkv_attend_sets_workspace_bytes(const bkv_params* p, int64_t n_seq, int32_t g, int32_t nq) {
    if (check_params(p) || n_seq < 0 || g <= 0 || nq <= 0) return 0;
    const size_t rows = (size_t)n_seq * g * nq;
    return align_up(bkv::attend_workspace_bytes(p->d, n_seq, g * nq), 256) + 2 * align_up(rows * 4, 256) +
           align_up(rows * (size_t)row_bytes(p), 256);
}

int bkv_attend_sets(const bkv_params* p, const void* K_n, const void* V_n, const float* w_n, int64_t count_n, int64_t stride_n,
                    const void* K_d, const float* w_d, int64_t count_d, int64_t stride_d, int64_t n_seq, const void* Q,
                    int32_t g, int32_t nq, void* out, float* lse_out, void* workspace, size_t ws_bytes, void* hip_stream) {
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq < 0 || g <= 0 || nq <= 0 || count_n < 0 || count_d < 0) return BKV_EINVAL;
    if (count_d == 0 && count_n > 0) return BKV_EINVAL;
    if (n_seq == 0) return BKV_OK;
    const size_t need = bkv_attend_sets_workspace_bytes(p, n_seq, g, nq);
    if (!workspace || ws_bytes < need || !aligned16(workspace)) return BKV_EWORKSPACE;
    const size_t rows = (size_t)n_seq * g * nq;
    char* ws = (char*)workspace;
    void* att_ws = ws;
    const size_t att_bytes = align_up(bkv::attend_workspace_bytes(p->d, n_seq, g * nq), 256);
    ws += att_bytes;
    float* lse_n = (float*)ws; ws += align_up(rows * 4, 256);
    float* lse_d = (float*)ws; ws += align_up(rows * 4, 256);
    void* scratch = ws;
    // numerator sum / its own normaliser, then the normaliser of the denominator set (no value rows are read for it)
    rc = bkv_attend_kv(p, K_n, V_n, w_n, n_seq, count_n, stride_n, Q, g, nq, out, lse_n, att_ws, att_bytes, hip_stream);
    if (rc) return rc;
    float* lse_den = lse_out ? lse_out : lse_d;
    hipError_t e;
    if (count_d == 0) {
        if ((e = bkv::launch_fill_u32(lse_den, 0xff800000u, (int64_t)rows, (hipStream_t)hip_stream)) != hipSuccess) return hip_fail(e);
    } else {
        if (stride_d < count_d || !K_d || !w_d || !aligned16(K_d) || !Q || !aligned16(Q)) return BKV_EINVAL;
        bkv::AttendArgs a;
        memset(&a, 0, sizeof(a));
        a.K = (const char*)K_d; a.V = nullptr; a.w = w_d; a.Q = (const char*)Q; a.out = (char*)scratch;
        a.lse_out = lse_den; a.stride_tokens = stride_d; a.count = count_d; a.n_q = g * nq;
        a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)p->d));
        if ((e = bkv::launch_attend(p->dtype, p->d, a, n_seq, att_ws, (hipStream_t)hip_stream)) != hipSuccess) return hip_fail(e);
    }
    e = bkv::launch_rescale(p->dtype, out, lse_n, lse_den, (int64_t)rows, p->d, (hipStream_t)hip_stream);
    return e == hipSuccess ? BKV_OK : hip_fail(e);
}

// ------------------------------------------------------------------------------------------ Alg. 3 streaming
size_t bkv_cache_bytes(const bkv_params* p, int64_t n_seq, int64_t max_tokens) {
    if (check_params(p) || n_seq <= 0 || max_tokens < p->block) return 0;
    const size_t rb = (size_t)row_bytes(p);
    return 2 * align_up((size_t)n_seq * max_tokens * rb, 256) + align_up((size_t)n_seq * max_tokens * 4, 256) + 256;
}

int bkv_cache_init(bkv_cache** out, const bkv_params* p, int64_t n_seq, int64_t max_tokens, void* device_storage,
                   size_t bytes, void* hip_stream) {
    if (!out) return BKV_EINVAL;
    *out = nullptr;
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq <= 0 || n_seq > 65535 || max_tokens < p->block) return BKV_EINVAL;
    const size_t need = bkv_cache_bytes(p, n_seq, max_tokens);
    if (!device_storage || (reinterpret_cast<uintptr_t>(device_storage) & 255u) || bytes < need) return BKV_EINVAL;
    bkv_cache* c = new (std::nothrow) bkv_cache;
    if (!c) return BKV_EINVAL;
    c->p = *p; c->n_seq = n_seq; c->cap = max_tokens;
    const size_t rb = (size_t)row_bytes(p);
    const size_t kv = align_up((size_t)n_seq * max_tokens * rb, 256);
    c->K = (char*)device_storage; c->V = c->K + kv; c->w = (float*)(c->V + kv);
    c->err = (int32_t*)((char*)c->w + align_up((size_t)n_seq * max_tokens * 4, 256));
    c->count = c->base_count = c->stream_j = 0;
    // weights start at 0 (= absent); K, V start finite so that masked lanes never meet NaN payloads
    hipError_t e = bkv::launch_fill_u32(device_storage, 0u, (int64_t)(need / 4), (hipStream_t)hip_stream);
    if (e != hipSuccess) { delete c; return hip_fail(e); }
    *out = c;
    return BKV_OK;
}

int bkv_cache_load(bkv_cache* c, const void* K_c, const void* V_c, const float* w, int64_t count, void* hip_stream) {
    if (!c || count < 0 || count > c->cap) return BKV_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (count > 0) {
        if (!K_c || !V_c || !w || !aligned16(K_c) || !aligned16(V_c)) return BKV_EINVAL;
        const int rb = row_bytes(&c->p);
        hipError_t e;
        if ((e = bkv::launch_copy_rows(K_c, c->K, c->n_seq, count, c->cap, count, rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_rows(V_c, c->V, c->n_seq, count, c->cap, count, rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_f32(w, c->w, c->n_seq, count, c->cap, count, st)) != hipSuccess) return hip_fail(e);
    }
    c->count = c->base_count = count;
    c->stream_j = 0;
    return BKV_OK;
}

size_t bkv_cache_prefill_workspace_bytes(const bkv_cache* c, const bkv_params* p, int64_t n) {
    if (!c) return 0;
    return bkv_merge_reduce_workspace_bytes(p, c->n_seq, n);
}

int bkv_cache_prefill(bkv_cache* c, const bkv_params* p, const void* K, const void* V, int64_t n, int32_t* status_out,
                      void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!c || !p) return BKV_EINVAL;
    int rc = check_params(p);
    if (rc) return rc;
    if (p->d != c->p.d || p->dtype != c->p.dtype) return BKV_ESHAPE;
    if (n < 0 || (n >> p->rounds) > c->cap) return BKV_ECAPACITY;
    rc = merge_reduce_impl(p, K, V, c->n_seq, n, 0, c->K, c->V, c->w, c->cap, nullptr, nullptr, status_out, workspace,
                           ws_bytes, hip_stream, nullptr, c->err);
    if (rc) return rc;
    c->count = c->base_count = n >> p->rounds;
    c->stream_j = 0;
    return BKV_OK;
}

int bkv_cache_free(bkv_cache* c) {
    if (!c) return BKV_EINVAL;
    delete c;
    return BKV_OK;
}

int64_t bkv_cache_count(const bkv_cache* c) { return c ? c->count : (int64_t)BKV_EINVAL; }
int64_t bkv_cache_tokens_seen(const bkv_cache* c) { return c ? c->stream_j : (int64_t)BKV_EINVAL; }

int bkv_cache_views(const bkv_cache* c, void** K, void** V, float** w) {
    if (!c) return BKV_EINVAL;
    if (K) *K = c->K;
    if (V) *V = c->V;
    if (w) *w = c->w;
    return BKV_OK;
}

int bkv_cache_error_word(const bkv_cache* c, const int32_t** device_word) {
    if (!c || !device_word) return BKV_EINVAL;
    *device_word = c->err;
    return BKV_OK;
}

// workspace of a carry: survivors K, V [n_seq, block/2, d]
size_t bkv_append_workspace_bytes(const bkv_cache* c) {
    if (!c) return 0;
    return 2 * align_up((size_t)c->n_seq * (c->p.block / 2) * row_bytes(&c->p), 256) + 256;
}

int bkv_append_token(bkv_cache* c, const void* k, const void* v, int32_t* status_out, const float* uniforms,
                     int8_t* signs_out, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!c || !k || !v || !aligned16(k) || !aligned16(v)) return BKV_EINVAL;
    if (c->count + 1 > c->cap) return BKV_ECAPACITY;
    const int b = c->p.block, T = c->p.rounds;
    const int rb = row_bytes(&c->p);
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t j = c->stream_j + 1;
    int halvings = 0;
    if (T > 0 && j % b == 0) {       // p = j/t is an integer: carry while p stays integral and i < T
        const int64_t pnum = j / b;
        while (halvings < T && pnum % (1ll << halvings) == 0) ++halvings;
        if (!workspace || ws_bytes < bkv_append_workspace_bytes(c) || !aligned16(workspace)) return BKV_EWORKSPACE;
    }
    hipError_t e;
    // C^0 <- C^0 U {(k_j, v_j)}, weight 1
    if ((e = bkv::launch_append(k, v, c->K, c->V, c->w, c->n_seq, c->cap, c->count, rb, st)) != hipSuccess) return hip_fail(e);
    c->count += 1;
    c->stream_j = j;
    if (halvings == 0) return 0;

    char* tmpK = (char*)workspace;
    char* tmpV = tmpK + align_up((size_t)c->n_seq * (b / 2) * rb, 256);
    for (int i = 0; i < halvings; ++i) {
        // C^{i+1} <- C^{i+1} U SoftmaxBalance(C^i): C^i is the last b stored tokens; survivors land where it began
        const int64_t first = c->count - b;
        bkv::CompressArgs a;
        fill_common(a, &c->p);
        a.K = c->K + (size_t)first * rb; a.V = c->V + (size_t)first * rb;
        a.K_out = tmpK; a.V_out = tmpV;
        a.status_out = status_out; a.status_stride = T; a.sticky_err = c->err;
        // decision-level hooks: the halving of level i reads / writes slice i of [T, n_seq, block]
        a.uniforms = uniforms ? uniforms + (size_t)i * c->n_seq * b : nullptr;
        a.signs_out = signs_out ? signs_out + (size_t)i * c->n_seq * b : nullptr;
        a.in_seq_stride = a.v_seq_stride = c->cap; a.out_seq_stride = a.idx_out_seq_stride = b / 2; a.blocks_per_seq = 1;
        a.tree_mode = 1; a.round = i; a.seq_base = 0;
        a.blk_base = (j / b) / (1ll << i) - 1;           // how many blocks reached level i before this one
        a.w_out_val = (float)(1u << (i + 1));
        e = bkv::launch_compress(c->p.dtype, c->p.d, false, a, c->n_seq, st);
        if (e != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_rows(tmpK, c->K + (size_t)first * rb, c->n_seq, b / 2, c->cap, b / 2, rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_copy_rows(tmpV, c->V + (size_t)first * rb, c->n_seq, b / 2, c->cap, b / 2, rb, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_fill_w(c->w, c->n_seq, c->cap, first, b / 2, a.w_out_val, st)) != hipSuccess) return hip_fail(e);
        if ((e = bkv::launch_fill_w(c->w, c->n_seq, c->cap, first + b / 2, b / 2, 0.f, st)) != hipSuccess) return hip_fail(e);
        c->count -= b / 2;
    }
    return halvings;
}

size_t bkv_cache_attend_workspace_bytes(const bkv_cache* c, int32_t g, int32_t nq) {
    if (!c || g <= 0 || nq <= 0) return 0;
    return bkv::attend_workspace_bytes(c->p.d, c->n_seq, g * nq);
}

int bkv_attend(const bkv_cache* c, const void* Q, int32_t g, int32_t nq, void* out, float* lse_out, void* workspace,
               size_t ws_bytes, void* hip_stream) {
    if (!c) return BKV_EINVAL;
    return bkv_attend_kv(&c->p, c->K, c->V, c->w, c->n_seq, c->count, c->cap, Q, g, nq, out, lse_out, workspace,
                         ws_bytes, hip_stream);
}


// ------------------------------------------------------------------------------------------ Alg. 1 token by token
size_t bkv_stream_bytes(const bkv_params* p, int64_t n_seq, int32_t regions, int64_t cap_num, int64_t cap_den) {
    if (check_params(p) || n_seq <= 0 || regions < 1 || regions > 64 || cap_num < p->block || cap_den < p->block) return 0;
    const size_t rb = (size_t)row_bytes(p), R = (size_t)regions, half = (size_t)p->block / 2;
    const size_t T = (size_t)(p->rounds > 0 ? p->rounds : 1);
    size_t s = 0;
    s += 2 * align_up((size_t)n_seq * R * cap_num * rb, 256) + 2 * align_up((size_t)n_seq * R * cap_num * 4, 256);
    s += align_up((size_t)n_seq * cap_den * rb, 256) + 2 * align_up((size_t)n_seq * cap_den * 4, 256);
    s += 2 * align_up((size_t)n_seq * (R + 1) * 4, 256) + align_up((size_t)n_seq * R * 4, 256) + align_up((size_t)n_seq * 4, 256);
    s += 256;
    s += align_up(T * 2 * (size_t)n_seq * sizeof(bkv::InstDesc), 256);
    s += 2 * align_up(2 * (size_t)n_seq * half * rb, 256) + align_up(2 * (size_t)n_seq * half * 4, 256);
    return s;
}

int bkv_stream_init(bkv_stream** out, const bkv_params* p, int64_t n_seq, int64_t seq_base, int32_t regions, int64_t cap_num,
                    int64_t cap_den, int64_t n_total, float eps, float r, void* device_storage, size_t bytes, void* hip_stream) {
    if (!out) return BKV_EINVAL;
    *out = nullptr;
    int rc = check_params(p);
    if (rc) return rc;
    if (n_seq <= 0 || seq_base < 0 || regions < 1 || regions > 64 || cap_num < p->block || cap_den < p->block || !(r >= 0.f))
        return BKV_EINVAL;
    if (n_seq > 65535 || cap_den > (1ll << 30) || (int64_t)regions * cap_num > (1ll << 30)) return BKV_ESHAPE;
    if (eps > 0.f && n_total <= 0) return BKV_EINVAL;
    const size_t need = bkv_stream_bytes(p, n_seq, regions, cap_num, cap_den);
    if (!device_storage || (reinterpret_cast<uintptr_t>(device_storage) & 255u) || bytes < need) return BKV_EINVAL;
    bkv_stream* h = new (std::nothrow) bkv_stream;
    if (!h) return BKV_EINVAL;
    h->p = *p; h->seen = 0;
    bkv::StreamState& s = h->s;
    memset(&s, 0, sizeof(s));
    const size_t rb = (size_t)row_bytes(p), R = (size_t)regions, half = (size_t)p->block / 2;
    const size_t T = (size_t)(p->rounds > 0 ? p->rounds : 1);
    char* at = (char*)device_storage;
    auto carve = [&](size_t b) { char* q = at; at += align_up(b, 256); return q; };
    s.Kn = carve((size_t)n_seq * R * cap_num * rb); s.Vn = carve((size_t)n_seq * R * cap_num * rb);
    s.wn = (float*)carve((size_t)n_seq * R * cap_num * 4); s.on = (int32_t*)carve((size_t)n_seq * R * cap_num * 4);
    s.Kd = carve((size_t)n_seq * cap_den * rb);
    s.wd = (float*)carve((size_t)n_seq * cap_den * 4); s.od = (int32_t*)carve((size_t)n_seq * cap_den * 4);
    s.cnt = (int32_t*)carve((size_t)n_seq * (R + 1) * 4); s.jj = (int32_t*)carve((size_t)n_seq * (R + 1) * 4);
    s.bucket = (int32_t*)carve((size_t)n_seq * R * 4);
    s.vmax2 = (unsigned int*)carve((size_t)n_seq * 4);
    s.err = (int32_t*)carve(256);
    s.desc = (bkv::InstDesc*)carve(T * 2 * (size_t)n_seq * sizeof(bkv::InstDesc));
    s.tmpK = carve(2 * (size_t)n_seq * half * rb); s.tmpV = carve(2 * (size_t)n_seq * half * rb);
    s.tmpIdx = (int32_t*)carve(2 * (size_t)n_seq * half * 4);
    s.n_seq = n_seq; s.seq_base = seq_base; s.cap_n = cap_num; s.cap_d = cap_den;
    s.regions = regions; s.b = p->block; s.T = p->rounds; s.row_bytes = (int32_t)rb; s.dtype = p->dtype; s.d = p->d;
    s.erase2 = 0.f;
    if (eps > 0.f) {
        const double f = (double)eps / (2.0 * (double)n_total) * exp(-(double)r * (double)r / sqrt((double)p->d));
        s.erase2 = (float)(f * f);
    }
    // weights 0 (no token), counters 0, rows finite; every region free
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e = bkv::launch_fill_u32(device_storage, 0u, (int64_t)(need / 4), st);
    if (e == hipSuccess) e = bkv::launch_fill_u32(s.bucket, 0x80000000u, n_seq * (int64_t)R, st);
    if (e != hipSuccess) { delete h; return hip_fail(e); }
    *out = h;
    return BKV_OK;
}

int bkv_stream_free(bkv_stream* s) {
    if (!s) return BKV_EINVAL;
    delete s;
    return BKV_OK;
}

int64_t bkv_stream_tokens_seen(const bkv_stream* s) { return s ? s->seen : (int64_t)BKV_EINVAL; }

int bkv_stream_append(bkv_stream* h, const void* k, const void* v, int32_t* status_num, int32_t* status_den, void* hip_stream) {
    if (!h || !k || !v || !aligned16(k) || !aligned16(v)) return BKV_EINVAL;
    if (h->seen >= (1ll << 31) - 1) return BKV_ECAPACITY;
    const bkv::StreamState& s = h->s;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    int launches = 0;
    if ((e = bkv::stream_route(s, k, v, h->seen, st)) != hipSuccess) return hip_fail(e);
    ++launches;
    const int64_t j = ++h->seen;
    const int b = s.b, half = b / 2;
    for (int r = 0; r < s.T; ++r) {
        // MR-Numerator_i: any sequence's current bucket may carry at this token; instances that do not are skipped on the device
        bkv_params pn = h->p;
        pn.flags |= BKV_VALUE_GRAM;
        bkv::CompressArgs a;
        fill_common(a, &pn);
        a.desc = s.desc + (size_t)(r * 2 + 0) * s.n_seq;
        a.K = s.Kn; a.V = s.Vn; a.K_out = s.tmpK; a.V_out = s.tmpV; a.idx_out = s.tmpIdx;
        a.v_seq_stride = (int64_t)s.regions * s.cap_n;
        a.status_out = status_num; a.status_stride = s.T; a.sticky_err = s.err;
        a.tree_mode = 1; a.round = r; a.blocks_per_seq = 1;
        if ((e = bkv::launch_compress(s.dtype, s.d, false, a, s.n_seq, st)) != hipSuccess) return hip_fail(e);
        ++launches;
        // MR-Denominator sees every token: it carries at round r exactly when block * 2^r divides j
        if (j % ((int64_t)b << r) == 0) {
            bkv_params pd = h->p;
            pd.flags &= ~(BKV_VALUE_GRAM | BKV_VALUE_AUGMENT);
            fill_common(a, &pd);
            a.desc = s.desc + (size_t)(r * 2 + 1) * s.n_seq;
            a.K = s.Kd; a.V = nullptr; a.K_out = s.tmpK + (size_t)s.n_seq * half * s.row_bytes; a.V_out = nullptr;
            a.idx_out = s.tmpIdx + (size_t)s.n_seq * half;
            a.v_seq_stride = s.cap_d;
            a.status_out = status_den; a.status_stride = s.T; a.sticky_err = s.err;
            a.tree_mode = 1; a.round = r; a.blocks_per_seq = 1;
            if ((e = bkv::launch_compress(s.dtype, s.d, false, a, s.n_seq, st)) != hipSuccess) return hip_fail(e);
            ++launches;
        }
        if ((e = bkv::stream_fixup(s, r, st)) != hipSuccess) return hip_fail(e);
        ++launches;
    }
    return launches;
}

int bkv_stream_views(const bkv_stream* h, void** K_n, void** V_n, float** w_n, int32_t** orig_n, void** K_d, float** w_d,
                     int32_t** orig_d, int32_t** count, int32_t** bucket, int32_t** error_word) {
    if (!h) return BKV_EINVAL;
    const bkv::StreamState& s = h->s;
    if (K_n) *K_n = s.Kn;
    if (V_n) *V_n = s.Vn;
    if (w_n) *w_n = s.wn;
    if (orig_n) *orig_n = s.on;
    if (K_d) *K_d = s.Kd;
    if (w_d) *w_d = s.wd;
    if (orig_d) *orig_d = s.od;
    if (count) *count = s.cnt;
    if (bucket) *bucket = s.bucket;
    if (error_word) *error_word = s.err;
    return BKV_OK;
}

size_t bkv_stream_attend_workspace_bytes(const bkv_stream* h, int32_t g, int32_t nq) {
    if (!h) return 0;
    return bkv_attend_sets_workspace_bytes(&h->p, h->s.n_seq, g, nq);
}

int bkv_stream_attend(const bkv_stream* h, const void* Q, int32_t g, int32_t nq, void* out, float* lse_out, void* workspace,
                      size_t ws_bytes, void* hip_stream) {
    if (!h) return BKV_EINVAL;
    const bkv::StreamState& s = h->s;
    if (h->seen == 0) return BKV_EINVAL;                   // the estimator of an empty stream is 0 / 0
    const int64_t places = (int64_t)s.regions * s.cap_n;
    // MR-Denominator holds a known number of tokens (every sequence has fed it every token); numerator regions are read whole
    int64_t count_d = h->seen;
    {
        const int64_t blocks = h->seen / s.b;
        count_d = h->seen - blocks * s.b;                  // tail
        int64_t reached = blocks;                          // blocks that reached level l
        for (int l = 1; l <= s.T; ++l) {
            if (l < s.T) { if (reached & 1) count_d += s.b / 2; reached >>= 1; }
            else count_d += reached * (int64_t)(s.b / 2);
        }
        if (s.T == 0) count_d = h->seen;
        if (count_d > s.cap_d) count_d = s.cap_d;
    }
    return bkv_attend_sets(&h->p, s.Kn, s.Vn, s.wn, places, places, s.Kd, s.wd, count_d, s.cap_d, s.n_seq, Q, g, nq, out, lse_out,
                           workspace, ws_bytes, hip_stream);
}

}  // extern "C"
