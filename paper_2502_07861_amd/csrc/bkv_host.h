// Host-side declarations shared by the translation units of libbalancekv (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/balancekv.h"

namespace bkv {

// One instance of a ragged launch (blocks of segments of different lengths, see sets.hip): where its block starts in
// the round's input and output buffers (tokens from the buffers' bases; idx_out and signs_out use the same
// coordinates as K_out and K), its sequence (value rows, status word), its generator stream and first counter, and
// r_value^2 (<= 0: as in CompressArgs).  valid = 0: the slot of the grid is not in use.
struct InstDesc {
    int64_t in_tok, out_tok;
    uint64_t stream, ctr0;
    int32_t seq, valid;
    float rvalue2;
    int32_t pad;
};

struct CompressArgs {
    const char* K;            // input keys, dtype T
    const char* V;            // input values or null
    char* K_out;              // survivors or null
    char* V_out;
    float* w_out;
    int32_t* idx_out;
    const int32_t* idx_in;    // original index of each input token, or null (position in sequence)
    int8_t* signs_out;
    int32_t* status_out;
    float* stats_out;
    int32_t* sticky_err;      // or null: one word that collects BKV_STATUS_INTERNAL of every instance (never cleared by the kernel)
    const uint64_t* inst_ids;
    const float* uniforms;
    const InstDesc* desc;     // ragged launches: per-instance coordinates (then blocks_per_seq, strides and bases are not read)
    float* G_out;             // kernel-weight dump (EMIT_G variant only)
    int64_t in_seq_stride;    // tokens between consecutive sequences in K / V / idx_in
    int64_t out_seq_stride;   // tokens between consecutive sequences in K_out / V_out / w_out
    int64_t idx_out_seq_stride;  // tokens between consecutive sequences in idx_out
    int64_t v_seq_stride;     // tokens between consecutive sequences in V; survivors are read at their ORIGINAL token index
    int64_t seq_base;         // added to the sequence number in the generator stream id
    int64_t blk_base;         // added to the block number in the generator counter
    int64_t idx_base;         // without idx_in: original index of the launch's first token within its sequence (V rows, idx_out)
    uint64_t seed;
    int32_t blocks_per_seq;
    int32_t b;
    int32_t chunk_rows;
    int32_t round;            // level of the tree this launch halves
    int32_t tree_mode;        // 1: stream = 64*(seq_base+seq)+round, ctr = (blk_base+blk)*b + j ; 0: stream = inst, ctr = j
    int32_t status_stride;    // tree mode: status_out[seq*status_stride + round] accumulated atomically
    float w_out_val;
    float alpha;              // log2(e)/sqrt(d)
    float cterm;              // -sqrt(d) * ln c
    float rkey2;              // r_key^2, <= 0: measure
    float rvalue2;            // r_value^2 (value factor only), <= 0: the largest |v_i|^2 of the block
    uint32_t flags;
    int32_t stagger_blocks;   // the first stagger_blocks workgroups (one per compute unit) start stagger_step clock
    int32_t stagger_step;     // ticks apart, so that the memory-bound phases of successive blocks do not coincide chip-wide
    int32_t k_by_idx;         // 1 (resident blocks only): the key rows of the block are read at their ORIGINAL index (idx_in), like
                              // the value rows, from K [n_seq, v_seq_stride, d]: no copy of the keys in block order is needed
    int32_t prefetch_ahead;   // > 0: while walking, touch the keys of block (this + prefetch_ahead) so that they sit in L2 / MALL
};

size_t compress_lds_bytes(int row_bytes, int b, bool value_gram = false);
bool compress_value_gram_fits(int row_bytes, int b);   // keys and values of one block resident in LDS together
bool compress_block_resident(int row_bytes, int b, bool value_gram);   // the block runs as one resident chunk
hipError_t launch_compress(int dtype, int d, bool emit_g, CompressArgs& a, int64_t n_inst, hipStream_t st);
hipError_t launch_fill_u32(void* p, uint32_t v, int64_t n, hipStream_t st);
hipError_t launch_copy_rows(const void* src, void* dst, int64_t n_seq, int64_t src_seq_stride,
                            int64_t dst_seq_stride, int64_t rows, int row_bytes, hipStream_t st);
hipError_t launch_append(const void* k, const void* v, void* K, void* V, float* w, int64_t n_seq, int64_t seq_stride,
                         int64_t pos, int row_bytes, hipStream_t st);
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n_seq, int64_t src_seq_stride,
                           int64_t dst_seq_stride, int64_t rows, hipStream_t st);
hipError_t launch_fill_w(float* w, int64_t n_seq, int64_t seq_stride, int64_t off, int64_t rows, float val,
                         hipStream_t st);
hipError_t launch_fill_iota(int32_t* idx, int64_t n_seq, int64_t seq_stride, int64_t off, int64_t rows, int32_t first,
                            hipStream_t st);

// Opt-in per-launch timing (diagnostics): start/stop events attached to the launches themselves.
enum { kProfCompress = 0, kProfAttend = 2, kProfAttendMerge = 3 };     // record kinds (1 is not in use)
int prof_enable(int n);
int prof_read(int32_t* kind, float* ms, int64_t* units, int cap);
// Reserves a timing record and hands out its two events (false: timing is off or the records are used up).  The
// caller passes them to hipExtLaunchKernelGGL, so that they carry the start and end of that kernel itself rather
// than of a stretch of the stream around it.
bool prof_slot(int kind, int64_t units, hipEvent_t* start, hipEvent_t* stop);
// launch `kern`, timed when a record is available
template <typename Kern, typename... Args>
inline hipError_t launch_timed(int kind, int64_t units, Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    hipEvent_t e0, e1;
    if (prof_slot(kind, units, &e0, &e1)) hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, st, e0, e1, 0, args...);
    else hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
    return hipGetLastError();
}

// peak micro-benchmarks (diagnostics): kind 0 bare bf16 MFMA loop, 1 the tile routine alone, 2 streaming read, 3 streaming copy
hipError_t measure_peak(int kind, int launches, void* workspace, size_t ws_bytes, hipStream_t st, double* per_second, double* ms_per_launch);

// Alg. 1's kept sets (sets.hip): value-norm buckets with one MergeAndReduce instance each (numerator = 1), or the
// keys-only instance over the whole sequence (numerator = 0), brought to the state Alg. 3 reaches after the last token.
struct SetsArgs {
    const char* K;            // [n_seq, n, d]
    const char* V;
    int64_t n_seq, n, seq_base, capacity;
    int32_t dtype, d, row_bytes, b, T, numerator;
    float erase2;             // (eps / (2n) * exp(-r^2 / sqrt d))^2, 0: nothing is erased
    CompressArgs common;      // flags, seed, alpha, cterm, radii
    char* K_out;              // [n_seq, capacity, d] or null
    char* V_out;
    float* w_out;             // [n_seq, capacity]: 2^level, 0 beyond the count
    int32_t* idx_ws;          // [n_seq, capacity]: original index of every kept token (required)
    int32_t* count_out;       // [n_seq] (required)
    int32_t* slot_out;        // [n_seq, n] or null
    int8_t* signs_out;        // rounds one after the other, round r at the coordinates of its level-r buffer [n_seq, n >> r]
    int32_t* status_out;      // [n_seq, T]
    void* workspace;
};
size_t sets_workspace_bytes(int row_bytes, int b, int64_t n_seq, int64_t n);
hipError_t run_sets(const SetsArgs& q, hipStream_t st);
hipError_t launch_rescale(int dtype, void* out, const float* lse_num, const float* lse_den, int64_t rows, int d, hipStream_t st);

// Alg. 1 token by token: device state of n_seq sequences.  Every sequence owns `regions` numerator regions of
// cap_n token places (one per live bucket, handed out on a bucket's first token and taken back when the bucket is
// erased) and one denominator region of cap_d places.  A region holds the levels of its MergeAndReduce instance as
// the streaming cache does: level-T survivors first, then levels T-1..1, then the tail; places beyond `cnt` have
// weight 0.  All counters live on the device: which instance carries at a token depends on the values.
struct StreamState {
    char* Kn; char* Vn; float* wn; int32_t* on;   // [n_seq, regions, cap_n(, d)]: keys, values, weights, original token index
    char* Kd; float* wd; int32_t* od;             // [n_seq, cap_d(, d)]
    int32_t* cnt;             // [n_seq, regions + 1]: stored tokens; entry `regions` is the denominator instance
    int32_t* jj;              // [n_seq, regions + 1]: tokens the instance has seen since it was created
    int32_t* bucket;          // [n_seq, regions]: bucket index of the region, INT32_MIN: free
    unsigned int* vmax2;      // [n_seq]: largest |v|^2 so far (bits of a non-negative float)
    int32_t* err;             // one word: BKV_STATUS_INTERNAL of any halving | BKV_STREAM_* overflow bits
    InstDesc* desc;           // [T, 2, n_seq]: the carries of the current token (0: numerator, 1: denominator)
    char* tmpK; char* tmpV;   // [2, n_seq, b/2, d]: survivors of the halving in flight
    int32_t* tmpIdx;          // [2, n_seq, b/2]: their places
    int64_t n_seq, seq_base, cap_n, cap_d;
    int32_t regions, b, T, row_bytes, dtype, d;
    float erase2;             // (eps / (2n) * exp(-r^2 / sqrt d))^2, 0: nothing is erased
};
hipError_t stream_route(const StreamState& s, const void* k, const void* v, int64_t j, hipStream_t st);
hipError_t stream_fixup(const StreamState& s, int round, hipStream_t st);

struct AttendArgs {
    const char* K;            // [n_seq, stride_tokens, d]
    const char* V;
    const float* w;           // [n_seq, stride_tokens]
    const char* Q;            // [n_seq, n_q, d]   (n_q = g * nq query vectors per sequence)
    char* out;                // [n_seq, n_q, d]
    float* lse_out;           // [n_seq, n_q] or null
    float* partial;           // workspace: [n_seq, n_qgroups, n_splits, QT, d + 2]
    int64_t stride_tokens;
    int64_t count;
    int32_t n_q;
    int32_t n_splits;
    int32_t rows_per_split;
    float scale_log2;         // log2(e)/sqrt(d)
};
size_t attend_workspace_bytes(int d, int64_t n_seq, int n_q);
hipError_t launch_attend(int dtype, int d, AttendArgs& a, int64_t n_seq, void* workspace, hipStream_t st);
// the entry point without allocations: what a launch of this shape writes into the partial buffer, and the
// library's own buffer for it (a file-scope device array; address of the current device's copy)
constexpr size_t kAttendStaticScratchBytes = 2304 * 1024;
size_t attend_partial_bytes(int dtype, int d, int64_t n_seq, int64_t count, int n_q);
hipError_t attend_static_scratch(void** ptr);

}  // namespace bkv
