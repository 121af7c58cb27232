/*
 * balancekv.h -- C ABI of the MI355X (gfx950) BalanceKV hot path.
 *
 * BalanceKV (arXiv 2502.07861) compresses a key/value cache by repeated
 * discrepancy-based halving and answers decode attention from the weighted
 * survivors.  This library implements, in hand-written HIP, the four verbs of
 * the paper's streaming problem statement (Section 2.1):
 *
 *   bkv_compress_block   one halving of independent blocks        (Alg. 2)
 *   bkv_merge_reduce     T rounds of block-parallel halving        (Alg. 3, offline
 *                        form in the proof of Thm 3.3; App. B "Implementation Detail")
 *   bkv_append_token     one streaming step incl. carries          (Alg. 3)
 *   bkv_attend           weighted softmax estimator                (Alg. 1, output line)
 *
 * and, on top of them, Alg. 1 as listed (value-norm buckets, numerator and denominator
 * instances): offline as bkv_balancekv_sets / bkv_attend_sets, token by token as bkv_stream_*.
 *
 * Conventions
 *  - Plain C, no exceptions.  Every tensor pointer is a DEVICE pointer owned by
 *    the caller unless stated otherwise; the library never frees or keeps it
 *    beyond the call, except the storage handed to bkv_cache_init / bkv_stream_init.
 *  - Scratch memory comes from the caller: query the size, pass `workspace`.
 *  - Every call only enqueues work on `hip_stream` (a hipStream_t passed as
 *    void*, NULL = default stream) and returns; nothing synchronises (the
 *    two diagnostics calls bkv_profile_read and bkv_measure_peak do, and say so).
 *  - Return value: BKV_OK or a negative code for misuse / launch failure.
 *    Algorithmic events (the FAIL branch of Alg. 2, near-tie decisions) are
 *    NOT errors: they are written to per-instance device arrays.
 *  - Layout: row-major, head dimension fastest.  A "sequence" is one
 *    (session, layer, KV head) stream; sequences are independent.
 *  - Supported: d in {64,128}; block in {64,128,...,1024} (multiple of 64);
 *    dtype BKV_F32 or BKV_BF16 (inputs, outputs and queries share it; all
 *    accumulation is fp32; the one narrowing is stated at bkv_attend_kv).
 *    Strict halving only (exactly block/2 survivors).
 */
#ifndef BALANCEKV_H
#define BALANCEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dtype */
#define BKV_F32  0
#define BKV_BF16 1

/* flags */
#define BKV_CENTER_KEYS 1u  /* shift keys by the block mean for the selection (App. B.5 item 1) */
#define BKV_STRICT_HALF 2u  /* keep exactly block/2 per block (App. B, Implementation Detail); required */
#define BKV_VALUE_GRAM  4u  /* multiply kernel weights by <v_i,v_j>/r_value^2 (Alg. 2 line 6): the walk then balances
                             * the numerator instance of Alg. 1.  Fast where keys and values of a block fit the
                             * 160 KB of LDS together (d=128: block <= 256 bf16 / 128 fp32; d=64: block <= 512 bf16 /
                             * 256 fp32); larger blocks read the value panels from L2 tile by tile.  V is required
                             * wherever K is.                                                                    */
#define BKV_VALUE_AUGMENT 8u /* with BKV_VALUE_GRAM: the walk sees the value [v / r_value ; 1] (Alg. 2 takes values of any
                             * dimension s), i.e. the factor (<v_i,v_j>/r_value^2 + 1) / 2: one kept set that balances the
                             * numerator and the denominator of Alg. 1's output line together.  A block whose values are
                             * all zero gets the factor 1 (the keys-only walk) when the radius is measured, 1/2 when given. */

/* return codes */
#define BKV_OK          0
#define BKV_EINVAL     -1   /* null / misaligned pointer, negative size, bad handle             */
#define BKV_ESHAPE     -2   /* unsupported d / block / rounds / dtype / flags, or n not a      */
                            /* multiple of block * 2^rounds                                    */
#define BKV_EWORKSPACE -3   /* workspace missing or too small                                  */
#define BKV_EHIP       -4   /* a HIP call failed; see bkv_last_hip_error()                     */
#define BKV_ECAPACITY  -5   /* the streaming cache is full                                     */

/* status word written per instance (bkv_compress_block) */
#define BKV_STATUS_FAIL 1   /* bit 0: |y^T eta| > c R^2 happened (Alg. 2 line 7); p was clamped */
#define BKV_STATUS_INTERNAL 2 /* bit 1: the kernel's internal pipeline timed out; the instance's outputs are invalid (never expected) */
/* bits 8..30: number of decisions whose margin |u_j - p_j| was below 1e-4 (per-sequence words of the tree calls
 * add the counts of their blocks and saturate at 2^23 - 1); bit 31 is never set */

typedef struct bkv_params {
    int32_t  d;        /* head dimension                                                       */
    int32_t  block;    /* b: block length (the batch size t of Alg. 3)                          */
    int32_t  rounds;   /* T: halving rounds; compression rate 2^-T                              */
    int32_t  dtype;    /* BKV_F32 | BKV_BF16                                                    */
    float    log_c;    /* ln c of Alg. 2 line 3; NaN => ln(30 ln(block/delta))                  */
    float    delta;    /* failure probability of Alg. 2; only read when log_c is NaN            */
    float    r_key;    /* key radius of Alg. 2; <= 0 => largest (centred) key norm of the block */
    float    r_value;  /* value radius (BKV_VALUE_GRAM only); <= 0 => largest value norm of the block */
    uint64_t seed;     /* key of the counter-based generator behind "with probability p_j"      */
    uint32_t flags;    /* BKV_* flags                                                           */
    uint32_t reserved; /* must be 0                                                             */
} bkv_params;

/* ---- misc ------------------------------------------------------------------------------- */
const char* bkv_version(void);
const char* bkv_error_string(int code);
int         bkv_last_hip_error(void);          /* hipError_t of the last BKV_EHIP on this thread */

/* The uniform draw of decision `ctr` in stream `stream`: top 24 bits of two rounds of the
 * SplitMix64 mixer over (seed, stream, ctr); u = bits * 2^-24 in [0,1).  Host function, same
 * integers as the device code.  Alg. 2 line 9 sets eta_j = +1 iff u_j < p_j.                    */
uint32_t bkv_uniform_bits(uint64_t seed, uint64_t stream, uint64_t ctr);

/* ---- Alg. 2: one halving of n_inst independent blocks ---------------------------------------
 * K, V          [n_inst, block, d] device, dtype as params.  V may be NULL (then V_out must be).
 * inst_ids      [n_inst] device or NULL: generator stream of each instance (NULL: 0,1,2,...);
 *               decision j of an instance draws u = uniform(seed, stream, j).
 * w_in          weight carried by every input token (2^level); survivors get 2*w_in.
 * uniforms      [n_inst, block] fp32 device or NULL: if given, replaces the generator (test hook).
 * K_out, V_out  [n_inst, block/2, d] survivors, rows of the ORIGINAL K, V, ascending input index.
 * w_out         [n_inst, block/2] fp32 or NULL.
 * idx_out       [n_inst, block/2] int32 or NULL: index within the block of each survivor.
 * signs_out     [n_inst, block] int8 (+1/-1) or NULL: eta of Alg. 2 before the output step.
 * status_out    [n_inst] int32 or NULL (BKV_STATUS_*).
 * stats_out     [n_inst, 2] fp32 or NULL: {min_j |u_j - p_j|, max_j |y^T eta|/(c R^2)}.
 * workspace     bkv_compress_workspace_bytes() bytes (may be 0 => NULL allowed).
 * Kernel weights are exp((<k_i,k_j> - r_key^2)/sqrt(d) - ln c) (Alg. 2 lines 2-8 divided
 * through by c R^2), keys optionally centred by the block mean, times <v_i,v_j>/r_value^2 with
 * BKV_VALUE_GRAM (V then must be given; a block of all-zero values has weight 0 everywhere);
 * n_inst == 0 is a no-op.                                                                        */
size_t bkv_compress_workspace_bytes(const bkv_params* p, int64_t n_inst);
int bkv_compress_block(const bkv_params* p, const void* K, const void* V, int64_t n_inst,
                       const uint64_t* inst_ids, float w_in, const float* uniforms,
                       void* K_out, void* V_out, float* w_out, int32_t* idx_out,
                       int8_t* signs_out, int32_t* status_out, float* stats_out,
                       void* workspace, size_t ws_bytes, void* hip_stream);

/* The kernel-weight matrix itself, for inspection: G_out [n_inst, block, block] fp32, entry
 * (i,j) = exp((<k_i,k_j> - r_key^2)/sqrt(d) - ln c) as the walk sees it (Alg. 2 line 6, v = 1).
 * Symmetric; produced by the same tile code as the walk.  BKV_VALUE_GRAM: BKV_ESHAPE (no values
 * are passed here).                                                                              */
int bkv_kernel_weights(const bkv_params* p, const void* K, int64_t n_inst, float* G_out,
                       void* hip_stream);

/* ---- Alg. 3 offline: T = p->rounds rounds over n_seq sequences of n tokens ---------------------
 * K, V          [n_seq, n, d] device.  n must be a multiple of block * 2^T.
 * Round r views the n>>r surviving tokens of a sequence as blocks of `block` (a merged block is
 * the left child's survivors then the right child's) and halves each.  Decision j of block blk in
 * round r of sequence s draws uniform(seed, 64*(seq_base+s) + r, blk*block + j).
 * K_out, V_out  [n_seq, n>>T, d]; w_out [n_seq, n>>T] fp32 (= 2^T) or NULL;
 * idx_out       [n_seq, n>>T] int32 or NULL: original token index of each survivor (ascending).
 * signs_out     int8 or NULL: eta of every round, round r at offset n_seq*(2n - (2n>>r)),
 *               laid out [n_seq, n>>r].
 * status_out    [n_seq, T] int32 or NULL: per sequence and round, bit 0 = any FAIL, bits 8.. =
 *               total number of margin decisions (|u-p| < 1e-4).
 * workspace     bkv_merge_reduce_workspace_bytes() bytes.  rounds == 0 copies the input.          */
size_t bkv_merge_reduce_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t n);
int bkv_merge_reduce(const bkv_params* p, const void* K, const void* V, int64_t n_seq, int64_t n,
                     int64_t seq_base, void* K_out, void* V_out, float* w_out, int32_t* idx_out,
                     int8_t* signs_out, int32_t* status_out,
                     void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Alg. 3 offline with protected windows (Full Experimental Details, single-layer attention
 * approximation: the first and the most recent tokens are kept as they are, BalanceKV runs on the
 * rows in between) --------------------------------------------------------------------------------
 * K, V          [n_seq, n, d] device.  The first n_sink and the last n_recent tokens of every
 *               sequence are copied (weight 1); the n - n_sink - n_recent tokens in between, which
 *               must be a multiple of block * 2^T, go through bkv_merge_reduce's tree as a sequence
 *               of their own (blocks and uniform draws counted from the first row after the sink).
 * Outputs hold count = n_sink + ((n - n_sink - n_recent) >> T) + n_recent tokens per sequence, in
 * ascending original order: K_out, V_out [n_seq, count, d]; w_out [n_seq, count] (1 | 2^T | 1) or
 * NULL; idx_out [n_seq, count] int32 original token index or NULL; status_out as bkv_merge_reduce.
 * workspace     bkv_merge_reduce_workspace_bytes(p, n_seq, n - n_sink - n_recent) bytes.
 * Errors as bkv_merge_reduce; BKV_EINVAL if the windows do not fit the sequence.                  */
int bkv_merge_reduce_protected(const bkv_params* p, const void* K, const void* V, int64_t n_seq,
                               int64_t n, int64_t n_sink, int64_t n_recent, int64_t seq_base,
                               void* K_out, void* V_out, float* w_out, int32_t* idx_out,
                               int32_t* status_out, void* workspace, size_t ws_bytes,
                               void* hip_stream);

/* ---- Alg. 1 output line on a flat weighted cache -------------------------------------------------
 * K_c, V_c      [n_seq, stride_tokens, d] device; only the first `count` tokens of each sequence
 *               are read.  w [n_seq, stride_tokens] fp32 (2^level; w == 0 marks an absent token).
 * Q             [n_seq, g, nq, d]: g query heads share each KV sequence (GQA), nq queries each.
 * out           [n_seq, g, nq, d] (dtype as params);  lse_out [n_seq, g, nq] fp32 or NULL: natural
 *               log of the estimator's denominator, so partial results over disjoint token ranges
 *               can be merged.  out = sum_i w_i e^{<k_i,q>/sqrt d} v_i / sum_i w_i e^{<k_i,q>/sqrt d}.
 * count == 0 writes zeros and lse = -inf.
 * Precision: logits, running maximum, numerator and denominator sums are fp32.  With BKV_BF16 every softmax weight
 * 2^(logit - max) is rounded to bf16 (to nearest even) before it multiplies its value row, and the denominator adds
 * the same rounded weights (relative error of a weight <= 2^-9, unbiased); with BKV_F32 the weights stay fp32.
 * Limits: n_seq <= 65535 and g * nq <= 262140 (else BKV_ESHAPE).                                    */
size_t bkv_attend_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t count, int32_t g,
                                  int32_t nq);   /* an upper bound valid for any smaller count too */
int bkv_attend_kv(const bkv_params* p, const void* K_c, const void* V_c, const float* w,
                  int64_t n_seq, int64_t count, int64_t stride_tokens, const void* Q, int32_t g,
                  int32_t nq, void* out, float* lse_out, void* workspace, size_t ws_bytes,
                  void* hip_stream);

/* The same call for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, results and error codes as
 * bkv_attend_kv, without `workspace`: the partial sums of a split token range go to a static device array inside the
 * library (bkv_attend_kv_static_max_bytes() bytes, 2.25 MiB, held by every GPU the library runs on until the process
 * ends).  The call allocates nothing and frees nothing.  A launch whose partials would not fit the array returns
 * BKV_EWORKSPACE (with today's launch plan -- at most 1023 (workgroup, split) pairs of 4 x (d + 2) floats whenever the
 * range is split -- every shape that bkv_attend_kv accepts fits).  All calls on one GPU share the array: calls that
 * overlap in time on the same GPU (different streams, different threads) race; calls on one stream do not.  The
 * array keeps the last call's partials; every launch writes all partials it later reads, nothing needs clearing.  */
size_t bkv_attend_kv_static_max_bytes(void);
int bkv_attend_kv_static(const bkv_params* p, const void* K_c, const void* V_c, const float* w,
                         int64_t n_seq, int64_t count, int64_t stride_tokens, const void* Q, int32_t g,
                         int32_t nq, void* out, float* lse_out, void* hip_stream);

/* ---- Alg. 1 as listed: value-norm buckets, MR-Numerator_i per bucket, MR-Denominator ---------------
 * Offline form on K, V [n_seq, n, d] (any n >= 0): every instance is brought to the state Alg. 3
 * (MergeAndReduce) holds after its last token -- full blocks halved level by level, at most one half
 * block left at each level 1..T-1 (weight 2^l), the level-T survivors (weight 2^T) and a tail of fewer
 * than `block` tokens (weight 1).
 *   which = BKV_SET_NUMERATOR   Alg. 1 lines 5-10: token j goes to bucket i, the smallest i with
 *           2^i >= |v_j| (|v_j|^2 accumulated in fp32; i is clamped to [-60, 60]); every bucket is an
 *           instance with the value factor of Alg. 2 line 6 and r_value = 2^i; buckets with
 *           2^i <= eps/(2n) e^{-r^2/sqrt d} max_j |v_j| are erased (line 8; eps <= 0: none).  Rows with
 *           a zero or non-finite norm belong to no bucket.  The result is the union of the buckets'
 *           sets V^l, bucket by bucket in ascending i.  BKV_VALUE_GRAM need not be set in p.
 *   which = BKV_SET_DENOMINATOR lines 11-12: one keys-only instance per sequence (the sets K^l).
 * Draws: instance q = 512 (seq_base + seq) + slot, slot = 0 for the denominator and 256 + i for bucket
 * i; decision j of the blk-th block reaching level l of instance q draws uniform(seed, 64 q + l,
 * blk*block + j).
 * Outputs (device): K_out, V_out [n_seq, capacity, d] or NULL; w_out [n_seq, capacity] fp32 or NULL
 * (0 beyond the count); idx_out [n_seq, capacity] int32 or NULL (original index of every kept token);
 * count_out [n_seq] int32 or NULL: tokens kept per sequence -- if it exceeds `capacity` the surplus was
 * not written (bkv_sets_capacity gives a bound).  slot_out [n_seq, n] int32 or NULL: slot of every token
 * (511: in no bucket).  signs_out int8 or NULL: eta of every halving, round r at offset
 * n_seq * sum_{r' < r} (n >> r') in the coordinates of that round's input [n_seq, n >> r]: the segment
 * of slot s that starts at position p of the slot-ordered sequence occupies positions from p >> r.
 * status_out [n_seq, max(rounds,1)] int32 or NULL as in bkv_merge_reduce (cleared here).
 * One host-independent pass: no count travels to the host, grids are upper bounds.
 * Limits: n <= 2^30, n_seq <= 65535 (else BKV_ESHAPE); workspace from
 * bkv_balancekv_sets_workspace_bytes (BKV_EWORKSPACE if missing or too small).                     */
#define BKV_SET_NUMERATOR   1
#define BKV_SET_DENOMINATOR 0
int64_t bkv_sets_capacity(const bkv_params* p, int64_t n, int32_t max_buckets);
size_t bkv_balancekv_sets_workspace_bytes(const bkv_params* p, int64_t n_seq, int64_t n, int64_t capacity);
int bkv_balancekv_sets(const bkv_params* p, int32_t which, const void* K, const void* V, int64_t n_seq,
                       int64_t n, int64_t seq_base, float eps, float r, void* K_out, void* V_out,
                       float* w_out, int32_t* idx_out, int64_t capacity, int32_t* count_out,
                       int32_t* slot_out, int8_t* signs_out, int32_t* status_out, void* workspace,
                       size_t ws_bytes, void* hip_stream);

/* Alg. 1 output line with separate sets: the numerator sum over (K_n, V_n, w_n) divided by the
 * denominator sum over (K_d, w_d); layouts as in bkv_attend_kv, each set with its own count and
 * stride.  lse_out: natural log of the denominator sum.  count_d == 0 with count_n > 0: BKV_EINVAL. */
size_t bkv_attend_sets_workspace_bytes(const bkv_params* p, int64_t n_seq, int32_t g, int32_t nq);
int bkv_attend_sets(const bkv_params* p, const void* K_n, const void* V_n, const float* w_n,
                    int64_t count_n, int64_t stride_n, const void* K_d, const float* w_d,
                    int64_t count_d, int64_t stride_d, int64_t n_seq, const void* Q, int32_t g,
                    int32_t nq, void* out, float* lse_out, void* workspace, size_t ws_bytes,
                    void* hip_stream);

/* ---- Alg. 3 streaming: the levels C^0..C^T of n_seq sequences --------------------------------------
 * The levels of one sequence live in one flat array, highest level first: level-T survivors, then
 * levels T-1..1 (each empty or block/2 tokens), then the raw tail C^0.  A carry halves the last
 * `block` tokens in place, so no token ever moves while it is live.  All sequences of a cache
 * advance in lock step (one token each per bkv_append_token), hence one host-side counter.
 * device_storage: bkv_cache_bytes() bytes, 256-byte aligned, caller-owned, must outlive the handle.
 * max_tokens: capacity in stored tokens per sequence (survivors + tail), >= block.
 * p->rounds and p->block govern the streaming phase; p->seed keys its draws: decision j of the
 * blk-th block reaching level l of sequence s draws uniform(seed, 64*s + l, blk*block + j).        */
typedef struct bkv_cache bkv_cache;
size_t bkv_cache_bytes(const bkv_params* p, int64_t n_seq, int64_t max_tokens);
int bkv_cache_init(bkv_cache** out, const bkv_params* p, int64_t n_seq, int64_t max_tokens,
                   void* device_storage, size_t bytes, void* hip_stream);
/* Adopt compressed tokens (e.g. a bkv_merge_reduce result) as already-final survivors:
 * K_c, V_c [n_seq, count, d], w [n_seq, count].  Resets the streaming counter.                      */
int bkv_cache_load(bkv_cache* c, const void* K_c, const void* V_c, const float* w, int64_t count,
                   void* hip_stream);
/* Prefill: run bkv_merge_reduce (parameters `pre`: its block, rounds, seed, ln c; d and dtype must
 * equal the cache's) on K, V [n_seq, n, d] and leave the survivors directly in the cache as final
 * survivors of weight 2^pre->rounds (no intermediate copy).  Resets the streaming counter.
 * Workspace as bkv_merge_reduce.  BKV_ECAPACITY if n >> rounds exceeds max_tokens.                   */
size_t bkv_cache_prefill_workspace_bytes(const bkv_cache* c, const bkv_params* pre, int64_t n);
int bkv_cache_prefill(bkv_cache* c, const bkv_params* pre, const void* K, const void* V, int64_t n,
                      int32_t* status_out, void* workspace, size_t ws_bytes, void* hip_stream);
int bkv_cache_free(bkv_cache* c);                      /* host handle only                          */
int64_t bkv_cache_count(const bkv_cache* c);           /* stored tokens per sequence                */
int64_t bkv_cache_tokens_seen(const bkv_cache* c);     /* tokens appended since init / load (j)     */
/* Device views of the storage: K, V [n_seq, max_tokens, d], w [n_seq, max_tokens].                  */
int bkv_cache_views(const bkv_cache* c, void** K, void** V, float** w);
/* One int32 in the cache's device storage, cleared by bkv_cache_init: every halving that runs for this cache
 * (bkv_cache_prefill, the carries of bkv_append_token) ORs BKV_STATUS_INTERNAL into it if its pipeline timed out,
 * whether or not the call was given a status array.  Non-zero: survivors written since the last init are not to be
 * trusted.  The pointer is a device pointer; read it in stream order (no call here synchronises).       */
int bkv_cache_error_word(const bkv_cache* c, const int32_t** device_word);

/* One streaming step: k, v [n_seq, d] (one new token per sequence) go to the tail with weight 1;
 * after every block-th token the carry loop of Alg. 3 runs (up to T halvings of the last `block`
 * tokens).  Returns the number of halvings performed (>= 0) or a negative code.
 * status_out [n_seq, T] int32 or NULL is OR-ed/added to as in bkv_merge_reduce (never cleared here).
 * Decision-level hooks, as in bkv_compress_block (both may be NULL):
 * uniforms   [T, n_seq, block] fp32 device: the halving of level i that this step runs takes u_j from
 *            uniforms[i][seq][j] instead of the generator (test hook);
 * signs_out  [T, n_seq, block] int8 device: eta of the halving of level i (its block in stored order,
 *            older half first) goes to signs_out[i]; slices of levels that did not carry are not written. */
size_t bkv_append_workspace_bytes(const bkv_cache* c);
int bkv_append_token(bkv_cache* c, const void* k, const void* v, int32_t* status_out,
                     const float* uniforms, int8_t* signs_out,
                     void* workspace, size_t ws_bytes, void* hip_stream);

/* Alg. 1 output line over everything the cache holds (all levels, weights 2^level).
 * Q, out, lse_out, precision and limits as in bkv_attend_kv (a cache holds at most 65535 sequences).  */
size_t bkv_cache_attend_workspace_bytes(const bkv_cache* c, int32_t g, int32_t nq);
int bkv_attend(const bkv_cache* c, const void* Q, int32_t g, int32_t nq, void* out, float* lse_out,
               void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Alg. 1 token by token: the streaming data structure of the listing ------------------------------
 * The state of n_seq sequences after j tokens each (all sequences advance in lock step, one token per call): per
 * sequence the instance MR-Denominator and one instance MR-Numerator_i per live value-norm bucket i, each holding the
 * levels Alg. 3 keeps.  Which numerator instance a token feeds, when it carries and which buckets are erased depend
 * on the values, so every counter lives on the device and no call reads anything back: bkv_stream_append is a fixed
 * sequence of launches (route the token; per round r < T: halve the numerator blocks that carry, halve the
 * denominator blocks -- launched only at the tokens where the host knows they carry --, move the survivors back).
 *   regions     numerator instances a sequence can hold at a time (1..64); a bucket takes a free one on its first
 *               token and gives it back when line 8 erases it
 *   cap_num     token places per numerator region, cap_den places of the denominator region (>= block each); an
 *               instance that has seen m tokens holds at most (m >> T) + (T + 1) * block / 2 + block of them
 *   n_total, eps, r   the erase rule of line 8: after every token the buckets with
 *               2^i <= eps/(2 n_total) e^{-r^2/sqrt d} max_{j' <= j} |v_j'| are dropped, their tokens with them
 *               (eps <= 0: none); a token that falls into such a bucket is not stored
 *   p           block, rounds, dtype, d, seed, ln c, BKV_CENTER_KEYS as in bkv_balancekv_sets; the numerator
 *               instances use the value factor with r_value = 2^i whether or not BKV_VALUE_GRAM is set
 * Buckets, bucket clamp, rows without a bucket, instance numbers and draws exactly as in bkv_balancekv_sets: with
 * eps <= 0 the state after n tokens holds the same tokens with the same weights as the offline call on those n tokens.
 * device_storage: bkv_stream_bytes() bytes, 256-byte aligned, caller-owned, must outlive the handle; cleared by init.
 * Overflow never writes out of bounds: the token is dropped for that instance and a bit is set in the error word. */
#define BKV_STREAM_NUM_FULL  4   /* error word: a numerator region was full, a token was not stored           */
#define BKV_STREAM_DEN_FULL  8   /* error word: the denominator region was full                               */
#define BKV_STREAM_NO_REGION 16  /* error word: more live buckets than regions, a token was not stored        */
typedef struct bkv_stream bkv_stream;
size_t bkv_stream_bytes(const bkv_params* p, int64_t n_seq, int32_t regions, int64_t cap_num, int64_t cap_den);
int bkv_stream_init(bkv_stream** out, const bkv_params* p, int64_t n_seq, int64_t seq_base, int32_t regions,
                    int64_t cap_num, int64_t cap_den, int64_t n_total, float eps, float r,
                    void* device_storage, size_t bytes, void* hip_stream);
int bkv_stream_free(bkv_stream* s);                      /* host handle only                          */
int64_t bkv_stream_tokens_seen(const bkv_stream* s);
/* One token per sequence: k, v [n_seq, d] device.  status_num, status_den [n_seq, T] int32 device or NULL: FAIL bit
 * and margin counts of this instance kind's halvings per round, accumulated as in bkv_merge_reduce (never cleared
 * here).  Returns the number of launches issued (> 0) or a negative code.                             */
int bkv_stream_append(bkv_stream* s, const void* k, const void* v, int32_t* status_num, int32_t* status_den,
                      void* hip_stream);
/* Device views (any pointer argument may be NULL): K_n, V_n [n_seq, regions, cap_num, d]; w_n (2^level, 0: no token),
 * orig_n (index in the stream of the token stored there) [n_seq, regions, cap_num]; K_d [n_seq, cap_den, d]; w_d,
 * orig_d [n_seq, cap_den]; count [n_seq, regions + 1] int32 stored tokens per region, the denominator last;
 * bucket [n_seq, regions] int32 bucket index of every region (INT32_MIN: free); error_word: one int32,
 * BKV_STATUS_INTERNAL | BKV_STREAM_* bits, sticky since init.  Read them in stream order.             */
int bkv_stream_views(const bkv_stream* s, void** K_n, void** V_n, float** w_n, int32_t** orig_n, void** K_d,
                     float** w_d, int32_t** orig_d, int32_t** count, int32_t** bucket, int32_t** error_word);
/* Alg. 1 output line over the current state: numerator sum over all regions / denominator sum over MR-Denominator's
 * levels.  Q, out, lse_out, precision and limits as in bkv_attend_sets.  Reads every place of every region (absent
 * places have weight 0), so its cost follows the capacities, not the occupancy.                        */
size_t bkv_stream_attend_workspace_bytes(const bkv_stream* s, int32_t g, int32_t nq);
int bkv_stream_attend(const bkv_stream* s, const void* Q, int32_t g, int32_t nq, void* out, float* lse_out,
                      void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- diagnostics: per-launch kernel times ---------------------------------------------------------
 * For callers that want the duration of the individual kernels behind a call (benchmarks): after
 * bkv_profile_enable(n > 0) the library attaches a start and a stop event to each kernel launch (the
 * dispatch's own begin and end; up to n launches; creating the events allocates; not for use under
 * stream capture).  bkv_profile_read waits for the
 * recorded launches, returns how many were written and clears the log.  kind: 0 halving kernel,
 * 2 attend pass, 3 attend merge (1 is not in use); units: tokens the launch consumed.
 * bkv_profile_enable(0) turns it off.  Not thread-safe; off by default.                             */
int bkv_profile_enable(int32_t max_records);
int bkv_profile_read(int32_t* kind, float* ms, int64_t* units, int32_t cap);

/* ---- diagnostics: measured peaks of this GPU --------------------------------------------------------
 * Micro-benchmarks that give the roofline fractions a measured denominator next to the vendor's:
 *   BKV_PEAK_MFMA_BF16    every wavefront of every compute unit issues 32x32x16 bf16 MFMAs back to back  -> FLOP/s
 *   BKV_PEAK_TILE_BF16    the halving kernel's tile routine alone on all compute units: 64x64 Gram tiles of bf16
 *                         rows (d = 128) from LDS, kernel weights exp2(alpha S + row term), signed column sums; no
 *                         walk, no waits, no HBM traffic                                -> FLOP/s of executed MFMA work
 *   BKV_PEAK_STREAM_READ  one pass of 16-byte loads over the workspace                                  -> bytes/s
 *   BKV_PEAK_STREAM_COPY  first half of the workspace copied to the second half                 -> bytes/s (read + written)
 * Runs the kernel `launches` times between two events, waits for them (this call synchronises) and reports the rate
 * and the time of one launch.  workspace: device memory, >= 8 MiB; the streaming kinds move all of it (use >= 1 GiB
 * to get past the caches).                                                                            */
#define BKV_PEAK_MFMA_BF16   0
#define BKV_PEAK_TILE_BF16   1
#define BKV_PEAK_STREAM_READ 2
#define BKV_PEAK_STREAM_COPY 3
int bkv_measure_peak(int32_t kind, int32_t launches, void* workspace, size_t ws_bytes, void* hip_stream,
                     double* per_second, double* ms_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* BALANCEKV_H */
