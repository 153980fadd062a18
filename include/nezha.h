/* nezha.h - C ABI of the MI355X (gfx950) implementation of NEZHA's decoding
 * step: batched self-drafting of semantic-ID items by beam search over the
 * codebook levels (Sec. 3.2, Eq. 1-3; Alg. 3, inference part) followed by the
 * model-free hash-set verification of the drafted tuples (Sec. 3.3, Eq. 4-5).
 *
 * Notation follows the paper: L levels, T_l codes at level l ("radices"), beam
 * size K, h_l the backbone's hidden state at placeholder l, s_l / c_l the
 * draft head's state, V the set of valid item indices.
 *
 * General rules
 *  - Every function returns NEZHA_OK (0) or a negative error code and never
 *    throws.  nezha_last_error() gives a text for the last failure on the
 *    calling thread.
 *  - All argument checks run on the host before anything is enqueued, so a
 *    failed call has no effect on the device.
 *  - "device pointer" = memory of the current HIP device; "host pointer" =
 *    ordinary process memory.  Inputs are borrowed and never written.
 *    Outputs and workspaces are allocated by the caller.  The only memory the
 *    library owns is inside a nezha_itemset.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    nezha_verify_tuples and nezha_draft_step only enqueue work on it and
 *    return; they never synchronise and never allocate, so they can be
 *    captured into a HIP graph.
 *  - Inputs must be finite (no NaN / inf).
 */
#ifndef NEZHA_H_
#define NEZHA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nezha_itemset nezha_itemset; /* opaque, device resident, owned by the library */

typedef enum { NEZHA_F32 = 0, NEZHA_BF16 = 1 } nezha_dtype;

enum {
  NEZHA_OK = 0,
  NEZHA_EINVAL = -1, /* bad argument (null pointer, size or shape outside the supported range) */
  NEZHA_ENOMEM = -2, /* device or host allocation failed */
  NEZHA_EHIP = -3,   /* a HIP runtime call failed */
  NEZHA_ERANGE = -4, /* prod T_l >= 2^64-1, or a catalog code outside [0, T_l) */
  NEZHA_EFULL = -5   /* the hash table could not take every key (should not happen) */
};

/* Limits of this implementation. */
#define NEZHA_MAX_LEVELS 8
#define NEZHA_MAX_BEAM 128       /* K and K_in of the in-register / in-LDS kernels */
#define NEZHA_MAX_WIDE_BEAM 1024 /* K and K_in overall: wider beams than NEZHA_MAX_BEAM take a path
                                    that keeps the level's logits in the workspace */

const char* nezha_last_error(void); /* thread local, never NULL */

/* ---- the set of valid items V (Sec. 3.3: "a hash set", pre-computed) ------------------
 *
 * Builds the set { P(v) : v in catalog } where P is the mixed-radix index of
 * Eq. 4 (level 1 is the least significant digit).
 *   codes       int32 [n, L] row major, tuple i = codes[i*L .. i*L+L-1], level 1 first;
 *               host pointer if codes_on_device == 0, else device pointer.  n >= 0.
 *   radices     host int32 [L] = T_1..T_L, each >= 1, 1 <= L <= NEZHA_MAX_LEVELS,
 *               prod T_l <= 2^64 - 1 (the value 2^64-1 is reserved for "empty").
 *   load_factor in (0, 0.9]; the table gets ceil(n / load_factor) key slots,
 *               rounded up to whole 64-byte buckets.
 *               Beside the table the set keeps a prefilter of about four bytes per item (bitmaps
 *               of the last codes present, in 64-byte blocks chosen by the prefix) that the draft
 *               step consults before the table: it can only rule keys out that are not in the set.
 * Duplicate tuples are stored once.  A code outside [0, T_l) gives NEZHA_ERANGE.
 * The work runs on hip_stream and the call waits for it (building is an offline
 * step in the paper).  On success *out holds the new set.  On any failure *out is NULL and
 * everything the call had allocated has been released.  (Test aid: with NEZHA_TEST_FAIL_ALLOC=N
 * in the environment the N-th allocation of a build -- 1 the handle, 2 the table, 3 status words,
 * then the staging buffer for a host catalog, last the prefilter -- is treated as failed:
 * NEZHA_ENOMEM, except for the prefilter, without which the set still works.) */
int nezha_build_itemset(const int32_t* codes, int64_t n, int32_t L, const int32_t* radices,
                        int codes_on_device, double load_factor, void* hip_stream,
                        nezha_itemset** out);

/* Any of the output pointers may be NULL.  radices: host int32 [L]. */
int nezha_itemset_info(const nezha_itemset* set, int64_t* n_distinct, int64_t* n_slots,
                       int32_t* L, int32_t* radices);

/* Frees the set (NULL is accepted).  The caller makes sure no enqueued work still uses it.  The
 * library keeps a registry of the sets it has handed out: a pointer that is not (or no longer) one
 * of them -- freed before, or never a set -- gives NEZHA_EINVAL here and in every call that takes
 * a set, and its memory is not read. */
int nezha_free_itemset(nezha_itemset* set);

/* Self-check of a built set (Sec. 3.3: the set must hold every valid item, or valid drafts would
 * be dropped): looks every tuple of `codes` up the way the draft step does -- through the
 * prefilter, then the table -- and returns in *n_missing how many were not found.  Called with
 * the catalog the set was built from, the answer must be 0.  codes as for nezha_build_itemset
 * (host or device pointer, int32 [n, L of the set]).  Allocates a few bytes (plus a staging buffer
 * for host codes) and waits for hip_stream: an offline call, like the build. */
int nezha_check_itemset(const nezha_itemset* set, const int32_t* codes, int64_t n,
                        int codes_on_device, void* hip_stream, int64_t* n_missing);

/* ---- stand-alone verification (Eq. 4 + Eq. 5 on a batch of tuples) ---------------------
 *
 *   codes      device int32 [n, L] (L of the set), n >= 0
 *   out_mask   device uint8 [n]: 1 if the tuple is a valid item, else 0.  A tuple
 *              with a code outside [0, T_l) is rejected (0); it is not an error.
 *   out_index  device int64 [n] or NULL: the indices i of the accepted tuples in
 *              ascending order (Eq. 5 filters "in place": order is kept);
 *              entries beyond the count are left untouched.
 *   out_count  device int64 [1] or NULL: number of accepted tuples.
 *   workspace  device memory of at least nezha_verify_workspace(n) bytes, 16-byte
 *              aligned; contents are scratch. */
int nezha_verify_tuples(const nezha_itemset* set, const int32_t* codes, int64_t n,
                        uint8_t* out_mask, int64_t* out_index, int64_t* out_count,
                        void* workspace, size_t workspace_bytes, void* hip_stream);
size_t nezha_verify_workspace(int64_t n);

/* nezha_verify_tuples for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation): the same kernels, with the block counts and offsets in a fixed array of
 * NEZHA_VERIFY_STATIC_MAX / 1024 * 12 bytes (384 KiB) that is part of the library's device code
 * (one copy per GPU, held until the process ends).  Arguments, results and error behaviour as for
 * nezha_verify_tuples, without workspace; n above NEZHA_VERIFY_STATIC_MAX gives NEZHA_EINVAL.
 * The call allocates nothing (the first call on a device asks the runtime for the array's address,
 * which is kept).  All calls on one GPU share that array: calls whose work overlaps on one GPU
 * (two streams, two threads) race; issue them on one stream or wait between them. */
#define NEZHA_VERIFY_STATIC_MAX (32 * 1024 * 1024)
int nezha_verify_tuples_static(const nezha_itemset* set, const int32_t* codes, int64_t n,
                               uint8_t* out_mask, int64_t* out_index, int64_t* out_count,
                               void* hip_stream);

/* ---- one level of the draft head's beam search (Alg. 3, inference loop body) -----------
 *
 * For each of B requests and each of its K_in live beams (rank order) the call
 *   1. forms the logits of Eq. 2, z = [h_l ; c] W_l (one linear layer on the
 *      concatenation of the placeholder hidden state and the beam's state, no
 *      bias), and their log-softmax over the T_level codes;
 *   2. takes the beam's K most probable codes (equal values: lower code first);
 *   3. gives each candidate the cumulative score parent_score + logp (float32;
 *      the log of the paper's cumulative probability) and the index
 *      parent_key + code * prod_{j<level} T_j (Eq. 4, one more digit);
 *   4. with a set given whose tuples have `level` digits (at level == L: the item
 *      set of Eq. 5; below it: a set of valid prefixes, the per-level filter the
 *      paper mentions in passing), drops every candidate whose index is not in it;
 *   5. keeps the K candidates of largest score (ties: lower parent rank, then
 *      better within-beam rank), in non-increasing score order;
 *   6. at level < L, forms each survivor's next state by Eq. 3: with the additive
 *      Transition c' = c_parent + E_l[code], or with the recurrent one (Sec. 3.2
 *      "an RNN"; read as a bias-free Elman cell) c' = tanh(U_l c_parent + E_l[code]).
 * A beam slot whose key_in is 2^64-1 is empty (the level before kept fewer than K beams)
 * and has no children.
 */
#define NEZHA_TRANSITION_ADD 0
#define NEZHA_TRANSITION_RNN 1
typedef struct {
  int32_t B;              /* requests in the batch, >= 0 */
  int32_t L;              /* levels of the semantic ID */
  int32_t level;          /* this call's level, 1..L */
  int32_t K;              /* beams kept, 1 <= K <= min(T_level, NEZHA_MAX_WIDE_BEAM) */
  int32_t K_in;           /* live beams entering: 1 at level 1, else K of the previous call */
  int32_t d;              /* width of h_l */
  int32_t e;              /* width of the state c and of the code embeddings */
  const int32_t* radices; /* host int32 [L] */
  nezha_dtype dtype;      /* of H, W, E and the states; scores are always float32 */
  int64_t h_row_stride;   /* elements between consecutive requests in H_l (>= d) */
  int32_t w_packed;       /* 0: W_l is row major; 1: W_l was written by nezha_pack_weights */
  const float* user_part; /* optional device float32 [B, T_level], 16-byte aligned: h_l W_l[0:d]
                             formed beforehand (nezha_user_projection[_levels]); then H_l is not
                             read.  NULL: the call forms it itself */
  int32_t transition;     /* NEZHA_TRANSITION_ADD or NEZHA_TRANSITION_RNN (used when level < L) */
  const void* U_l;        /* NEZHA_TRANSITION_RNN: device [e, e] row major, same dtype as the
                             states, 16-byte aligned: c'[j] = tanh(sum_i U_l[j][i] c[i] + E_l[code][j]).
                             Ignored (may be NULL) otherwise */
  const void* state_init; /* read by nezha_draft_levels and nezha_decode only: the state the single
                             beam of level 1 starts from (Eq. 1: the initial context state),
                             device [B, 1, e], 16-byte aligned; NULL = zeros.  nezha_draft_step
                             takes it as its state_in argument instead */
} nezha_step_desc;

/* All data pointers are device pointers.
 *   in:  H_l [B, d] (row b at H_l + b*h_row_stride); W_l [(d+e), T_level] row major,
 *        rows 0..d-1 act on h_l, rows d..d+e-1 on the state; E_l [T_level, e]
 *        (ignored when level == L, may be NULL there); state_in [B, K_in, e]
 *        (NULL = all zero, the initial state); key_in uint64 [B, K_in] and
 *        score_in float32 [B, K_in] (NULL = 0, the empty prefix);
 *        set: NULL = no verification.  Built over all L radices it is consulted when
 *        level == L (and ignored below); built over the first `level` radices (a set of
 *        prefixes) it is consulted at this level.  Any other length is NEZHA_EINVAL.
 *   out: key_out uint64 [B, K], score_out float32 [B, K], parent_out int32 [B, K]
 *        (rank of the parent beam), code_out int32 [B, K], state_out [B, K, e]
 *        (NULL allowed when level == L), count_out int32 [B] (NULL allowed):
 *        number of beams kept, = K unless verification left fewer.  Slots at or
 *        beyond the count hold key 2^64-1, score -inf, parent -1, code -1, state 0.
 *   workspace: device memory of at least nezha_draft_step_workspace(desc) bytes,
 *        256-byte aligned; scratch.
 * Alignment: E_l and the states 16 bytes; H_l (every row) and W_l 16 bytes with NEZHA_BF16,
 * 4 bytes with NEZHA_F32.
 * Shape limits: K, K_in <= NEZHA_MAX_WIDE_BEAM (the recall setting of Sec. 1: beam 512 to
 * 1000; above NEZHA_MAX_BEAM the workspace also holds 4 * B * K_in * T_level bytes of logits
 * and K_in * T_level must stay below 2^31); T_level a multiple of 16; with
 * NEZHA_BF16 d and e multiples of 32, with NEZHA_F32 d >= 1 and e a multiple
 * of 4; e <= 256.  Anything else gives NEZHA_EINVAL. */
int nezha_draft_step(const nezha_step_desc* desc, const void* H_l, const void* W_l,
                     const void* E_l, const void* state_in, const uint64_t* key_in,
                     const float* score_in, const nezha_itemset* set, uint64_t* key_out,
                     float* score_out, int32_t* parent_out, int32_t* code_out,
                     void* state_out, int32_t* count_out, void* workspace,
                     size_t workspace_bytes, void* hip_stream);
size_t nezha_draft_step_workspace(const nezha_step_desc* desc); /* 0 if desc is invalid */

/* All L levels of the inference loop of Alg. 3 in one call: exactly what L calls of
 * nezha_draft_step do with level = 1..L, K_in = 1 at level 1 and K after it, each level's
 * key_out / score_out / state_out feeding the next level's key_in / score_in / state_in.
 * desc gives B, L, K, d, e, radices, dtype, h_row_stride, w_packed, transition and state_init
 * for all levels; its level, K_in, user_part and U_l are not read (they come from io[l-1]).  The
 * arguments of all L levels are checked before anything is enqueued.  io: host
 * array of L entries; the pointers in it follow the rules of the like-named arguments of
 * nezha_draft_step (device memory; set = items at level L or prefixes of length l below it or
 * NULL; user_part and U_l optional).  When every level is small enough for the single-launch
 * level kernel (NEZHA_BF16, packed weights, K <= 32, T_l <= 512) and every io[l-1].user_part is
 * given, one kernel launch runs all levels; otherwise the levels are launched one after the
 * other.  workspace: at least nezha_draft_levels_workspace(desc) bytes, 256-byte aligned.
 * Asynchronous on hip_stream; allocates nothing. */
typedef struct {
  const void* H_l;            /* [B, d] hidden states of this level (may be NULL with user_part) */
  const void* W_l;            /* weights of this level (packed when desc->w_packed) */
  const void* E_l;            /* code embeddings (NULL allowed at level L) */
  const nezha_itemset* set;   /* or NULL */
  const float* user_part;     /* or NULL */
  const void* U_l;            /* NEZHA_TRANSITION_RNN: [e, e]; else NULL */
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;            /* NULL allowed at level L */
  int32_t* count_out;         /* or NULL */
} nezha_level_io;
int nezha_draft_levels(const nezha_step_desc* desc, const nezha_level_io* io, void* workspace,
                       size_t workspace_bytes, void* hip_stream);
size_t nezha_draft_levels_workspace(const nezha_step_desc* desc); /* 0 if desc is invalid */

/* One decode of a batch in one call: the user parts of all L levels (the beam-independent part
 * of Eq. 2, as nezha_user_projection_levels forms them) followed by the L levels of the loop of
 * Alg. 3 (as nezha_draft_levels runs them).  NEZHA_BF16 with desc->w_packed = 1 only.  io as for
 * nezha_draft_levels, with every io[l-1].H_l given and every io[l-1].user_part pointing to
 * float32 [B, T_l] device memory that this call WRITES (the level's user part) before the level
 * reads it.  A serving loop that calls this once per batch pays one host call per decode.
 * Asynchronous on hip_stream; allocates nothing; workspace as for nezha_draft_levels. */
int nezha_decode(const nezha_step_desc* desc, const nezha_level_io* io, void* workspace,
                 size_t workspace_bytes, void* hip_stream);

/* The user parts of levels 1..n_levels in one launch.  They do not depend on the beams, and all
 * hidden states h_1..h_L come out of the same prefill, so they can be formed before the level
 * loop and handed to nezha_draft_step through desc->user_part.  H, W_packed, A_out: host arrays
 * of n_levels device pointers: H[i] = hidden states of level i+1 ([B, d], rows h_row_stride
 * apart), W_packed[i] = that level's weights from nezha_pack_weights, A_out[i] = float32
 * [B, T_{i+1}].  NEZHA_BF16 with desc->w_packed = 1 only; level, K, K_in of desc are not used.
 * Asynchronous on hip_stream; allocates nothing. */
int nezha_user_projection_levels(const nezha_step_desc* desc, int32_t n_levels,
                                 const void* const* H, const void* const* W_packed,
                                 float* const* A_out, void* hip_stream);

/* The head's weights are trained parameters and do not change between calls, so their
 * rearrangement into the order the matrix instructions read (done inside nezha_draft_step on
 * every call when w_packed == 0) can be done once: nezha_pack_weights writes that form of W_l
 * (NEZHA_BF16 only; desc gives d, e, radices, level) into W_packed, device memory of
 * nezha_packed_weights_bytes(desc) bytes, 16-byte aligned, which is then passed as W_l with
 * desc->w_packed = 1.  Asynchronous on hip_stream; allocates nothing. */
size_t nezha_packed_weights_bytes(const nezha_step_desc* desc); /* 0 if not applicable */
int nezha_pack_weights(const nezha_step_desc* desc, const void* W_l, void* W_packed,
                       void* hip_stream);

/* The beam-independent part of Eq. 2 alone: A_out[b, :] = h_{b,l} W_l[0:d, :] as float32
 * [B, T_level] (these are the level-1 logits, where the state is zero).  Same desc, H_l, W_l,
 * alignment and workspace rules as nezha_draft_step; K, K_in and the outputs are not used.
 * Asynchronous on hip_stream. */
int nezha_user_projection(const nezha_step_desc* desc, const void* H_l, const void* W_l,
                          float* A_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* ---- per-kernel timing (measurement aid, not part of the paper's method) -----------------
 * While enabled, every kernel launch of the library is bracketed by two HIP events on the
 * launch stream (this creates events, so calls made while it is on cannot be captured into a
 * graph).  nezha_profile_read waits for the events of one kernel kind (0 <=
 * kind < nezha_profile_kinds()) and returns its name, number of launches and summed
 * duration in milliseconds; nezha_profile_reset drops all records. */
int nezha_profile_enable(int on);
int nezha_profile_reset(void);
int nezha_profile_kinds(void);
int nezha_profile_read(int kind, const char** name, int64_t* launches, double* total_ms);
/* What the same event bracket reports for an EMPTY kernel (mean over `launches` launches on
 * hip_stream, microseconds): the dispatch latency that every duration from nezha_profile_read
 * contains on top of the kernel's own run time (a profiler's kernel trace does not count it).
 * Waits for the stream. */
int nezha_profile_event_overhead(int launches, void* hip_stream, double* mean_us);

/* Measurement aid for the verifier's roofline: n independent reads of whole, aligned lines of
 * line_bytes (64 or 128) at pseudo-random places of the device buffer buf (bytes long, 128-byte
 * aligned), four reads in flight per lane as in the verifier.  Timing n * line_bytes against the
 * kernel's duration gives the random-access bandwidth the memory system can actually deliver
 * for that buffer size.  sink: device uint64 [1], scratch.  Asynchronous on hip_stream. */
int nezha_bench_random_gather(const void* buf, size_t bytes, int64_t n, int line_bytes,
                              uint64_t seed, void* sink, void* hip_stream);
/* The same with the number of lines in flight chosen: depth = 1, 2, 4, 8 or 16 (16: 64-byte
 * lines only) per lane, or, with lanes_per_line = 8 (64-byte lines), per group of eight lanes that
 * read each line together, eight bytes apiece.  The best of these forms is what "achievable
 * random-access rate" means in the verifier's roofline: a denominator that does not copy the
 * verifier's own launch shape. */
int nezha_bench_random_gather_depth(const void* buf, size_t bytes, int64_t n, int line_bytes,
                                    int depth, int lanes_per_line, uint64_t seed, void* sink,
                                    void* hip_stream);

/* Measurement aid for the projections' roofline: `workgroups` workgroups of four waves (one wave
 * per SIMD, as in the large projection kernel) each run `iters` iterations of 32 independent
 * 32x32x16 bf16 matrix instructions on operand values taken from `operands` (device, `bytes`
 * long, 16-byte aligned; pass the hidden states or weights of the workload: the clock the chip
 * sustains under matrix load depends on the values) and record, per workgroup, the core-clock
 * cycles and the ticks of the constant 100 MHz counter the loop took: ticks[2*w], ticks[2*w+1]
 * (device uint64 [2 * workgroups]).  flops = workgroups * 4 * iters * 32 * 32768; clock = 100 MHz
 * * cycles / ticks.  sink: device float [1], scratch.  Asynchronous on hip_stream. */
int nezha_bench_mfma_rate(const void* operands, size_t bytes, int iters, int workgroups,
                          uint64_t* ticks, float* sink, void* hip_stream);

/* Measurement aid for the per-request expansion's roofline (Alg. 3's expansion at K_in >= 16):
 * `workgroups` workgroups of four waves each run `iters` tile steps of that kernel's first sweep
 * without its LDS traffic: mode 0 the four dependent 16x16x32 bf16 matrix instructions of one
 * 16 x 16 logit tile at e = 128 alone, mode 1 the vector work on one tile alone (per lane four
 * fused multiply-adds, exponentials and additions, two conversions to packed halves, two packed
 * maxima), mode 2 both, interleaved as the kernel issues them.  With workgroups = (compute units)
 * * w every SIMD holds w waves.  values: device float [256] that the operands are formed from.
 * ticks (device uint64 [2 * workgroups]): core-clock cycles and ticks of the constant 100 MHz
 * counter per workgroup.  Tile steps = workgroups * 4 * iters.  sink: device float [1], scratch.
 * Asynchronous on hip_stream. */
int nezha_bench_tile_step(int mode, int iters, int workgroups, const float* values,
                          uint64_t* ticks, float* sink, void* hip_stream);

/* Inverse of Eq. 4 on the host: keys[n] -> codes int32 [n, L] (level 1 first).  Host pointers. */
int nezha_unpack_keys(const uint64_t* keys, int64_t n, int32_t L, const int32_t* radices,
                      int32_t* codes);

#ifdef __cplusplus
}
#endif
#endif /* NEZHA_H_ */
