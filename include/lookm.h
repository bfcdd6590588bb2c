/*
 * liblookm - one-shot, prefill-time KV-cache compression for multimodal prompts (LOOK-M),
 * hand-written HIP kernels for gfx950 (MI355X) behind a plain C ABI.
 *
 * One call compresses the KV cache of one transformer layer of one prompt.  For every head,
 * independently (the paper omits head and layer indices, Section 3.1):
 *   1. accumulated attention scores A_s[j] = sum_i softmax_causal(Q K^T / sqrt(d))[i, j]
 *      (Section 3.2, Eq. 4; the scale is the one of Eq. 3) - never materialising the L x L matrix;
 *   2. text-prior selection: text tokens and the last `recent_window` positions are always
 *      conserved, the rest of the budget goes to the highest-scoring image tokens
 *      (Section 3.2, Eq. 5-8); equal scores go to the lower position;
 *   3. every evicted key is matched to its most cosine-similar conserved key
 *      (Section 3.3, Eq. 9; original keys, ties to the lower position);
 *   4. evicted K/V rows are merged into their match by the averaged (Eq. 10), pivotal (Eq. 11)
 *      or weighted (Eq. 12) rule; values reuse the keys' matching and weights;
 *   5. the conserved, merged rows are written as a compact cache in ascending position order.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are
 *     ordinary host memory.  Nothing here takes or returns framework types.
 *   - Tensors are dense, row-major, innermost stride 1: q, k, v are [H, L, d] (row stride d,
 *     head stride L*d).  Device tensor pointers must be 16-byte aligned.
 *   - The library allocates and frees no memory: inputs, outputs and the scratch `workspace` are
 *     owned by the caller; inputs are never written.  All work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream; lookm_compress_batch_two_streams takes a
 *     second one) and calls do not synchronise (the measurement aids at the end of this header do, and
 *     say so).  The library creates no stream; it keeps no state between calls except "kernel attributes
 *     are set on this device" (see lookm_init).
 *   - The return value reports everything the host can check (negative lookm_status); those checks
 *     run before any kernel is launched and need no GPU.  The one check that needs device data
 *     (budget smaller than the number of protected positions) is reported through `status_out`.
 *   - A pointer to an array that is empty for the given sizes (budget 0, or budget = L) may be NULL.
 *   - Results are deterministic: no floating-point atomics, fixed reduction orders.
 *   - Supported: dt in {LOOKM_F32, LOOKM_BF16}; d a multiple of 8 with 8 <= d <= 256;
 *     1 <= L <= LOOKM_MAX_L; H >= 1 with H*L*d below 2^40 elements.
 */
#ifndef LOOKM_H
#define LOOKM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LOOKM_MAX_L 32768

typedef enum {
    LOOKM_OK = 0,
    LOOKM_ERR_INVALID_ARG = -1,            /* null pointer, non-positive size, misaligned pointer, bad enum */
    LOOKM_ERR_UNSUPPORTED = -2,            /* dtype / head_dim / length outside the supported set */
    LOOKM_ERR_BUDGET_RANGE = -3,           /* budget > L, budget < recent_window, or recent_window > L */
    LOOKM_ERR_BUDGET_BELOW_PROTECTED = -4, /* budget < |text u recent|: they cannot all be conserved */
    LOOKM_ERR_WORKSPACE = -5,              /* workspace missing, misaligned or too small */
    LOOKM_ERR_DEVICE = -6                  /* a HIP runtime call failed */
} lookm_status;

/* Every enumeration that is an ARGUMENT carries two range markers (never valid values): they make each int a
 * representable value of the type, so that a caller's out-of-range value reaches the library's validation
 * (LOOKM_ERR_INVALID_ARG) instead of being undefined behaviour in a C++ translation unit. */
#define LOOKM_ENUM_RANGE_(prefix) prefix##_RANGE_LO_ = -0x7fffffff - 1, prefix##_RANGE_HI_ = 0x7fffffff

typedef enum {
    LOOKM_MERGE_NONE = 0,     /* eviction only: outputs are exact gathers of the conserved rows */
    LOOKM_MERGE_AVERAGED = 1, /* Eq. 10 */
    LOOKM_MERGE_PIVOTAL = 2,  /* Eq. 11 */
    LOOKM_MERGE_WEIGHTED = 3, /* Eq. 12 (taken literally: divisor n+1, weights = matching cosines) */
    LOOKM_ENUM_RANGE_(LOOKM_MERGE)
} lookm_merge_mode;

typedef enum { LOOKM_F32 = 0, LOOKM_BF16 = 1, LOOKM_ENUM_RANGE_(LOOKM_DTYPE) } lookm_dtype;

typedef enum {
    /* text tokens and the recent window are always conserved; a budget below |T u R| is an error */
    LOOKM_SELECT_PROTECT_TEXT = 0,
    /* Eq. 5 and Eq. 8 exactly as printed, for any recent_window <= budget <= L: the N = budget - recent_window
     * places before the window go to the highest boosted scores; when they cannot hold every text token, the
     * text tokens compete for them by score and no image token is conserved.  Same result as
     * LOOKM_SELECT_PROTECT_TEXT whenever that rule accepts the budget. */
    LOOKM_SELECT_LITERAL = 1,
    LOOKM_ENUM_RANGE_(LOOKM_SELECT)
} lookm_select_rule;

/* Library version string, static storage. */
const char* lookm_version(void);

/*
 * Optional: sets, once for the current device, the attributes some kernels need (larger dynamic LDS for every
 * template instance).  Every launching entry point does the same on its first call on a device; a caller that
 * captures HIP graphs calls this once per device beforehand, so that nothing but launches happens under capture.
 * Returns LOOKM_OK or LOOKM_ERR_DEVICE.  Thread-safe.
 */
int lookm_init(void);

/* Human-readable name of a lookm_status value, static storage. */
const char* lookm_status_string(int status);

/*
 * Host helper: the number of protected positions |T u R| for a HOST copy of the modality mask
 * (T = text positions, mask 0; R = the last recent_window positions; Section 3.2).  A caller
 * sizes `budget` with it: budget = protected + number of image tokens to conserve.
 * Returns a negative lookm_status on bad arguments.
 */
int lookm_protected_count(const uint8_t* mask_host, int L, int recent_window);

/*
 * Bytes of device scratch that lookm_compress (and each stage call) needs for these sizes;
 * 0 on invalid sizes.  The workspace must be 256-byte aligned.
 */
size_t lookm_workspace_bytes(int H, int L, int d, int budget, lookm_dtype dt);

/*
 * The whole path (Section 3.2 + 3.3) for one layer.
 *   q, k, v        device, [H, L, d] of dtype dt.
 *   modality_mask  device, uint8 [L]: 1 = image token (evictable), 0 = text token (always conserved);
 *                  shared by all heads.  An all-ones mask switches the text prior off.
 *   budget         B, total rows conserved per head (the paper's S = N + M).  Needs
 *                  recent_window <= B <= L (else LOOKM_ERR_BUDGET_RANGE) and B >= |T u R|
 *                  (else *status_out = LOOKM_ERR_BUDGET_BELOW_PROTECTED and outputs are unspecified).
 *   recent_window  M, the last M positions are always conserved.
 *   k_out, v_out   device, [H, B, d] of dtype dt; row r of head h is the (merged) row of original
 *                  position kept_idx[h, r].  fp32 accumulation, one round-to-nearest-even to bf16.
 *   kept_idx       device, int32 [H, B], strictly ascending original positions.
 *   scores_out     device, float [H, L], the raw A_s of Eq. 4 (no text prior added), or NULL.  With NULL (and
 *                  bf16, d = 128) the second score pass runs only over the keys that compete in the selection -
 *                  image tokens before the recent window - which is faster; the cache comes out bit for bit the same.
 *   status_out     device, int32 [1]: LOOKM_OK or LOOKM_ERR_BUDGET_BELOW_PROTECTED. Must not be NULL.
 *   workspace      device scratch of at least lookm_workspace_bytes(H, L, d, budget, dt) bytes.
 */
int lookm_compress(const void* q, const void* k, const void* v, const uint8_t* modality_mask,
                   int H, int L, int d, lookm_dtype dt,
                   int budget, int recent_window, lookm_merge_mode merge_mode,
                   void* k_out, void* v_out, int32_t* kept_idx,
                   float* scores_out, int32_t* status_out,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- the stages of the path, callable one by one (same conventions) ------------------------------ */

/*
 * Eq. 4: scores_out[h, j] = sum over rows i >= j of exp(q_i.k_j/sqrt(d) - lse_i), where lse_i is the
 * log-sum-exp of row i over columns <= i.  Two flash-style passes over Q K^T (row log-sum-exp, then
 * column sums); bf16 inputs with d = 128 run on the matrix cores with fp32 accumulation.
 *   scores_out  device, float [H, L].
 */
int lookm_scores(const void* q, const void* k, int H, int L, int d, lookm_dtype dt,
                 float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Eq. 5-8: per head, conserve every text position, the last recent_window positions, and the
 * budget - |T u R| image positions outside the window with the highest score (ties -> lower position).
 * The text prior of Eq. 5 is realised as a ranking class (text above any image token), not as a
 * floating-point addition.
 *   scores       device, float [H, L] (any finite values; compared as IEEE floats).
 *   kept_idx     device, int32 [H, budget] ascending.   evicted_idx  device, int32 [H, L - budget] ascending.
 *   status_out   device, int32 [1], as in lookm_compress.
 */
int lookm_select(const float* scores, const uint8_t* modality_mask, int H, int L,
                 int budget, int recent_window,
                 int32_t* kept_idx, int32_t* evicted_idx, int32_t* status_out, void* hip_stream);

/*
 * Eq. 9: for every evicted position e of head h, the slot r in [0, budget) of the conserved key with
 * the highest cosine similarity to key e (original keys; ties -> lower slot, i.e. lower position;
 * a zero-norm key has cosine 0 with everything), and that cosine.
 *   For bf16 keys of 128 dims the choice is the one the definition gives when every cosine is evaluated in binary64
 *   (sums over the dims in order, square roots, one product, one division; first maximum in slot order): the matrix
 *   cores find the candidates, and every candidate that their fp32 values cannot tell from the best is evaluated
 *   again that way.  Other shapes compare fp32 cosines.
 *   kept_idx, evicted_idx  device, as produced by lookm_select (in-range, ascending).
 *   assign  device, int32 [H, L - budget].   sim  device, float [H, L - budget].
 */
int lookm_nearest(const void* k, const int32_t* kept_idx, const int32_t* evicted_idx,
                  int H, int L, int d, lookm_dtype dt, int budget,
                  int32_t* assign, float* sim,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Eq. 10-12 + compaction: x_out[h, r] = merge of row kept_idx[h, r] of x with the rows
 * {evicted_idx[h, e] : assign[h, e] = r}, taken in ascending position, for x in {k, v}.
 *   assign  device, int32 [H, L - budget], values in [0, budget).   sim  device, float [H, L - budget]
 *   (used as weights by LOOKM_MERGE_WEIGHTED; must be a valid array for every merging mode).
 */
int lookm_merge(const void* k, const void* v, const int32_t* kept_idx, const int32_t* evicted_idx,
                const int32_t* assign, const float* sim,
                int H, int L, int d, lookm_dtype dt, int budget, lookm_merge_mode merge_mode,
                void* k_out, void* v_out,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- reuse of the prefill's row log-sum-exp ------------------------------------------------------------ */

/*
 * A flash-style prefill attention kernel already holds, for every query row i, the natural-log
 * log-sum-exp of its scaled causal logits, row_lse[h, i] = log sum_{j<=i} exp(q_i.k_j/sqrt(d)) - the
 * normaliser of the attention weights A_p of Eq. 4.  Handing it over skips the first of the two score
 * passes (half of the path's matrix work).  The values must belong to the same q, k (an inconsistent
 * row_lse scales that row's contribution to every score).
 *   row_lse  device, float [H, L].  Everything else as in lookm_scores / lookm_compress.
 */
int lookm_scores_lse(const void* q, const void* k, const float* row_lse, int H, int L, int d, lookm_dtype dt,
                     float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

int lookm_compress_lse(const void* q, const void* k, const void* v, const uint8_t* modality_mask,
                       const float* row_lse,
                       int H, int L, int d, lookm_dtype dt,
                       int budget, int recent_window, lookm_merge_mode merge_mode,
                       void* k_out, void* v_out, int32_t* kept_idx,
                       float* scores_out, int32_t* status_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- paper-style budgets, the literal form of Eq. 8, several layers / prompts in one call --------------------- */

/*
 * Host helper for the budgets of Section 4 ("Implementation Details"): recent window M = alpha_recent * L,
 * important tokens N = alpha_important * L (each rounded to nearest), cache size S = N + M (Eq. 8).
 * Writes *recent_window = M and *budget = S.  LOOKM_ERR_INVALID_ARG for a ratio outside [0, 1] or a null
 * pointer, LOOKM_ERR_BUDGET_RANGE when M + N > L.  With text-heavy prompts such budgets fall below |T u R|:
 * use them with LOOKM_SELECT_LITERAL.
 */
int lookm_budget_from_ratios(int L, double alpha_recent, double alpha_important, int* recent_window, int* budget);

/*
 * A variant of Eq. 4: only the last `window` query rows are summed, scores_out[h, j] = sum over rows
 * i >= L - window of the attention of row i on key j - the observation-window scoring of the pooling baseline the
 * paper compares with (Section 4.2), on the same kernels; the work drops from L^2 to window * L.  window = L is
 * lookm_scores.  1 <= window <= L, else LOOKM_ERR_INVALID_ARG.  Other arguments as for lookm_scores.
 */
int lookm_scores_window(const void* q, const void* k, int H, int L, int d, lookm_dtype dt, int window,
                        float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Grouped query heads: H query heads in groups of H / kv_heads consecutive heads that share one key head (query head
 * h reads key head h / (H / kv_heads)).  The paper omits head indices (Section 3.1); one cache row then serves a whole
 * group, so its score is the sum of Eq. 4 over the group's query heads, and selection, matching and merging run once
 * per key / value head.
 *   q  device, [H, L, d];  k  device, [kv_heads, L, d];  scores_out  device, float [kv_heads, L].
 *   kv_heads must divide H (else LOOKM_ERR_INVALID_ARG); size the workspace with lookm_workspace_bytes(H, ...).
 */
int lookm_scores_grouped(const void* q, const void* k, int H, int kv_heads, int L, int d, lookm_dtype dt,
                         float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* lookm_select under a chosen rule (lookm_select itself is LOOKM_SELECT_PROTECT_TEXT). */
int lookm_select_rule_(const float* scores, const uint8_t* modality_mask, int H, int L,
                       int budget, int recent_window, lookm_select_rule rule,
                       int32_t* kept_idx, int32_t* evicted_idx, int32_t* status_out, void* hip_stream);

/*
 * One compression job: the arguments of lookm_compress, plus the selection rule and an optional row
 * log-sum-exp (NULL = compute it; see lookm_scores_lse).  All pointers as documented for lookm_compress.
 */
typedef struct lookm_job {
    const void* q;
    const void* k;
    const void* v;
    const uint8_t* modality_mask;
    const float* row_lse;            /* device [H, L] or NULL */
    int H, L, d;
    lookm_dtype dt;
    int budget, recent_window;
    lookm_merge_mode merge_mode;
    lookm_select_rule rule;
    int score_window;                /* 0: Eq. 4 as printed (all query rows); w > 0: see lookm_scores_window */
    int kv_heads;                    /* 0 (or H): one key / value head per query head.  Otherwise grouped query heads,
                                        see lookm_scores_grouped: q and row_lse have H heads; k, v, k_out, v_out,
                                        kept_idx and scores_out have kv_heads heads; kv_heads must divide H */
    void* k_out;
    void* v_out;
    int32_t* kept_idx;
    float* scores_out;               /* or NULL */
    int32_t* status_out;             /* one word per job (jobs may not share it) */
    void* workspace;                 /* jobs may share it: jobs whose memory overlaps run in the order given */
    size_t workspace_bytes;
} lookm_job;

/*
 * The whole path for n_jobs (prompt, layer) pairs - e.g. the 32 layers of each prompt of a batch, of
 * different lengths.  EVERY job is validated before the first launch: on an invalid job nothing is enqueued,
 * the return value is that job's error and *bad_job (if not NULL) its index.  n_jobs = 0 is a no-op.
 *
 * The jobs are enqueued on hip_stream in the order given.
 */
int lookm_compress_batch(const lookm_job* jobs, int n_jobs, int* bad_job, void* hip_stream);

/*
 * The same on two streams of the caller (both of default priority, on the current device, hip_stream_aux different
 * from hip_stream, else LOOKM_ERR_INVALID_ARG).  The result is what running the jobs one after the other in the
 * order given would give.  Jobs that touch disjoint memory need not wait for each other, though: the library
 * alternates such jobs between the two streams, so that the short latency-bound kernels of one job run under the long
 * kernels of another.  Two jobs are kept in order whenever one writes (workspace, k_out, v_out, kept_idx, scores_out,
 * status_out) what the other reads or writes; give independent prompts - or the two halves of one layer's heads -
 * their own workspace and outputs to let them overlap, and pass the jobs in the order a prefill produces them (layer
 * 0 of every prompt, then layer 1, ...).  All work of the call starts after the work already enqueued on hip_stream
 * and is complete before anything enqueued on hip_stream afterwards (event fork / join; no host synchronisation; the
 * events are created and destroyed inside the call, the library keeps no stream and no event).  Work enqueued on
 * hip_stream_aux BEFORE the call is not waited for, and work enqueued there afterwards is ordered only after the
 * jobs that ran on it.  When either stream is being captured into a graph the jobs are simply enqueued in order on
 * hip_stream.
 */
int lookm_compress_batch_two_streams(const lookm_job* jobs, int n_jobs, int* bad_job, void* hip_stream,
                                     void* hip_stream_aux);

/* ---- the step after the path: one new token attends to the (compressed) cache ------------------------------ */

/* Bytes of device scratch lookm_decode_attention needs; 0 on invalid sizes.  256-byte aligned. */
size_t lookm_decode_workspace_bytes(int H, int d);

/*
 * Section 3.1, Eq. 3: out[h] = Softmax(q[h] . K[h]^T / sqrt(d)) V[h] over the first S rows of each head's cache -
 * what every decoding step does with the conserved cache (K_c, V_c) of Eq. 6-7, after the new token's own key
 * and value have been appended (Eq. 2; the caller does that).  The order of the cache rows does not matter.
 *   q        device, [H, d] of dtype dt.
 *   k_cache, v_cache  device, [H, rows, d] of dtype dt (head stride rows * d); rows 0 .. S-1 are attended.
 *   out      device, [H, d] of dtype dt (fp32 accumulation, one rounding).
 *   1 <= S <= rows, else LOOKM_ERR_INVALID_ARG; d as for lookm_compress.
 */
int lookm_decode_attention(const void* q, const void* k_cache, const void* v_cache, int H, int rows, int S, int d,
                           lookm_dtype dt, void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace - code running under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: lookm_decode_attention with its partial results kept in a
 * buffer of LOOKM_DECODE_NOALLOC_SCRATCH_BYTES that the library holds in static device memory (one copy per GPU the
 * library runs on, until the process ends).  Same kernels, same results bit for bit.  The call allocates and frees
 * nothing (its first call on a device, or lookm_init, looks up the buffer's device address).
 *   Sizes whose partial results (H x pieces x (d + 2) floats, pieces <= 256 growing with S) exceed the buffer are
 *   refused with LOOKM_ERR_WORKSPACE before anything is launched; 32 heads x d 128 fit at any S.
 *   All calls on one GPU share the buffer: calls that may overlap in time (different streams, different host
 *   threads) race on it - keep them on one stream or order them yourself.
 * Other arguments and errors as for lookm_decode_attention.
 */
#define LOOKM_DECODE_NOALLOC_SCRATCH_BYTES (8u << 20)
int lookm_decode_attention_noalloc(const void* q, const void* k_cache, const void* v_cache, int H, int rows, int S,
                                   int d, lookm_dtype dt, void* out, void* hip_stream);

/* ---- measurement aid ------------------------------------------------------------------------------- */

/* Intermediate results that lookm_compress (or a job) leaves in its workspace, for callers that want to inspect
 * them (the parity tests do): the evicted positions of Eq. 8's complement, and the matching of Eq. 9. */
typedef enum {
    LOOKM_WS_EVICTED = 0,   /* int32 [kv_heads, L - budget], ascending positions */
    LOOKM_WS_ASSIGN = 1,    /* int32 [kv_heads, L - budget], slot of the matched conserved key */
    LOOKM_WS_SIM = 2,       /* float [kv_heads, L - budget], the matching cosine */
    LOOKM_ENUM_RANGE_(LOOKM_WS)
} lookm_workspace_item;

/*
 * Host helper: byte offset of an intermediate array inside a (256-byte aligned) workspace of the given problem,
 * valid after the work of a lookm_compress / lookm_compress_lse / job call with the same sizes has completed
 * (H query heads, kv_heads key / value heads; kv_heads = H without grouped query heads).  Returns (size_t)-1 on
 * invalid sizes or item.  The arrays hold what the call computed when it merged (merge_mode != NONE, 0 < budget < L).
 */
size_t lookm_workspace_offset(int H, int kv_heads, int L, int d, int budget, lookm_dtype dt, lookm_workspace_item item);

/* Kernels of the path, in launch order (Section 3.2: the two score passes and the selection;
 * Section 3.3: key norms, matching, similarity sets, merge + compaction).  For bf16 with d = 128 the key norms are
 * written by score pass 2 and no norm kernel is launched: that slot then reads the cost of an empty event interval. */
enum {
    LOOKM_K_SCORE_LSE = 0, LOOKM_K_SCORE_LSE_FOLD = 1,        /* pass 1 and the fold of its chunk partials */
    LOOKM_K_SCORE_COLSUM = 2, LOOKM_K_SCORE_COLSUM_FOLD = 3,  /* pass 2 and the fold of its chunk partials */
    LOOKM_K_SELECT = 4, LOOKM_K_RNORM = 5, LOOKM_K_NEAREST = 6, LOOKM_K_NEAREST_FOLD = 7,
    LOOKM_K_BUCKET = 8, LOOKM_K_MERGE = 9, LOOKM_N_KERNELS = 10
};

/*
 * lookm_compress, run `reps` times with a HIP event recorded on `hip_stream` after every kernel.
 * Unlike every other call it SYNCHRONISES the stream (once per repetition) and creates / destroys
 * HIP events.  kernel_ms_host: host, float [LOOKM_N_KERNELS], average milliseconds per kernel
 * (0 for a kernel the given sizes skip).  All other arguments and results as for lookm_compress.
 */
int lookm_compress_profile(const void* q, const void* k, const void* v, const uint8_t* modality_mask,
                           int H, int L, int d, lookm_dtype dt,
                           int budget, int recent_window, lookm_merge_mode merge_mode,
                           void* k_out, void* v_out, int32_t* kept_idx,
                           float* scores_out, int32_t* status_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream,
                           int reps, float* kernel_ms_host);

/* The same for any job (selection rule, observation window, supplied row log-sum-exp). */
int lookm_job_profile(const lookm_job* job, int reps, float* kernel_ms_host, void* hip_stream);

/*
 * Measurement aid, no part of the method (for callers that want the realistic ceiling of the MFMA-bound kernels
 * next to the datasheet peak): the rate at which this GPU sustains the bf16 MFMA instructions the score and matching
 * kernels are built on, from registers alone - 8 A and 16 B fragments per wave, blocks of 64 x 32 x 128 multiply-adds
 * as 16 MFMAs of 32x32x16 in two accumulator chains (the matching kernel's block) or as 32 MFMAs of 16x16x32 on eight
 * accumulators (the score kernels' block), no memory traffic.
 *   random_operands  0: every operand element is 1.0, 32x32x16;  1: pseudo-random bf16 values of magnitude [0.25, 4)
 *                    that differ from instruction to instruction, as real queries and keys do (the chip sustains
 *                    less then), 32x32x16;  2: the same operands through 16x16x32
 *   waves_per_simd   1..3: the grid is (compute units x waves_per_simd) workgroups of 256 threads
 *   iters            1..2^20 blocks per wave and launch;  reps  1..1000 launches, the first half untimed
 *   tflops_host      host, one float: 2*64*32*128 flop per block over the time of the timed launches, in TFLOP/s
 *   workspace        device, at least compute units x waves_per_simd x 1024 bytes (1 MiB always suffices), written
 * Like the profile calls it SYNCHRONISES the stream and creates / destroys two HIP events.  Errors: INVALID_ARG
 * for a null pointer or a count outside the ranges above, WORKSPACE for a workspace that is too small, DEVICE.
 */
int lookm_probe_mfma(int random_operands, int waves_per_simd, int iters, int reps, float* tflops_host,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LOOKM_H */
