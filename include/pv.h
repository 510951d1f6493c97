/* pv.h -- C ABI of the parallel-prefix-verification attention library (AMD MI355X, gfx950).
 *
 * The library evaluates, for one transformer layer, the attention of the single forward pass
 * in which K short suffix copies ("segments") are appended after a full draft and judged at
 * once (paper section "Parallel Prefix Verification"): prompt and draft tokens attend causally;
 * segment k attends to the prompt, to the first p_k draft tokens, and causally to itself,
 * never to another segment; its rotary positions continue from the end of the prefix it
 * judges.  A readout turns the per-segment Correct/Incorrect logits into the maximal valid
 * prefix (appendix "Notation and judge calibration", "Parallel partial verify",
 * "Adopted-prefix length").
 *
 * Conventions shared by every entry point
 *   Layout     Packed variable length: the tokens of all requests are concatenated; request b
 *              owns rows [tok_start[b], tok_start[b+1]) in the order
 *              [prompt | draft | segment_0 | ... | segment_{K-1}] (PV_LAYOUT_APPENDED), or with
 *              every segment directly after the draft tokens it judges,
 *              [prompt | draft[0:p_0] | segment_0 | draft[p_0:p_1] | segment_1 | ... | draft[p_{K-1}:T]]
 *              (PV_LAYOUT_INTERLEAVED, the packing of appendix "Parallel partial verify").  Both
 *              hold the same tokens with the same visibility and positions; only the row order of
 *              the caller's tensors differs.  Q and O are
 *              [total_tokens][Hq][D], K and V are [total_tokens][Hkv][D], innermost contiguous,
 *              base pointers 16-byte aligned.
 *   Memory     "host" pointers are ordinary CPU memory read only during the call.  "device"
 *              pointers are GPU memory owned by the caller (e.g. a torch tensor); the library
 *              never allocates or frees device memory, never synchronises, never creates
 *              streams.  All GPU work is enqueued on the caller's stream (a hipStream_t passed
 *              as void*; NULL = the default stream) and outputs are valid once that stream
 *              has reached the end of the enqueued work.
 *   Errors     Every call returns a pv_status.  Argument errors are detected on the host
 *              before anything is launched (nothing has been enqueued when an error other
 *              than PV_ERR_HIP is returned).  A failing HIP call maps to PV_ERR_HIP and the
 *              raw hipError_t is kept per thread for pv_last_hip_error().
 *   Determinism Fixed tile order and no atomics: results are bit-identical run to run.
 */
#ifndef PV_H_
#define PV_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t pv_status;
enum {
  PV_OK = 0,
  PV_ERR_NULL = -1,       /* a required pointer is NULL */
  PV_ERR_SHAPE = -2,      /* bad batch / lengths / head counts / head_dim / sizes struct */
  PV_ERR_BOUNDARY = -3,   /* boundaries not non-decreasing or outside [0, T] */
  PV_ERR_WORKSPACE = -4,  /* plan / mask / workspace buffer smaller than pv_query_sizes says */
  PV_ERR_ALIGN = -5,      /* a device pointer is not 16-byte aligned */
  PV_ERR_DTYPE = -6,      /* unsupported dtype combination */
  PV_ERR_ARCH = -7,       /* current device is not gfx950 */
  PV_ERR_HIP = -8         /* a HIP runtime call failed, see pv_last_hip_error() */
};

enum { PV_BF16 = 0, PV_F32 = 1 };
enum { PV_LAYOUT_APPENDED = 0, PV_LAYOUT_INTERLEAVED = 1 };

/* Rows that see at most this many keys (the first tokens of a request, or a segment whose prefix is
 * almost empty) are evaluated in plain fp32 by the bf16 path: with so few terms the bf16 rounding
 * of the operands is not averaged out and would dominate the error of the whole output. */
enum { PV_SHORT_ROW_KEYS = 16 };

/* Structure of a packed verification batch.  HOST memory, owned by the caller. */
typedef struct {
  int32_t batch;                 /* B >= 1 */
  const int32_t* prompt_len;     /* [B]  P_b >= 0 */
  const int32_t* draft_len;      /* [B]  T_b >= 1 */
  const int32_t* num_segments;   /* [B]  K_b >= 0   (0 => plain causal attention) */
  const int32_t* segment_len;    /* [B]  S_b >= 1   (same for all segments of a request) */
  const int32_t* boundaries;     /* [sum K_b] p_k = number of draft tokens segment k sees;
                                    per request non-decreasing and 0 <= p_k <= T_b */
  int32_t layout;                /* PV_LAYOUT_APPENDED or PV_LAYOUT_INTERLEAVED (whole batch) */
} pv_problem;

/* Sizes derived from a pv_problem; filled by pv_query_sizes, passed back to the other calls. */
typedef struct {
  int64_t batch;
  int64_t total_tokens;          /* sum_b (P_b + T_b + K_b * S_b) */
  int64_t total_segments;        /* sum_b K_b */
  int64_t max_seq_len;           /* max_b N_b */
  int64_t n_q_tiles;             /* work items per kv head */
  int64_t padded_keys;           /* sum_b N_b rounded up to the key tile */
  int64_t plan_bytes;            /* device bytes pv_build_mask writes */
  int64_t dense_mask_bytes;      /* sum_b N_b^2 (uint8), only if the dense mask is requested */
  int64_t attn_workspace_bytes;  /* device scratch pv_masked_attention needs */
  int32_t n_q_heads, n_kv_heads, head_dim, in_dtype;
  int32_t tile_m, tile_n;        /* query tokens per work item, keys per tile */
  int32_t n_short_rows;          /* rows with at most PV_SHORT_ROW_KEYS visible keys (see below) */
  int32_t layout;                /* the problem's layout */
  int32_t n_seg_tiles;           /* query tiles that hold at least one segment row */
  int32_t n_quads;               /* groups of four consecutive query tiles of a request; 0 unless
                                    Hq/Hkv is a group size whose kernels take them as work items */
  int32_t n_short_seg_rows;      /* those of the n_short_rows that are segment rows */
} pv_sizes;

/* Host only: validates the problem and the head configuration and fills `out`.
 * Supported: head_dim 64 or 128, Hq <= 1024 a multiple of Hkv with Hq/Hkv <= 8, in_dtype PV_BF16
 * (MFMA path) or PV_F32 (debug path).  Limits (PV_ERR_SHAPE beyond them): B <= 2^20, N_b <= 2^24,
 * total_tokens and padded_keys <= 2^27, so that every index of the plan fits int32.  A problem
 * inside these limits whose kernels would still need a grid of 2^32 threads or more (for
 * instance more than 2^24 work items times kv heads) is refused at launch time: PV_ERR_HIP with
 * hipErrorInvalidConfiguration, nothing truncated. */
pv_status pv_query_sizes(const pv_problem* problem, int32_t n_q_heads, int32_t n_kv_heads,
                         int32_t head_dim, int32_t in_dtype, pv_sizes* out);

/* The prefix attention mask of "Parallel Prefix Verification" as a device-resident plan:
 * per token its rotary position and the row descriptor (a_end, b_start) such that key j of the
 * same request is visible to query i iff j < a_end or b_start <= j <= i; per segment the row
 * that carries its verdict (its last token); and the list of query tiles with the key-tile
 * ranges that contain at least one visible pair (fully masked tiles are never listed), ordered
 * longest first.
 *   problem         host, validated again here
 *   plan_dev        device, >= sizes->plan_bytes, 16-byte aligned; opaque, position independent
 *   dense_mask_dev  device or NULL.  If given, also writes the mask entry by entry (uint8 0/1,
 *                   request b at byte offset sum_{b'<b} N_b'^2, row-major [N_b][N_b]); meant
 *                   for tests, sizes->dense_mask_bytes bytes. */
pv_status pv_build_mask(const pv_problem* problem, const pv_sizes* sizes, void* plan_dev,
                        int64_t plan_bytes, uint8_t* dense_mask_dev, int64_t dense_mask_bytes,
                        void* stream);

/* O = softmax(mask(Q K^T * scale)) V under the plan's mask, with rotary embedding applied to Q
 * and K at the plan's positions (angle pos * theta^(-2c/D) on the pair (c, c + D/2)).
 *   q, k, v          device, in_dtype, layout above; not modified
 *   out              device, out_dtype, [total_tokens][Hq][D]
 *   lse              device or NULL: natural-log softmax normaliser, float [Hq][total_tokens]
 *   in_dtype/out_dtype  PV_BF16 in -> PV_BF16 or PV_F32 out (bf16 MFMA, fp32 accumulate);
 *                       PV_F32 in  -> PV_F32 out (fp32 debug path)
 *   softmax_scale    0 => 1/sqrt(D)
 *   rope_theta       0 => no rotation
 *   workspace        device scratch, >= sizes->attn_workspace_bytes, 16-byte aligned */
pv_status pv_masked_attention(const pv_sizes* sizes, const void* plan_dev, const void* q,
                              const void* k, const void* v, void* out, float* lse,
                              int32_t out_dtype, float softmax_scale, float rope_theta,
                              void* workspace, int64_t workspace_bytes, void* stream);

/* The same attention for the rows of the segments only ("extend" use: the prompt and draft rows
 * were evaluated by an earlier pass, e.g. the full-answer verification, and only the K*S judge rows
 * are wanted).  Arguments as for pv_masked_attention, bf16 inputs only (PV_ERR_DTYPE otherwise).
 * K and V must still hold every token (the keys of prompt and draft are what the segments attend
 * to); the Q rows of prompt and draft tokens are not read.  Writes `out` (and `lse`) for segment
 * rows only and leaves all other rows untouched.  Few, long work items are split along the keys
 * into pieces that run in parallel and are merged afterwards, with partial results in the
 * workspace (attn_workspace_bytes covers them); every segment row gets the value
 * pv_masked_attention gives it, up to the rounding of that merge.
 * Callers: a judge pass over a KV prefix that already exists ("Parallel partial verify" after
 * "Full verify", or the periodic premature verification of appendix "Full pipeline"). */
pv_status pv_segment_attention(const pv_sizes* sizes, const void* plan_dev, const void* q,
                               const void* k, const void* v, void* out, float* lse,
                               int32_t out_dtype, float softmax_scale, float rope_theta,
                               void* workspace, int64_t workspace_bytes, void* stream);

/* pv_masked_attention with K and V held as FP8: OCP E4M3 codes (1 sign, 4 exponent, 3 mantissa bits,
 * bias 7, no infinities) and one fp32 scale per kv head, K[t][h][:] = decode(code) * k_scale[h] and
 * likewise V -- the storage of the FP8 serving stack the paper's experiments run on (section
 * "Experiments", Setup: FP8 checkpoints of the target models).  The keys are what a KV cache holds,
 * i.e. rotated at their positions when they were written (pv_plan_export gives the positions): only
 * Q, bf16, is rotated by this call.  Both products run on the FP8 matrix instruction; for that Q is
 * rounded to E4M3 after rotation (per-row power-of-two scale) and the probabilities are rounded to
 * E4M3 (the row sum is taken over the rounded values), which is where the tolerance of this path
 * comes from.  Rows that see at most PV_SHORT_ROW_KEYS keys are evaluated in fp32.
 *   q               device bf16 [total_tokens][Hq][128]  (head_dim 128 only: PV_ERR_SHAPE otherwise)
 *   k_fp8, v_fp8    device uint8 [total_tokens][Hkv][128], 16-byte aligned, not modified
 *   k_scale_dev, v_scale_dev   device float [Hkv]
 *   out, lse, out_dtype, softmax_scale, rope_theta, workspace   as for pv_masked_attention
 *                   (sizes from pv_query_sizes with in_dtype PV_BF16) */
pv_status pv_masked_attention_fp8kv(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                    const void* k_fp8, const void* v_fp8, const float* k_scale_dev,
                                    const float* v_scale_dev, void* out, float* lse, int32_t out_dtype,
                                    float softmax_scale, float rope_theta, void* workspace,
                                    int64_t workspace_bytes, void* stream);

/* The two halves of pv_segment_attention as calls of their own, for a judge pass over keys that an
 * earlier pass already prepared (the serving engine keeps the prompt and draft keys between the
 * premature verification at T_p tokens and the later passes of appendix "Full pipeline"; Stage 2 of
 * "Design" calls the passes prefill-only and KV-cache-light), and for K/V that live in a paged cache.
 *
 * pv_prepare_kv writes, for the tokens [first_token, last_token) of the packed batch (counted in the
 * order [prompt | draft | segments] of every request), what the attention kernels read instead of
 * K and V: the rotary table, K rotated at the plan's positions and V, both re-laid-out per kv head.
 * Tokens outside the range keep what an earlier call prepared; blocks of 16 consecutive tokens of a
 * request are written whole (a range that starts inside a block re-prepares that block from K and
 * V).
 *   key_capacity     0, or a multiple of 64 >= sizes->padded_keys: the per-head stride of the
 *                    prepared keys, so that calls under different plans find each other's keys.
 *                    A draft that grew from T_p to T tokens with the same prompt (one request in
 *                    the batch: its rows do not move) keeps its first P + T_p prepared keys when
 *                    both passes use the capacity of the larger one and the second pass
 *                    prepares first_token = P + T_p onwards.  The workspace then needs
 *                    pv_prepared_workspace_bytes(sizes, key_capacity) bytes; 0 means the layout
 *                    and size of pv_segment_attention.
 *   k, v             device bf16; dense [total_tokens][Hkv][D] (block_table_dev NULL), or a pool of
 *                    pages [n_pages][page_size][Hkv][D] with block_table_dev: device int32
 *                    [ceil(total_tokens / page_size)], token row r of the packed batch (caller's
 *                    row order) living at row block_table[r / page_size] * page_size + r % page_size
 *   workspace        as for pv_segment_attention; it carries the prepared keys to the next call
 * pv_segment_attention_prepared is pv_segment_attention without the preparation: the segment rows
 * against the keys already in `workspace`.  k, v (and the block table) are read only for segment
 * rows that see at most PV_SHORT_ROW_KEYS keys.  With every token prepared by pv_prepare_kv under
 * the same plan and rope_theta the result is bit-identical to pv_segment_attention.
 * bf16 inputs only (PV_ERR_DTYPE otherwise). */
pv_status pv_prepare_kv(const pv_sizes* sizes, const void* plan_dev, const void* k, const void* v,
                        const int32_t* block_table_dev, int32_t page_size, int64_t first_token,
                        int64_t last_token, int64_t key_capacity, float rope_theta,
                        void* workspace, int64_t workspace_bytes, void* stream);
pv_status pv_segment_attention_prepared(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                        const void* k, const void* v,
                                        const int32_t* block_table_dev, int32_t page_size,
                                        int64_t key_capacity, void* out, float* lse,
                                        int32_t out_dtype, float softmax_scale, float rope_theta,
                                        void* workspace, int64_t workspace_bytes, void* stream);
/* Host only: workspace bytes of the two calls above for a per-head stride of key_capacity keys. */
pv_status pv_prepared_workspace_bytes(const pv_sizes* sizes, int64_t key_capacity, int64_t* bytes_out);

/* pv_masked_attention for callers that cannot allocate device memory or keep a workspace of their
 * own (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * workspace is a fixed array inside the library's device image, PV_STATIC_WORKSPACE_BYTES per GPU,
 * held from the first use on that GPU until the process ends.  No workspace arguments; everything
 * else as for pv_masked_attention, and the result is bit-identical to it.  The call allocates
 * nothing and frees nothing.
 *   Limit      the bytes this call needs (rotary table, rotated K, transposed V: about
 *              2 * Hkv * D * 2 + 4 * D bytes per token; pv_static_workspace_needed reports them;
 *              the partial results of pv_segment_attention are not part of it) must not exceed
 *              PV_STATIC_WORKSPACE_BYTES, else PV_ERR_WORKSPACE and nothing is launched.  The
 *              8B-like configuration of 3 072 tokens needs 14.2 MB.
 *   Sharing    every call on a GPU uses that GPU's one array: calls that may overlap on one GPU
 *              (different streams, different threads) race and must be serialised by the caller.
 *              Nothing in the array has to survive between calls or start at zero: each call
 *              rewrites every byte it later reads, padding included.
 *   First use  the first call on a device looks the array's address up once (a host-side query,
 *              no launch); make that call outside graph capture. */
enum { PV_STATIC_WORKSPACE_BYTES = 32 << 20 };
pv_status pv_masked_attention_static(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                     const void* k, const void* v, void* out, float* lse,
                                     int32_t out_dtype, float softmax_scale, float rope_theta,
                                     void* stream);
/* Host only: workspace bytes pv_masked_attention_static would use for `sizes`. */
pv_status pv_static_workspace_needed(const pv_sizes* sizes, int64_t* bytes_out);

/* Host only.  The logit margin at which the two-way confidence p_2w = e^{l_C} / (e^{l_C} + e^{l_I})
 * of appendix "Notation and judge calibration" equals tau: ln(tau / (1 - tau)), the form in which
 * every threshold of pv_first_reject and pv_policy is given.  0 < tau < 1, else PV_ERR_SHAPE. */
pv_status pv_margin_from_tau(double tau, double* margin_out);

/* Readout.  Verdict of segment k is Correct iff l_C >= l_I and l_C - l_I >= margin_threshold
 * (margin_threshold = ln(tau / (1 - tau)) makes this the two-way-confidence rule p_2w >= tau),
 * compared in fp64.  Per request writes int32 (first_reject, k_star, L_star, n_incorrect):
 *   first_reject  index of the first Incorrect segment, K_b if none
 *   mode 0        k_star = first_reject - 1 (largest Correct index with no Incorrect before it)
 *   mode 1        k_star = largest Correct index (t* = max{t_i : Correct} of the main text)
 *   L_star        boundary p_{k_star}, 0 if k_star = -1 (restart from scratch)
 *   logits_dev    device float [total_segments][2] = (l_C, l_I), segment order of the problem
 *   out_dev       device int32 [B][4] */
pv_status pv_first_reject(const pv_sizes* sizes, const void* plan_dev, const float* logits_dev,
                          double margin_threshold, int32_t mode, int32_t* out_dev, void* stream);

/* Judge logits.  For every segment k of every request, the hidden state at its judge row (the
 * last token of the segment, where the verifier's answer is read) times the two lm-head rows of
 * the Correct and Incorrect tokens (appendix "Notation and judge calibration": the verifier's
 * logits l_C, l_I at the judgment position).  bf16 inputs, fp32 accumulation.
 *   hidden_dev   device bf16 [total_tokens][hidden_size], 16-byte aligned, not modified
 *   w2_dev       device bf16 [2][hidden_size]: row 0 = Correct token, row 1 = Incorrect token
 *   hidden_size  multiple of 8, 8 .. 65536
 *   logits_dev   device float [total_segments][2] = (l_C, l_I): the input of pv_first_reject /
 *                pv_decide */
pv_status pv_judge_logits(const pv_sizes* sizes, const void* plan_dev, const void* hidden_dev,
                          const void* w2_dev, int32_t hidden_size, float* logits_dev,
                          void* stream);

/* Decision policy of the detailed algorithm (appendix "Full pipeline") once the judge logits are
 * known.  Every confidence threshold tau is given as the logit margin ln(tau / (1 - tau)), and a
 * confidence p_2w >= tau is tested as l_C - l_I >= margin in fp64 (see pv_first_reject). */
#define PV_MAX_SHORT_CHUNKS 8
typedef struct {
  double margin_chunk;          /* strict per-chunk threshold tau_P */
  double margin_chunk_relaxed;  /* relaxed per-chunk threshold tau_C^rx */
  double margin_full;           /* strict full-verify threshold tau_F */
  double margin_full_relaxed;   /* relaxed full-verify threshold tau_F^rx */
  double margin_short[PV_MAX_SHORT_CHUNKS]; /* short-draft threshold for K = 1 .. n_short chunks:
                                   min(tau_sd + 0.02 (K - 1), tau_F^rx) */
  double rho;                   /* the chunk run rejects when n_incorrect / K exceeds rho ... */
  double eta;                   /* rollback margin in chunks, >= 0 */
  int32_t kappa;                /* ... or the trailing run of Incorrect chunks reaches kappa (0: off) */
  int32_t n_short;              /* short-draft ceiling K^sd, 0 .. PV_MAX_SHORT_CHUNKS */
  int32_t relaxed_count_min;    /* premature exit: this many chunks below tau_C^rx abort (paper: 3) */
  int32_t premature;            /* 0: Stages 2-6;  1: premature-PV early exit (pass rho_p as rho) */
} pv_policy;

enum { PV_LABEL_SM = 0, PV_LABEL_SM_LG = 1, PV_LABEL_LG = 2 };

/* Per request writes 12 int32:
 *   [0] label         PV_LABEL_SM ship the draft, PV_LABEL_SM_LG continue from L*, PV_LABEL_LG
 *                     restart; premature mode without abort: -1 (keep drafting)
 *   [1] stage         stage that decided (2 strict accept, 3 short-draft accept, 5 relaxed accept,
 *                     6 hand-off); premature mode: 1 abort, 0 go on
 *   [2] L*            adopted prefix: boundary p_{m-1}, m = floor(max(0, k* + 1 - eta)); 0 if m = 0
 *   [3] k*            largest Correct chunk with no Incorrect before it, -1 if none
 *   [4] first_reject  [5] n_incorrect  [6] trailing run of Incorrect chunks
 *   [7] 1 if the rho / kappa rules reject the chunk run
 *   [8] chunks whose confidence is below tau_C^rx
 *   [9] full-answer verdict at tau_F (premature mode: -1)
 *   [10] index of the least confident chunk (first of equals; -1 if K = 0)   [11] K
 *   logits_dev       device float [total_segments][2]
 *   full_logits_dev  device float [B][2] (l_C^F, l_I^F) of the full-answer judge; NULL allowed in
 *                    premature mode only
 *   out_dev          device int32 [B][12], 16-byte aligned */
pv_status pv_decide(const pv_sizes* sizes, const void* plan_dev, const float* logits_dev,
                    const float* full_logits_dev, const pv_policy* policy, int32_t* out_dev,
                    void* stream);

/* Copies of the plan's per-token / per-segment arrays for inspection (device to device, on
 * `stream`): positions, a_end, b_start are int32 [total_tokens], one entry per row of the caller's
 * tensors; judge_row is int32 [total_segments] (row of the caller's tensors).  The row descriptor
 * (a_end, b_start) counts keys in the appended order of the request whatever the layout.  Any
 * output may be NULL. */
pv_status pv_plan_export(const pv_sizes* sizes, const void* plan_dev, int32_t* positions_dev,
                         int32_t* a_end_dev, int32_t* b_start_dev, int32_t* judge_row_dev,
                         void* stream);

/* Profiling aid for benchmarks (one thread at a time): when enabled, pv_masked_attention brackets
 * its main attention kernel with a pair of HIP events on the caller's stream, one pair per call out
 * of a ring of PV_PROFILE_RING pairs, without waiting for anything.  Enabling restarts the count.
 *   pv_profile_read      waits for the latest pair; the kernel's duration in milliseconds
 *                        (PV_ERR_SHAPE if nothing was recorded).
 *   pv_profile_read_all  waits for and returns the durations of the calls since enabling, oldest
 *                        first: the last min(calls, PV_PROFILE_RING, capacity) of them into
 *                        ms_host (host memory), their number into *n_out.
 * Disabling destroys the events (read the durations first); the three calls serialise on a lock. */
enum { PV_PROFILE_RING = 1024 };
pv_status pv_profile_enable(int32_t on);
pv_status pv_profile_read(float* main_kernel_ms);
pv_status pv_profile_read_all(float* ms_host, int32_t capacity, int32_t* n_out);

const char* pv_strerror(pv_status status);
int32_t pv_last_hip_error(void);
const char* pv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PV_H_ */
