/*
 * simple_sample.h -- C boundary of the decision-plane sampling epilogue for AMD MI355X (gfx950).
 *
 * One call turns a [B, V] logits matrix that is resident in device memory into B next-token
 * ids, entirely on the GPU:
 *
 *   (1) logits adjustment  Z' = ApplyPenalty(Z, Y_<s)                 (paper section 2.1 Eq. (1);
 *       repetition / frequency / presence penalties from each row's    penalty algorithm section 2.2;
 *       token history, touching only the penalised columns             column-wise penalties, 5.2)
 *   (2) p~ = softmax(Filter(Z' / tau; k, p_nuc, min_p))               (section 2.1 Eq. (2);
 *       the filter is applied before any normalisation                 truncation-first filtering, 5.2)
 *   (3) y ~ Categorical(p~), by inverse CDF with a counter-based       (section 2.1 (3); deterministic
 *       uniform keyed by (seed, row, step)                             random numbers, section 5.1)
 *   and, when a hot set H is given, speculative hot-vocab sampling:    (section 5.3, Eq. (6)-(9))
 *       accept a draw from the hot proposal with probability alpha_b, else draw from the tail
 *       proposal, which reproduces p~ exactly.
 *
 * Conventions the paper leaves open (they are the same ones the CPU oracle of this repository
 * states, so ids can be compared one to one):
 *   - repetition is sign-aware (z > 0 ? z / rep : z * rep); frequency subtracts freq * count and
 *     presence subtracts pres on tokens *generated* so far; repetition also sees prompt tokens;
 *   - temperature 0 selects greedy decoding: argmax of the penalised logits, lowest id on ties;
 *   - y = z' / tau is an IEEE float32 division; survivors are a prefix of the total order
 *     (y descending, token id ascending): top-k keeps exactly k, min-p keeps
 *     y >= fl32(y_max + fl32(ln min_p)), top-p keeps the shortest prefix of the top-k prefix whose
 *     mass reaches top_p times the top-k prefix mass; the shortest of the three wins, never empty;
 *   - one Philox4x32-10 block per (row, step): key = (seed lo, seed hi), counter =
 *     (r lo, step lo, step hi, r hi) with r = row_offset + row the 64-bit global row index;
 *     word w -> (x >> 8) * 2^-24; word 0 drives the draw,
 *     word 1 the SHVS acceptance test (accept iff u * S_K <= S_H), word 2 the SHVS tail draw;
 *   - every CDF walk (full, hot, tail) runs in ascending token id and returns the first id whose
 *     running mass exceeds u * total.
 *
 * All pointers named *_dev are DEVICE pointers owned by the caller; the library never frees or
 * retains them beyond the call.  logits are read-only and never modified.  All work is enqueued
 * on the given HIP stream and the calls return without synchronising.  Nothing is allocated on
 * the sampling path: the only allocation happens in simple_create.
 *
 * Errors: host-checkable argument errors return a negative code, enqueue nothing and leave
 * out_ids untouched.  Data errors that only the device can see (NaN or +inf logit, all -inf row,
 * negative temperature, non-positive repetition penalty, history longer than the context's
 * capacity) make that row's id -1 and set bits in its diagnostics record; a history id outside
 * [0, V) is ignored and flagged.
 *
 * Determinism: ids depend only on (logits, params, history, hot set, seed, step, global row
 * index), never on launch geometry or on how a batch is split into calls.
 *
 * Concurrency: a context owns device-side queues and workspace that every simple_sample call on
 * it uses, so the calls on one context must be ordered: issue them on one stream (or order the
 * streams with events), from one host thread at a time.  Different contexts are independent.
 */
#ifndef SIMPLE_SAMPLE_H
#define SIMPLE_SAMPLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct simple_ctx simple_ctx; /* opaque; owns the hot-set bitmap, the row queues and their workspace */

enum { SIMPLE_F32 = 0, SIMPLE_BF16 = 1 };

enum {
  SIMPLE_OK = 0,
  SIMPLE_EINVAL = -1,    /* bad argument */
  SIMPLE_ENOMEM = -2,    /* device allocation failed in simple_create */
  SIMPLE_EDEVICE = -3,   /* a HIP runtime call failed */
  SIMPLE_ECAPACITY = -4  /* sizes exceed what the context was created for, or the LDS of a CU */
};

/* One row's sampling controls (32 bytes, device memory, array of B). */
typedef struct {
  float temperature;  /* tau; 0 => greedy; must be >= 0 */
  int32_t top_k;      /* <= 0 or >= V => disabled */
  float top_p;        /* p_nuc; >= 1 => disabled; <= 0 keeps one token */
  float min_p;        /* <= 0 => disabled */
  float rep_penalty;  /* lambda_rep; 1 => disabled; must be > 0 */
  float freq_penalty; /* 0 => disabled */
  float pres_penalty; /* 0 => disabled */
  int32_t n_prompt;   /* the first n_prompt ids of the row's history are prompt tokens (repetition
                         only); the rest are generated tokens (all three penalties) */
} simple_row_params;

/* Optional per-row diagnostics (32 bytes, device memory, array of B). */
typedef struct {
  double alpha;        /* SHVS hot mass alpha_b = S_H / S_K (Eq. (7)); NaN without a hot set */
  double s_k;          /* mass of the top-k prefix relative to the row maximum; formed (and reported)
                          on rows with 0 < top_p < 1, whose nucleus target it scales; unspecified
                          on other rows, which never need it */
  float p_chosen;      /* p~ of the returned id */
  int32_t n_survivors; /* |K_b| */
  uint32_t flags;      /* SIMPLE_DIAG_* */
  uint32_t reserved;
} simple_row_diag;

enum {
  SIMPLE_DIAG_ERROR = 1u << 0,         /* id is -1 */
  SIMPLE_DIAG_GREEDY = 1u << 1,
  SIMPLE_DIAG_WIDE = 1u << 2,          /* K_b did not fit the on-chip candidate list (or is all of V): multi-pass route */
  SIMPLE_DIAG_SHVS = 1u << 3,          /* a hot set was used */
  SIMPLE_DIAG_ACCEPTED = 1u << 4,      /* SHVS hot candidate accepted */
  SIMPLE_DIAG_CAREFUL = 1u << 5,       /* candidate list overflowed: segment replayed in small pieces */
  SIMPLE_DIAG_REPLAY = 1u << 6,        /* sampled threshold missed: row streamed again with a rising one */
  SIMPLE_DIAG_GENERAL = 1u << 7,       /* row left by the single-pass kernel and completed by the general kernel */
  SIMPLE_DIAG_BAD_PARAM = 1u << 8,
  SIMPLE_DIAG_BAD_LOGIT = 1u << 9,     /* NaN or +inf logit, or every logit -inf */
  SIMPLE_DIAG_BAD_HISTORY_ID = 1u << 10, /* ignored */
  SIMPLE_DIAG_HISTORY_TOO_LONG = 1u << 11,
  SIMPLE_DIAG_BAD_HOT_SET = 1u << 12,  /* hot id outside [0, V) or duplicated (ignored) */
  SIMPLE_DIAG_PATTERN = 1u << 13       /* bfloat16 row without top-k and penalties, completed from counts per bit pattern */
};

/* Optional aggregate over the rows of the calls made while it is installed (64 bytes, device
 * memory; the "basic observability" of the paper's implementation section: acceptance rate and
 * sampler counts without reading one record per row).  The kernels add to it with atomics; the
 * caller zeroes it and reads it (stream-ordered copies).  Mean alpha = sum_alpha_q32 / 2^32 /
 * (shvs_accepted + shvs_rejected), a fixed-point sum, so its value does not depend on the order of
 * the additions. */
typedef struct {
  uint64_t rows;             /* rows completed */
  uint64_t greedy_rows;
  uint64_t shvs_accepted;    /* rows that used a hot set and accepted the hot draw */
  uint64_t shvs_rejected;    /* rows that used a hot set and drew from the tail */
  uint64_t second_pass_rows; /* rows whose survivors did not fit the on-chip candidate list (SIMPLE_DIAG_WIDE) */
  uint64_t general_rows;     /* rows completed by the general kernel (SIMPLE_DIAG_GENERAL) */
  uint64_t sum_alpha_q32;    /* sum over SHVS rows of alpha_b * 2^32, rounded to nearest */
  uint32_t error_flags;      /* OR of the SIMPLE_DIAG_* error bits of all rows */
  uint32_t reserved;
} simple_stats;

/*
 * Create a context on HIP device `device` for calls with up to max_B rows, at most max_V vocabulary
 * entries and at most max_nnz_per_row history ids per row (0 if no history will ever be passed).
 * Allocates, in one block of device memory, the hot-set membership bitmap (max_V bits), the row
 * queues and one workspace slot per row of a launch, for the rows whose survivors do not fit the
 * on-chip candidate list (min(max_B, 4096) slots of about 52 KB plus the size of one row's history
 * tables; a call with more rows than slots is still served, in several launches, so no row ever
 * lacks a slot).  Returns SIMPLE_ECAPACITY if one row's on-chip state (history bitmap, counts,
 * candidate list) cannot fit the LDS of one compute unit.  Host pointers: out.
 */
int simple_create(simple_ctx** out, int device, int64_t max_B, int64_t max_V, int64_t max_nnz_per_row);

/* Free the context (synchronises the device it lives on).  NULL is accepted. */
void simple_destroy(simple_ctx* ctx);

/*
 * Install a hot set H (section 5.3) for later calls that pass H = -1: builds the V-bit membership
 * bitmap on `stream`.  hot_ids_dev: H distinct ids in [0, V), any order (device).  Out-of-range or
 * duplicate ids are ignored and reported through SIMPLE_DIAG_BAD_HOT_SET on later rows.
 */
int simple_set_hot_set(simple_ctx* ctx, const int32_t* hot_ids_dev, int32_t H, int64_t V, void* hip_stream);

/*
 * Install (or, with NULL, remove) the aggregate that later simple_sample calls on this context add
 * to.  stats_dev: device memory, 8-byte aligned, owned and zeroed by the caller, alive until it is
 * removed or the context destroyed.  Host-side only: nothing is enqueued.  Returns SIMPLE_EINVAL
 * for a NULL context or a misaligned pointer.
 */
int simple_set_stats(simple_ctx* ctx, simple_stats* stats_dev);

/*
 * The rest of the decisions record the paper's samplers return beside the token ids (section 4.2,
 * step 6: "next-token ids, EOS flags, optional log-probs").  Install (or, with NULLs, remove)
 * per-row outputs that later sampling calls on this context fill, row b of a call at index b:
 *   logprobs_dev   [max rows of a call] float: natural log of p~ of the returned id (0 for a greedy
 *                  row, -inf for a row whose id is -1)
 *   eos_dev        [max rows of a call] uint8: 1 if the returned id is one of the end-of-sequence ids
 * eos_ids_host: n_eos (0..8) token ids, host memory, copied.  Either output pointer may be NULL.
 * Host-side only: nothing is enqueued.  SIMPLE_EINVAL for a NULL context, n_eos outside [0, 8] or
 * n_eos > 0 without eos_ids_host.
 */
int simple_set_decision_outputs(simple_ctx* ctx, float* logprobs_dev, uint8_t* eos_dev, const int32_t* eos_ids_host, int n_eos);

/*
 * The sampling call (section 2.1 steps (1)-(3); section 5.3 when a hot set is in force).
 *
 *  logits_dev        [B, row_stride_elems] row-major, dtype SIMPLE_F32 (float) or SIMPLE_BF16
 *                    (bfloat16 bit patterns, uint16); only the first V columns of a row are read
 *  params_dev        [B] simple_row_params
 *  hist_ptr_dev      [B+1] CSR offsets into hist_ids_dev, or NULL for "no history"
 *  hist_ids_dev      token ids of every row's history (prompt first), or NULL with hist_ptr_dev
 *  hot_ids_dev, H    hot set for this call: (ptr, H > 0) builds the bitmap on the stream first;
 *                    (NULL, 0) disables SHVS; (NULL, -1) uses the set installed by
 *                    simple_set_hot_set for this V
 *  seed, step        key and counter words of the random numbers; row b uses global row index
 *                    row_offset + b, so a batch may be split into calls without changing ids
 *  out_ids_dev       [B] int32 token ids (-1 for a row with a data error)
 *  diag_dev          [B] simple_row_diag, or NULL
 *  hip_stream        hipStream_t (NULL = the default stream)
 *
 * Which kernel completes a row depends on its controls and on the call (dtype, alignment, V); the
 * id does not, beyond the rounding of masses near a decision boundary, and is the same for the
 * same call repeated.  Rows of a bfloat16 call without top-k and without a penalty in force are
 * sampled from counts per bit pattern (SIMPLE_DIAG_PATTERN in the row's record).
 *
 * B = 0 is a no-op that returns SIMPLE_OK.  Returns SIMPLE_EINVAL for NULL required pointers,
 * B < 0, V <= 0, row_stride_elems < V, an unknown dtype, H < -1, H > V, H = -1 without an
 * installed set of that V, or hist_ptr_dev given without hist_ids_dev; SIMPLE_ECAPACITY for
 * V > max_V or history given to a context created with max_nnz_per_row = 0.
 */
int simple_sample(simple_ctx* ctx, const void* logits_dev, int64_t B, int64_t V, int dtype,
                  int64_t row_stride_elems, const simple_row_params* params_dev,
                  const int64_t* hist_ptr_dev, const int32_t* hist_ids_dev,
                  const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step,
                  uint64_t row_offset, int32_t* out_ids_dev, simple_row_diag* diag_dev,
                  void* hip_stream);

/*
 * Speculative hot-vocab sampling that reads only the hot columns when the hot draw is accepted
 * (section 5.3; the cost model of section 5.4: H columns on acceptance, the other V - H on
 * rejection).  The vocabulary must be laid out hot-first: the hot set is the columns [0, H) (an
 * LM head whose rows are permuted offline).  alpha_b needs the mass of the tail, so each row
 * comes with two numbers from the kernel that wrote the logits (section 5.3: the weights "can be
 * pre-computed on GPUs when writing logits"):
 *   tail_max   max over v >= H of logits[b, v]                          (-inf if H == V)
 *   tail_sum   sum over v >= H of exp((logits[b, v] - tail_max) / temperature_b)   (0 if H == V)
 * Rows served from the hot columns: temperature > 0, no top-k / top-p / min-p, no penalties (their
 * survivor set is all of V, so Eq. (7) needs nothing of the tail but its mass); a rejected row
 * streams its tail for the tail proposal.  Every other row (truncated, greedy, invalid) is served
 * by the general kernel with [0, H) as the hot set, so all rows get the ids of SHVS as defined for
 * simple_sample with hot_ids = 0 .. H-1 (same uniforms, same walk order).  No history arguments:
 * penalised rows belong to simple_sample.  H must be a positive multiple of 1024 (float32) or
 * 2048 (bfloat16) columns, at most V; rows and logits_dev 16-byte aligned; V - H and H at most
 * 2^20 (float32) or 2^21 (bfloat16).  Otherwise as simple_sample (stream semantics, errors, diag,
 * statistics and decision outputs).  A NaN or +inf tail_max, or a negative / NaN tail_sum, is a
 * data error of the row (id -1).
 */
typedef struct {
  double tail_sum;
  float tail_max;
  float reserved;
} simple_tail_stats;
int simple_sample_hot_first(simple_ctx* ctx, const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                            const simple_row_params* params_dev, int32_t H, const simple_tail_stats* tail_stats_dev,
                            uint64_t seed, uint64_t step, uint64_t row_offset, int32_t* out_ids_dev,
                            simple_row_diag* diag_dev, void* hip_stream);

/*
 * Logit bias and allow-lists (section 5.2 names allow-lists among the constraints that compose on the
 * survivor set; the implementation section mentions optional biases), as a pass ahead of the
 * sampling call: out[b, v] = fl32(z[b, v] + bias(b, v)) for the columns row b allows, -inf for the
 * others, written as float32 to out_dev ([B, out_stride_elems], device, owned by the caller), which
 * the caller then hands to simple_sample with dtype SIMPLE_F32.  Constraints come before the
 * penalties and are independent of the order of the survivors.
 *   bias_ptr_dev / bias_ids_dev / bias_vals_dev   CSR over rows ([B + 1] offsets, ids, float32
 *       values), or all NULL.  Entries of a row that name the same column add up in list order.
 *   allow_ptr_dev / allow_ids_dev                 CSR over rows, or both NULL.  A row with entries keeps
 *       only the listed columns (a bias on a column it masks leaves it masked); a row with none
 *       has no allow-list.
 * Ids outside [0, V) are ignored.  out_dev may be logits_dev itself when dtype is SIMPLE_F32 and the
 * strides are equal.  A call without constraints never needs this pass; one with them pays one more
 * read and one write of its logits.  No context, nothing allocated; enqueued on hip_stream.
 * SIMPLE_EINVAL for NULL / negative / inconsistent arguments (offsets without their arrays, strides
 * below V, unknown dtype), SIMPLE_ECAPACITY if an allow-list's V-bit mask exceeds 96 KB of LDS.
 */
int simple_apply_logit_constraints(const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                                   const int64_t* bias_ptr_dev, const int32_t* bias_ids_dev, const float* bias_vals_dev,
                                   const int64_t* allow_ptr_dev, const int32_t* allow_ids_dev,
                                   float* out_dev, int64_t out_stride_elems, void* hip_stream);

/*
 * Incremental penalty state (paper section 5.2: row-append token buffer; the histograms are carried
 * from step to step, C_o^{s+1} = C_o^s + Hist(Y_s), M_o = (C_o > 0), C_p and M_p fixed per sequence,
 * instead of being rebuilt from the token list on every call).
 *
 * A state has max_seqs sequence slots for vocabulary size V; a slot holds up to L_max tokens (prompt
 * plus generated) in device memory, together with the presence mask, rank directory and generated-
 * token counts that the sampling kernel otherwise builds on chip from the CSR history.
 *   simple_state_restart   evicts what n slots held and installs their prompts: slot slots_dev[i]
 *                          (or i, with slots_dev NULL) gets prompt_ids_dev[prompt_ptr_dev[i] ..
 *                          prompt_ptr_dev[i + 1]) (prompt_ptr_dev NULL: empty prompts).  Prompt
 *                          tokens count towards the repetition penalty only.  With n_prompt_dev
 *                          (n values, else NULL) only the first n_prompt_dev[i] ids of list i are
 *                          the prompt and the rest are tokens the sequence has already generated
 *                          (a sequence that moves in from another sampler, or a bulk load).
 *   simple_state_append    one step: new_ids_dev[b] (device, B ids; negative = none) is appended to
 *                          slot slots_dev[b] (or b) as a generated token.  Cost per sequence: one
 *                          counter, or for an id not seen before O(V / 64 + distinct ids).
 *   simple_sample_state    simple_sample with the rows' histories taken from the state: row b uses
 *                          slot slots_dev[b] (or b); params[b].n_prompt is ignored (the state knows
 *                          each sequence's prompt length).  Ids equal those of simple_sample called
 *                          with the same token lists as CSR history.
 * All three enqueue on hip_stream and return without synchronising; calls that touch the same state
 * must be ordered by the caller (one stream, or events).  No two rows of one call may name the same
 * slot.  A slot index outside [0, max_seqs) is skipped by restart / append and makes the row's id -1
 * (SIMPLE_DIAG_HISTORY_TOO_LONG) in simple_sample_state, as does a sequence longer than L_max or
 * than the context's max_nnz_per_row.  A token id outside [0, V) is kept in the list, ignored by the
 * penalties and reported as SIMPLE_DIAG_BAD_HISTORY_ID on the sequence's later rows.
 * Errors: SIMPLE_EINVAL for NULL / negative / inconsistent arguments (a state of another V or
 * device than the call's, B > max_seqs without slots_dev), SIMPLE_ECAPACITY for L_max > 65535, a
 * slot whose tables exceed the LDS of a compute unit, or L_max above the context's
 * max_nnz_per_row; SIMPLE_ENOMEM / SIMPLE_EDEVICE as for simple_create.
 */
typedef struct simple_state simple_state;
int simple_state_create(simple_state** out, int device, int64_t max_seqs, int64_t V, int64_t L_max);
void simple_state_destroy(simple_state* state);
int simple_state_restart(simple_state* state, const int32_t* slots_dev, int64_t n, const int64_t* prompt_ptr_dev,
                         const int32_t* prompt_ids_dev, const int32_t* n_prompt_dev, void* hip_stream);
int simple_state_append(simple_state* state, const int32_t* slots_dev, const int32_t* new_ids_dev, int64_t B, void* hip_stream);
int simple_sample_state(simple_ctx* ctx, const simple_state* state, const int32_t* slots_dev, const void* logits_dev, int64_t B, int64_t V,
                        int dtype, int64_t row_stride_elems, const simple_row_params* params_dev,
                        const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step, uint64_t row_offset,
                        int32_t* out_ids_dev, simple_row_diag* diag_dev, void* hip_stream);

/*
 * simple_sample for callers that cannot allocate device memory or create a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * simple_sample, on the current HIP device, without a context: the row queues, the workspace slots
 * and the hot-set bitmap live in a static device array of simple_static_limit(3) bytes (8 MiB) that
 * each GPU the library runs on holds until the process ends.  Limits: V <= simple_static_limit(0)
 * (2^18 - 1), at most simple_static_limit(1) (8192) history ids per row (a longer row gets id -1 and
 * SIMPLE_DIAG_HISTORY_TOO_LONG), simple_static_limit(2) (64) rows per launch (a larger batch is
 * served in several launches).  A hot set is passed with the call (hot_ids_dev, H > 0; H = -1 is
 * SIMPLE_EINVAL) and its bitmap is rebuilt on the stream every time.  Returns SIMPLE_ECAPACITY for a
 * larger V, else what simple_sample returns.  Calls no hipMalloc / hipFree or other allocating
 * routine; the first call on a device looks up the array's address and the device's attributes.
 * All calls on one GPU share the array: calls that overlap on one GPU (two streams, two host
 * threads) race; issue them on one stream or order them with events.
 */
int simple_sample_static(const void* logits_dev, int64_t B, int64_t V, int dtype,
                         int64_t row_stride_elems, const simple_row_params* params_dev,
                         const int64_t* hist_ptr_dev, const int32_t* hist_ids_dev,
                         const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step,
                         uint64_t row_offset, int32_t* out_ids_dev, simple_row_diag* diag_dev,
                         void* hip_stream);
/* Limits of simple_sample_static: what = 0 max V, 1 max history ids per row, 2 rows per launch,
 * 3 bytes of the static array; SIMPLE_EINVAL otherwise. */
int64_t simple_static_limit(int what);

/*
 * Timing aid for benchmarks (not part of the method): while enabled, every simple_sample call
 * brackets the launch of its dominant kernel (the single-pass row kernel when the call can use
 * it, else the general row kernel) with two HIP events on the call's stream.
 * simple_profile_enable(ctx, 1) creates the events (up to 1024 launches are kept, later ones are
 * not recorded) and resets the record; simple_profile_enable(ctx, 0) destroys them.
 * simple_profile_read synchronises with the recorded events and returns the number of recorded
 * launches; *total_ms_host (host pointer) receives the sum of their durations in milliseconds.
 * simple_profile_read_launches does the same and also writes the duration of each of the first
 * min(cap, recorded) launches, in launch order, to ms_host[] (host pointer, cap floats; may be
 * NULL with cap = 0).  Both return a negative error code on failure.
 */
int simple_profile_enable(simple_ctx* ctx, int on);
int simple_profile_read(simple_ctx* ctx, double* total_ms_host);
int simple_profile_read_launches(simple_ctx* ctx, float* ms_host, int cap, double* total_ms_host);

/*
 * Bandwidth yardstick for benchmarks (not part of the method): a read-only streaming reduction
 * over the same kind of buffer simple_sample reads.  row_max_dev[b] (device, B floats, written)
 * receives the maximum of the first V columns of row b, NaNs ignored, -inf for none; one
 * workgroup per row with the sampling kernel's load pattern and none of its arithmetic, so its
 * rate is the ceiling a one-pass row kernel can reach on the device.  Enqueued on hip_stream on
 * the current device; no context is needed and nothing is allocated.  logits_dev and every row
 * must be 16-byte aligned (SIMPLE_EINVAL otherwise, as for NULL pointers, B < 0, V <= 0,
 * row_stride_elems < V or an unknown dtype); B = 0 is a no-op.
 */
int simple_stream_probe(const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                        float* row_max_dev, void* hip_stream);

/* Bytes of LDS one row's workgroup uses for the given context (for occupancy reasoning). */
int64_t simple_lds_bytes(const simple_ctx* ctx);

/* Static description of an error code. */
const char* simple_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int simple_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SIMPLE_SAMPLE_H */
