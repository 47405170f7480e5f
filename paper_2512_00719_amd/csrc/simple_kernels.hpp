// Host-visible launch interface of the sampling kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_sample.h"

namespace simple {

// Byte offsets of one row's LDS regions in the general kernel's workgroup.
struct LdsLayout {
  uint32_t bitmap;  // history presence mask, V bits rounded up to groups of 8 words
  uint32_t grp;     // rank directory, one word per group
  uint32_t counts;  // 16-bit generated-token counts by rank
  uint32_t cand;    // candidate list: CAP keys then CAP ids (32 KB); reused by the multi-pass route
  uint32_t hist;    // radix histogram / staging (8 KB)
  uint32_t total;
};

// LDS of the single-pass kernel's workgroup.  One region is shared in time: it holds the history
// tables while the threshold is sampled and again in the epilogue, and the candidate list (later the
// epilogue's tables) in between.
struct FastLayout {
  uint32_t bitmap;    // history presence mask, one bit per column (region offset 0)
  uint32_t dir;       // 16-bit count of set bits before each pair of mask words
  uint32_t cnt;       // 16-bit generated-token counts, indexed by the rank of the id among the set bits
  uint32_t claim;     // one bit per rank: set by the thread that corrects that column's mass (long histories)
  uint32_t list_cap;  // entries of the candidate list (value word + id word each) the region holds
  uint32_t long_cap;  // entries of a long certified list that fit beside its bucket tables
  uint32_t samp;      // threshold sample merge area
  uint32_t total;     // 0: the call cannot use the kernel
  int threads;        // workgroup size the layout was made for (256, 512 or 1024)
};

constexpr int SAMPLE_PER_WAVE = 48;   // keys of the threshold sample a wave hands to the merge (sizes the merge area)
constexpr int CAPF_PER_THREAD = 12;  // candidate-list entries per thread the single-pass kernel's epilogue holds in registers
constexpr int KMAXF = 1024;   // largest top-k its list certifies
constexpr int32_t PENDING = -2;  // id left by the single-pass kernel on rows the general kernel completes
constexpr int32_t NOT_TAKEN = -3;  // id left by the pattern-count kernel on every row that the single-pass kernel still has to do
constexpr int PEND_ROWS = 65536; // rows per launch (capacity of the pending-row queue)
constexpr int WIDE_SLOTS = 4096; // workspace slots of the whole-vocabulary-nucleus kernels; a launch takes no more rows than this,
                                 // so every row of it can be queued for them
constexpr uint32_t WIDE_SLOT_FIXED = 53312;  // workspace per such row, before its history tables

// Incremental penalty state (paper section 5.2), one record per sequence slot.
struct StateRec {
  int32_t len;       // tokens of the sequence so far (prompt, then generated); above the capacity: too long
  int32_t n_prompt;  // the first n_prompt of them are the prompt
  int32_t distinct;  // distinct ids among them (set bits of the presence mask)
  uint32_t flags;    // SIMPLE_DIAG_BAD_HISTORY_ID if an id outside [0, V) was met (it is ignored)
};

struct SampleArgs {
  const void* logits;
  int64_t stride;  // elements between rows
  int V, B;
  const simple_row_params* params;
  const int64_t* hist_ptr;
  const int32_t* hist_ids;
  const uint32_t* hot_bits;   // V-bit hot-set mask or nullptr
  const uint32_t* hot_flags;  // bit 0: id out of range, bit 1: duplicate
  uint64_t seed, step, row_offset;
  int32_t* out;
  simple_row_diag* diag;
  simple_stats* stats;  // aggregate over rows, or nullptr
  float* logprobs;      // ln p~ of the returned id per row, or nullptr
  uint8_t* eos_out;     // 1 where the returned id is an end-of-sequence id, or nullptr
  int32_t eos_ids[8];
  int n_eos;
  // With an incremental penalty state (st_rec != nullptr) a row's history is its sequence slot's:
  // the token list in st_tokens and, ready-made, the tables the single-pass kernel otherwise builds
  // in LDS from that list (presence mask, rank directory, counts by rank, at the same offsets).
  const StateRec* st_rec;
  const int32_t* st_tokens;         // st_lmax ids per slot
  const unsigned char* st_tables;   // st_stride bytes per slot
  const int32_t* st_slots;          // slot of each row of the launch, or nullptr: row b uses slot st_slot0 + b
  int st_lmax, st_nslots, st_slot0;
  uint32_t st_stride;
  int max_nnz;
  int gated;       // 1: the single-pass kernel runs first and queues the rows it leaves
  int pattern_on;  // the pattern-count kernel (bfloat16 rows without penalties and without a short top-k) ran first: 1 before the
                   // single-pass kernel, 2 before the hot-first kernel (it then leaves that kernel's own rows alone)
  // Queues filled by the single-pass kernel.  Word [parity] counts the entries of this launch; the
  // single-pass kernel clears word [parity ^ 1], which the previous launch on the stream used.
  uint32_t* pend;  // rows left to the general kernel: [0], [1] counts, [2 ..] row indices
  int32_t* order;  // row of each workgroup of the single-pass kernel (written by the ordering kernel of a launch with more rows
                   // than compute units), or nullptr: workgroup b takes row b
  uint32_t* wq;    // rows with a whole-vocabulary nucleus wider than the list: [0], [1] counts, records from word 16
  unsigned char* wws;  // one workspace slot per queued row
  int wide_slots;
  uint32_t ws_stride;  // bytes per slot: fixed part, then the row's history tables
  int parity;
  int n_cu;        // compute units of the device (sizes the grids of the sliced kernels)
  LdsLayout L;
  FastLayout F;
};

// The decision outputs of one completed row (called by one thread): log-probability and EOS flag.
__device__ __forceinline__ void write_decision(const SampleArgs& a, int row, int id, float p, bool greedy) {
  if (a.logprobs) a.logprobs[row] = id < 0 ? -INFINITY : (greedy ? 0.0f : logf(p));
  if (a.eos_out) {
    bool e = false;
    for (int i = 0; i < a.n_eos; ++i) e = e || (id == a.eos_ids[i]);
    a.eos_out[row] = (id >= 0 && e) ? 1 : 0;
  }
}

// Where a row's token history comes from: the CSR arrays of the call, or its slot of the state.
struct RowHist { const int32_t* ids; int nnz, n_prompt, slot; uint32_t flags; };
__device__ __forceinline__ RowHist row_history_csr(const SampleArgs& a, int row, int par_n_prompt) {
  RowHist h;
  h.ids = nullptr; h.nnz = 0; h.n_prompt = par_n_prompt; h.slot = -1; h.flags = 0u;
  if (a.hist_ptr) {
    const long long h0 = a.hist_ptr[row], h1 = a.hist_ptr[row + 1];
    long long n = h1 - h0;
    if (n < 0) n = 0;
    if (n > (long long)a.max_nnz + 1) n = (long long)a.max_nnz + 1;
    h.nnz = (int)n;
    h.ids = a.hist_ids + h0;
  }
  return h;
}
__device__ __forceinline__ RowHist row_history_state(const SampleArgs& a, int row, int par_n_prompt) {
  RowHist h;
  h.ids = nullptr; h.nnz = 0; h.n_prompt = par_n_prompt; h.slot = -1; h.flags = 0u;
  const int slot = a.st_slots ? a.st_slots[row] : a.st_slot0 + row;
  if ((unsigned)slot >= (unsigned)a.st_nslots) { h.nnz = a.max_nnz + 1; return h; }  // reported as a history that is too long
  const StateRec rec = a.st_rec[slot];
  h.slot = slot;
  h.ids = a.st_tokens + (size_t)slot * (size_t)a.st_lmax;
  h.nnz = (rec.len > a.st_lmax || rec.len > a.max_nnz) ? a.max_nnz + 1 : max(rec.len, 0);
  h.n_prompt = rec.n_prompt;
  h.flags = rec.flags;
  return h;
}
__device__ __forceinline__ RowHist row_history(const SampleArgs& a, int row, int par_n_prompt) {
  return a.st_rec ? row_history_state(a, row, par_n_prompt) : row_history_csr(a, row, par_n_prompt);
}

// Rows of the pattern-count route (bfloat16 calls only): survivors are a long prefix of the vocabulary
// (top-p, min-p or no truncation without top-k, or a top-k above what the single-pass kernel's list
// certifies), no penalty is in force, and the parameters are valid.
__device__ __forceinline__ bool pattern_route(const simple_row_params& par, int V, int nnz, int max_nnz) {
  const bool pen_on = par.rep_penalty != 1.0f || par.freq_penalty != 0.0f || par.pres_penalty != 0.0f;
  const bool small_k = par.top_k >= 1 && par.top_k < V && par.top_k <= KMAXF;
  return par.temperature > 0.0f && par.temperature < INFINITY && par.rep_penalty > 0.0f && !small_k && par.top_p > 0.0f &&
         !(nnz > 0 && pen_on) && nnz <= max_nnz;
}

// Rows that the hot-first kernel decides from the hot columns and the caller's tail statistics alone:
// temperature sampling without truncation and without penalties.
__device__ __forceinline__ bool hot_first_plain(const simple_row_params& par, int V) {
  return par.temperature > 0.0f && !(par.top_k >= 1 && par.top_k < V) && !(par.top_p < 1.0f) && !(par.min_p > 0.0f) &&
         par.rep_penalty == 1.0f && par.freq_penalty == 0.0f && par.pres_penalty == 0.0f;
}

// Rows whose work in the single-pass kernel goes on longest after the stream: those that sum the whole row
// (a nucleus without top-k) and top-k rows with long lists.
__device__ __forceinline__ bool long_epilogue(const simple_row_params& par, int V) {
  const bool greedy = par.temperature == 0.0f;
  const bool k_on = par.top_k >= 1 && par.top_k < V;
  const bool need_sum = !greedy && !k_on && par.top_p < 1.0f && !(par.top_p <= 0.0f);
  return need_sum || (k_on && par.top_k > 512);
}

LdsLayout make_layout(int64_t V, int64_t max_nnz, bool with_history);
// Layout of the single-pass kernel; total = 0 when the call cannot use it.
FastLayout make_fast_layout(int64_t V, int dtype, int64_t max_nnz, bool with_history, bool vec, int lds_limit,
                            int64_t B, int n_cu);
hipError_t launch_sample(const SampleArgs& a, int dtype, bool vec, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_fast(const SampleArgs& a, int dtype, hipStream_t st);
hipError_t launch_order(const SampleArgs& a, hipStream_t st);  // fills a.order; before launch_fast
hipError_t launch_pattern(const SampleArgs& a, hipStream_t st);  // before launch_fast, when a.pattern_on
hipError_t launch_wide(const SampleArgs& a, int dtype, hipStream_t st);  // after launch_fast, before the general kernel
hipError_t set_max_lds(unsigned bytes);
hipError_t set_max_lds_fast(unsigned bytes);
hipError_t launch_state_reset(StateRec* rec, int32_t* tokens, unsigned char* tables, int n_slots, int lmax, int V, uint32_t stride,
                              uint32_t off_dir, uint32_t off_cnt, const int32_t* slots, int n, const int64_t* prompt_ptr,
                              const int32_t* prompt_ids, const int32_t* n_prompt, hipStream_t st);
hipError_t launch_state_append(StateRec* rec, int32_t* tokens, unsigned char* tables, int n_slots, int lmax, int V, uint32_t stride,
                               uint32_t off_dir, uint32_t off_cnt, const int32_t* slots, const int32_t* new_ids, int B, hipStream_t st);
hipError_t set_max_lds_state(unsigned bytes);
hipError_t launch_pending_rows(const SampleArgs& a, int dtype, bool vec, hipStream_t st);  // the general kernel on the queued rows
hipError_t launch_hot_range(uint32_t* bits, uint32_t* flags, int V, int H, hipStream_t st);  // hot set [0, H) as a mask
hipError_t launch_hot_first(const SampleArgs& a, int dtype, int H, const simple_tail_stats* tail, hipStream_t st);
int hot_first_tile(int dtype);   // columns per tile of the hot-first kernel: H must be a multiple
int hot_first_max_tiles();       // tiles of hot set or tail it can index
hipError_t launch_hot_build(const int32_t* ids, int H, int V, uint32_t* bits, uint32_t* flags, hipStream_t st);

}  // namespace simple
