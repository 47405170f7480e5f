// Rows whose survivors are not a short prefix that the single-pass kernel's candidate list can hold:
// a nucleus over the whole vocabulary that is wider than the list (top-p over all of V, section 2.1
// Eq. (2)), no truncation at all (every column survives), a min-p cut below the list's reach, or
// top-k alone with k above what the list certifies.
//
// The single-pass kernel queues such rows with their threshold g.  Their remaining work is two more
// reads of the row, which one workgroup per row would do at the latency of a single compute unit;
// here every queued row is cut into slices of 4096 columns that spread over the whole chip:
//
//   bins      per slice, the penalised, tempered logits below g are binned (bins linear in the
//             tempered logit, 1/64 of a factor two in probability wide) with their masses relative
//             to the mass at g (integers, LDS atomics); the mass at or above g goes to one more
//             slot.  The bins are exact sums, so they also give the mass of the whole row, and they
//             point at the bin that holds the cut.
//   classify  that bin follows from the cumulated masses.  Tempered value, bin and the comparison
//             with g are monotone in the logit, so the class of a column (surely inside, in the
//             cut's bin, outside) is decided by two thresholds on the logit itself, found once per
//             row by a search over floats.  Per tile, the exact (integer) masses of the columns
//             surely inside are summed by class (tail / hot) and the columns of the cut's bin are
//             collected.
//   finish    one workgroup per row checks that the cut does lie in the collected bin (else the
//             general kernel takes the row), finds it exactly among those columns by a radix
//             descent over (value, id) weighted by mass, however many of them tie (total order:
//             value descending, id ascending), applies the SHVS acceptance test (section 5.3), walks
//             the per-tile masses of the drawn class in ascending id and reads one tile a last time
//             to locate the drawn id (inverse CDF, step (3) of section 2.1).
//
// The first two kernels are software pipelines over a workgroup's slices: the loads of the next
// slice (logits, hot-set bits, history mask) are requested before the current one is processed, and
// a slice's own dependent loads (history counts, logits of its history columns) are requested
// before its main line runs, so that no trip through memory is waited for in full.  Loads return in
// order: what is needed first is requested first.
//
// Rows without truncation skip the first kernel and have no cut; rows with a min-p cut use the first
// kernel for the row maximum only (the cut is a value).  Rows with top-k alone run the same three
// kernels by count instead of mass: a bin also counts its columns, the cut's bin is the one in which
// the count from the top reaches k, and the descent inside it weighs every column as one.
//
// Penalties (section 2.2) are applied on the fly: the single-pass kernel leaves the row's history
// tables (presence mask, rank directory, counts by rank) in the row's workspace slot, and a slice
// loads its part of them into LDS.  All masses are
// integers, so no result depends on the order of the additions.  A row for which a table overflows
// or the passes disagree is handed to the general kernel.
#include <type_traits>

#include "simple_rowdev.hpp"

namespace simple {
namespace fast {


constexpr int WT = 256;      // threads per workgroup
constexpr int WNW = WT / 64;
constexpr int SLC = 4096;    // columns per slice
constexpr int ICAP = 1024;   // columns of the boundary bin one slice can always stage
constexpr int LCAP = 2048;   // size of the stage: written out once fewer than ICAP places are free
static_assert(WS_HT == WIDE_SLOT_FIXED, "workspace slot size");
static_assert(sizeof(WideRec) == 64, "queue record size");

// Per-row constants of a queued row, identical in every thread.
struct WideRow {
  int row;
  StreamCtx C;
  float tau, top_p, min_p;
  uint32_t mode, flags;
  bool h_active;
  float rep, freq, pres;
  double inv_rep;
  uint32_t distinct;
  int top_k;
  unsigned char* ws;
};

// The record is the same in every lane; saying so keeps the row's constants in scalar registers.
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uni(float v) { return __uint_as_float(uni(__float_as_uint(v))); }
__device__ __forceinline__ double uni(double v) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  return __longlong_as_double((long long)(((unsigned long long)uni((uint32_t)(b >> 32)) << 32) | (unsigned long long)uni((uint32_t)b)));
}

__device__ __forceinline__ WideRow load_row(const SampleArgs& a, unsigned slot) {
  WideRow W;
  slot = uni(slot);
  const WideRec rec = reinterpret_cast<const WideRec*>(a.wq + WQ_HEAD)[slot];
  W.row = uni((int)rec.row); W.mode = uni(rec.mode); W.flags = uni(rec.flags);
  W.tau = uni(rec.tau); W.top_p = uni(rec.top_p); W.min_p = uni(rec.min_p);
  W.C.g = uni(rec.g); W.C.y_g = uni(rec.g / rec.tau); W.C.inv_tau = uni(1.0 / (double)rec.tau); W.C.need_sum = true;
  W.C.l2e_tau = 0.0f;
  W.rep = uni(rec.rep); W.freq = uni(rec.freq); W.pres = uni(rec.pres);
  W.inv_rep = uni(1.0 / (double)rec.rep);
  W.h_active = uni(rec.h_active) != 0;
  W.distinct = uni(rec.distinct);
  W.top_k = uni(rec.top_k);
  W.ws = a.wws + (size_t)slot * a.ws_stride;
  return W;
}

// threadIdx.x as a value the compiler cannot trace: what is derived from it below (table indices, LDS
// addresses) is then formed where it is used instead of being kept across the kernels' item loops,
// where a register too many is spilled and its reload waits behind every load in flight.
__device__ __forceinline__ int fresh_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// A slice's part of the row's history tables, in LDS: the mask words of its columns, the
// rank at the start of each of its word pairs (and of the next slice), and the counts of its
// columns, indexed by rank minus the slice's first rank.
constexpr int HCAP = 512;  // history columns of a slice that are spread over all threads; more stay with their mask word's thread
struct SliceTabs {
  uint32_t bm[SLC / 32];
  uint32_t dir[SLC / 64 + 2];
  uint16_t cnt[SLC];
  float hz[HCAP];       // logit of the history column of rank j in the slice, as read
  uint16_t hcol[HCAP];  // its column, counted from the slice's first
};
static_assert(WT == 256, "the finishing kernel maps one tile of each class to a thread");
static_assert(SLC / 32 + SLC / 64 + 1 <= WT, "one mask word or directory entry per thread");
// The tables of the slice that starts at column c0 come in two steps, so that their loads overlap
// with the other loads of an item.  First this thread's mask word or directory entry (the addresses
// follow from the slot alone):
__device__ __forceinline__ uint32_t slice_fetch(const unsigned char* ws, const SampleArgs& a, int c0) {
  const int tid = fresh_tid();
  const unsigned char* ht = ws + WS_HT;
  const int n_pairs = (((a.V + 31) >> 5) + 1) >> 1;  // the mask is stored in whole pairs of words
  const int w0 = c0 >> 5, p0 = c0 >> 6;
  uint32_t v = 0u;
  if (tid < SLC / 32) { if (w0 + tid < 2 * n_pairs) v = as_global(reinterpret_cast<const uint32_t*>(ht))[w0 + tid]; }
  else if (tid < SLC / 32 + SLC / 64 + 1) {
    const int j = tid - SLC / 32;
    if (p0 + j < n_pairs) v = (uint32_t)as_global(reinterpret_cast<const uint16_t*>(ht + a.F.dir))[p0 + j];
  }
  return v;
}
// ... stored to LDS (past the directory's end stands the number of distinct columns); a barrier must follow.
__device__ __forceinline__ void slice_store(SliceTabs& T, uint32_t v, const SampleArgs& a, int c0, uint32_t distinct) {
  const int tid = fresh_tid();
  const int n_pairs = (((a.V + 31) >> 5) + 1) >> 1;
  if (tid < SLC / 32) T.bm[tid] = v;
  else if (tid < SLC / 32 + SLC / 64 + 1) {
    const int j = tid - SLC / 32;
    T.dir[j] = ((c0 >> 6) + j < n_pairs) ? v : distinct;
  }
}
// Then, once the directory is in LDS, the counts of the slice's columns; a barrier must follow.
__device__ __forceinline__ void slice_counts(SliceTabs& T, const unsigned char* ws, const SampleArgs& a) {
  const uint16_t* gcnt = reinterpret_cast<const uint16_t*>(ws + WS_HT + a.F.cnt);
  const unsigned r0 = T.dir[0];
  const unsigned nc = min(T.dir[SLC / 64] - r0, (unsigned)SLC);
  for (unsigned t = threadIdx.x; t < nc; t += WT) T.cnt[t] = as_global(gcnt)[r0 + t];
}
__device__ inline void load_slice(SliceTabs& T, const WideRow& W, const SampleArgs& a, int c0) {  // ends with a barrier
  const uint32_t v = slice_fetch(W.ws, a, c0);
  slice_store(T, v, a, c0, W.distinct);
  __syncthreads();
  slice_counts(T, W.ws, a);
  __syncthreads();
}
// Z' of column c0 + o, whose mask bit is set.
__device__ __forceinline__ float slice_value(float z, int o, const SliceTabs& T, const WideRow& W) {
  const int wl = o >> 5;
  const uint32_t word = T.bm[wl];
  unsigned r = T.dir[wl >> 1] - T.dir[0];
  if (wl & 1) r += (unsigned)__popc(T.bm[wl - 1]);
  r += (unsigned)__popc(word & ((1u << (o & 31)) - 1u));
  return apply_penalties(z, (uint32_t)T.cnt[min(r, (unsigned)SLC - 1u)], W.rep, W.inv_rep, W.freq, W.pres);
}
__device__ __forceinline__ bool slice_bit(int o, const SliceTabs& T) { return (T.bm[o >> 5] >> (o & 31)) & 1u; }
// The history columns of a slice, one mask word per thread.  Their logits and the slice's counts are
// requested first (hist_fetch, right after the mask and directory reached LDS) and used later
// (hist_columns), so that their way through memory overlaps with the slice's main line, which skips
// these columns and carries no table lookups.
constexpr int HPRE = 4;  // history columns per mask word whose logits are requested ahead; more are read in place
template <typename DT>
struct HistPre { typename Io<DT>::Elem z[HPRE]; uint32_t cnt; };
template <typename DT>
__device__ __forceinline__ void hist_fetch(HistPre<DT>& P, const SliceTabs& T, const unsigned char* ws, const SampleArgs& a,
                                           const DT* rowp, int c0, int V) {
  const int tid = fresh_tid();
  const uint16_t* gcnt = reinterpret_cast<const uint16_t*>(ws + WS_HT + a.F.cnt);
  const unsigned r0 = T.dir[0];
  const unsigned nc = min(T.dir[SLC / 64] - r0, (unsigned)SLC);
  P.cnt = 0u;
  if ((unsigned)tid < nc) P.cnt = (uint32_t)as_global(gcnt)[r0 + tid];
#pragma unroll
  for (int k = 0; k < HPRE; ++k) P.z[k] = typename Io<DT>::Elem();
  if (tid < SLC / 32) {
    uint32_t word = T.bm[tid];
#pragma unroll
    for (int k = 0; k < HPRE; ++k) {
      if (word) {
        const int idx = c0 + 32 * tid + (__ffs((int)word) - 1);
        word &= word - 1u;
        if (idx < V) P.z[k] = Io<DT>::raw(rowp + idx);
      }
    }
  }
}
// The counts go to LDS (first WT of them from the registers, the rest from memory), and so do the
// logits and columns of the first HCAP history columns, by rank; a barrier must follow.
template <typename DT>
__device__ __forceinline__ void hist_stage(SliceTabs& T, const HistPre<DT>& P, const unsigned char* ws, const SampleArgs& a,
                                           const DT* rowp, int c0, int V) {
  const int tid = fresh_tid();
  const uint16_t* gcnt = reinterpret_cast<const uint16_t*>(ws + WS_HT + a.F.cnt);
  const unsigned r0 = T.dir[0];
  const unsigned nc = min(T.dir[SLC / 64] - r0, (unsigned)SLC);
  if ((unsigned)tid < nc) T.cnt[tid] = (uint16_t)P.cnt;
  for (unsigned t = tid + WT; t < nc; t += WT) T.cnt[t] = as_global(gcnt)[r0 + t];
  if (tid < SLC / 32) {
    uint32_t word = T.bm[tid];
    unsigned r = T.dir[tid >> 1] - r0 + ((tid & 1) ? (unsigned)__popc(T.bm[tid - 1]) : 0u);
    auto put = [&](float z_raw) {
      T.hz[r] = z_raw;
      T.hcol[r] = (uint16_t)(32 * tid + (__ffs((int)word) - 1));
      word &= word - 1u;
      ++r;
    };
#pragma unroll
    for (int k = 0; k < HPRE; ++k) if (word && r < (unsigned)HCAP) put(Io<DT>::cvt(P.z[k]));
    while (word && r < (unsigned)HCAP) {
      const int idx = c0 + 32 * tid + (__ffs((int)word) - 1);
      put(idx < V ? Io<DT>::one(rowp + idx) : 0.0f);
    }
  }
}
// f(z', idx) for each history column of the slice, with its penalised value: the staged ones one per
// thread, the rest (a slice with more than HCAP of them) by their mask word's thread.
template <typename DT, typename F>
__device__ __forceinline__ void hist_columns(const SliceTabs& T, const WideRow& W, const DT* rowp, int c0, int V, F&& f) {
  const int tid = fresh_tid();
  const unsigned nc = min(T.dir[SLC / 64] - T.dir[0], (unsigned)SLC);
  for (unsigned j = tid; j < min(nc, (unsigned)HCAP); j += WT) {
    const int idx = c0 + (int)T.hcol[j];
    if (idx < V) f(apply_penalties(T.hz[j], (uint32_t)T.cnt[j], W.rep, W.inv_rep, W.freq, W.pres), idx);
  }
  if (nc > (unsigned)HCAP && tid < SLC / 32) {
    uint32_t word = T.bm[tid];
    unsigned r = T.dir[tid >> 1] - T.dir[0] + ((tid & 1) ? (unsigned)__popc(T.bm[tid - 1]) : 0u);
    while (word) {
      const int idx = c0 + 32 * tid + (__ffs((int)word) - 1);
      word &= word - 1u;
      if (r >= (unsigned)HCAP && idx < V)
        f(apply_penalties(Io<DT>::one(rowp + idx), (uint32_t)T.cnt[min(r, (unsigned)SLC - 1u)], W.rep, W.inv_rep, W.freq, W.pres), idx);
      ++r;
    }
  }
}

// The bin that holds the cut, from the masses of the first pass: cumulative mass from the top
// reaches top_p * total.  bstar < 0 if none.  Ends with a barrier.
constexpr u64 MASS_BITS = (1ull << CNT_SHIFT) - 1ull;
__device__ inline int find_cut(FS& S, const WideRow& W, u64& s_tot) {
  const int tid = threadIdx.x;
  constexpr int BPT = NBW / WT;
  const u64* gh = reinterpret_cast<const u64*>(W.ws + WS_HIST);
  const u64 m_top = as_global(reinterpret_cast<const u64*>(W.ws + WS_SCAL))[0];
  u64 hm[BPT]; u64 loc = 0ull;
#pragma unroll
  for (int j = 0; j < BPT; ++j) { hm[j] = as_global(gh)[tid * BPT + j] & MASS_BITS; loc += hm[j]; }
  if (tid == 0) S.bk = -1;
  unsigned ce, ct; u64 me, mt;
  blk_excl_scan2<WNW>(S, 0u, loc, ce, me, ct, mt);
  s_tot = m_top + mt;  // the bins are exact sums: this is the mass of the whole row
  const u64 target = (u64)__double2ull_ru((double)W.top_p * (double)s_tot);
  u64 run = m_top + me;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    if (run < target && run + hm[j] >= target) S.bk = tid * BPT + j;
    run += hm[j];
  }
  __syncthreads();
  const int bstar = S.bk;
  __syncthreads();
  return bstar;
}
// The same by count, for top-k alone: the bin in which the number of columns from the top reaches
// top_k.  bstar < 0 if none (already top_k columns at or above g, or fewer than top_k in all).
__device__ inline int find_cut_k(FS& S, const WideRow& W) {
  const int tid = threadIdx.x;
  constexpr int BPT = NBW / WT;
  const u64* gh = reinterpret_cast<const u64*>(W.ws + WS_HIST);
  const unsigned n_top = as_global(reinterpret_cast<const uint32_t*>(W.ws + WS_SCAL))[7];
  unsigned hc[BPT], loc = 0u;
#pragma unroll
  for (int j = 0; j < BPT; ++j) { hc[j] = (unsigned)(as_global(gh)[tid * BPT + j] >> CNT_SHIFT); loc += hc[j]; }
  if (tid == 0) S.bk = -1;
  unsigned ce, ct; u64 me, mt;
  blk_excl_scan2<WNW>(S, loc, 0ull, ce, me, ct, mt);
  const unsigned target = (unsigned)W.top_k;
  unsigned run = n_top + ce;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    if (run < target && run + hc[j] >= target) S.bk = tid * BPT + j;
    run += hc[j];
  }
  __syncthreads();
  const int bstar = S.bk;
  __syncthreads();
  return bstar;
}

// How a column is classified, per route: it surely survives iff its tempered value reaches thr_y and it
// lies at or above g or in a bin before bstar; columns of bin bstar are resolved one by one.
struct RowCut { int bstar; float thr_y; bool valid; u64 s_tot; /* top-p route: exact mass of the row */ };
__device__ inline RowCut row_cut(FS& S, const WideRow& W) {  // every thread calls; barriers inside on one route
  RowCut c;
  c.thr_y = -INFINITY; c.valid = true; c.s_tot = 0ull;
  if (W.mode == WIDE_TOP_P) { c.bstar = find_cut(S, W, c.s_tot); c.valid = c.bstar >= 0; }
  else if (W.mode == WIDE_TOP_K) { c.bstar = find_cut_k(S, W); c.valid = c.bstar >= 0; }
  else c.bstar = NBW;  // no bin holds a cut
  if (W.mode != WIDE_ALL && W.min_p > 0.0f) {  // min-p, alone or on top of top-p: the shorter prefix wins
    const uint32_t kmax = as_global(reinterpret_cast<const uint32_t*>(W.ws + WS_SCAL))[6];
    c.valid = c.valid && kmax > KEY_NEG_INF;
    c.thr_y = keyf(kmax) + (float)log((double)W.min_p);  // fl(y_max + fl(ln min_p)), as in the list's epilogue
  }
  return c;
}

// Smallest float, in the order of the keys, at which a predicate that is monotone in its argument
// (false, then true) holds; +inf if it holds nowhere.  One wave, 64 candidates per round, no LDS
// and no barrier; the result is the same in every lane.
template <typename P>
__device__ __forceinline__ float wave_lower_bound(P&& pred) {
  const unsigned lane = threadIdx.x & 63u;
  uint32_t lo = KEY_NEG_INF, hi = KEY_POS_INF;
  if (__ballot(pred(keyf(hi))) == 0ull) return INFINITY;
  while (lo < hi) {  // the answer lies in [lo, hi] and the predicate holds at hi
    const u64 step = ((u64)hi - (u64)lo + 63ull) / 64ull;
    const u64 c = (u64)lo + step * (u64)lane;
    const uint32_t cand = (c < (u64)hi) ? (uint32_t)c : hi;
    const u64 m = __ballot(pred(keyf(cand)));
    if (m == 0ull) { lo = (uint32_t)((u64)lo + 63ull * step) + 1u; continue; }  // lane 63 stood below hi
    const unsigned f = (unsigned)__ffsll((long long)m) - 1u;
    const u64 cf = (u64)lo + step * (u64)f;
    const uint32_t top = (cf < (u64)hi) ? (uint32_t)cf : hi;
    lo = f ? (uint32_t)((u64)lo + step * (u64)(f - 1u)) + 1u : top;
    hi = top;
  }
  return keyf(uni(lo));
}
// The same, trying first the 64 floats around a guess: one round when the answer lies among them.
template <typename P>
__device__ __forceinline__ float wave_lower_bound_near(float guess, P&& pred) {
  const unsigned lane = threadIdx.x & 63u;
  const uint32_t kg = fkey(uni(guess));
  if (guess == guess && kg >= KEY_NEG_INF + 32u && kg <= KEY_POS_INF - 32u) {
    const u64 m = __ballot(pred(keyf(kg - 32u + lane)));
    if (!(m & 1ull) && (m >> 63)) return keyf(uni(kg - 32u + (uint32_t)__ffsll((long long)m) - 1u));
  }
  return wave_lower_bound(pred);
}
// The classification of a column by its logit alone.  Tempered value, bin and the comparison with
// g are all monotone in z, so each test holds from one float upwards, and so do their
// combinations: a column surely survives iff z >= z_sure, and is a boundary column iff
// z_edge <= z < z_sure.  Every wave computes the same two numbers.
struct ZCut { float z_sure, z_edge; };
__device__ __forceinline__ ZCut z_cut(const WideRow& W, int bstar, float thr_y) {
  // smallest z whose tempered value reaches the min-p threshold
  float z_thr = -INFINITY;
  if (thr_y > -INFINITY) z_thr = wave_lower_bound_near(thr_y * W.tau, [&](float z) { return tempered(z, W.C) >= thr_y; });
  // smallest z whose bin lies before `limit` (bins count downwards from y_g, 1 / BINS_PER_LOG2 of a log2 each)
  auto before_bin = [&](int limit) -> float {
    if (limit >= NBW) return -INFINITY;
    if (limit <= 0) return INFINITY;
    const float y_guess = W.C.y_g - (float)limit * (0.6931471805599453f / BINS_PER_LOG2);
    return wave_lower_bound_near(y_guess * W.tau, [&](float z) { int b; (void)mass_term(z, W.C, b); return b < limit; });
  };
  const float z_a = before_bin(bstar), z_b = before_bin(bstar + 1);
  ZCut c;  // sure: y >= thr and (z >= g or bin < bstar); sure or boundary: the same with bin <= bstar
  c.z_sure = fmaxf(z_thr, fminf(W.C.g, z_a));
  c.z_edge = fmaxf(z_thr, fminf(W.C.g, z_b));
  return c;
}

// Work split: items are (queued row, slice) pairs in row-major order; a workgroup takes a
// contiguous range, so that it meets few distinct rows.
struct Items { unsigned i0, i1, n_sl; };
__device__ __forceinline__ Items my_items(const SampleArgs& a) {
  Items I;
  const unsigned n_wide = min(as_global(a.wq)[a.parity], (unsigned)a.wide_slots);
  I.n_sl = (unsigned)((a.V + SLC - 1) / SLC);
  const unsigned items = n_wide * I.n_sl;
  const unsigned chunk = (items + gridDim.x - 1u) / gridDim.x;
  I.i0 = min(items, blockIdx.x * chunk);
  I.i1 = min(items, I.i0 + chunk);
  return I;
}

// What an item needs from memory before its columns can be processed; requested one item ahead.
// The row and history flag of a queue slot come from the slot's record: a workgroup's items are
// contiguous, so it keeps them for its current slot and the next.
template <typename DT>
struct ItemLoads {
  static constexpr int G = SLC / (WT * Io<DT>::EPL);  // 16-byte groups per thread and slice
  typename Io<DT>::Raw A[G];
  uint32_t hq[G];  // hot-set bits of each group's columns
  uint32_t pre;    // this thread's mask word or directory entry
};
struct SlotIds {
  uint32_t row_c, act_c, row_n, act_n;  // current slot, next slot; act: bit 0 history in force, bit 1 no truncation
  __device__ __forceinline__ void request(const SampleArgs& a, unsigned slot, unsigned n_wide, uint32_t& row, uint32_t& act) {
    row = 0u; act = 0u;
    if (slot < n_wide) {
      const uint32_t* rec = reinterpret_cast<const uint32_t*>(reinterpret_cast<const WideRec*>(a.wq + WQ_HEAD) + slot);
      row = as_global(rec)[0];
      act = (as_global(rec)[11] != 0u ? 1u : 0u) | (as_global(rec)[2] == (uint32_t)WIDE_ALL ? 2u : 0u);
    }
  }
  // The record is the same in every lane: scalars from here on.  Called where the workgroup waits
  // for its loads anyway (a row's record), so that no later use has to wait for loads in flight.
  __device__ __forceinline__ void settle() { row_c = uni(row_c); act_c = uni(act_c); row_n = uni(row_n); act_n = uni(act_n); }
};
static_assert(offsetof(WideRec, row) == 0 && offsetof(WideRec, mode) == 8 && offsetof(WideRec, h_active) == 44, "record words read by SlotIds");
// skip_all: rows without truncation need nothing from this pass (the bins kernel)
template <typename DT, bool use_hot, bool skip_all = false>
__device__ __forceinline__ void item_fetch(ItemLoads<DT>& L, const SampleArgs& a, unsigned item, unsigned n_sl, int cur_slot, const SlotIds& ids) {
  constexpr int EPL = Io<DT>::EPL;
  const int tid = threadIdx.x;
  const int slot = (int)(item / n_sl), c0 = (int)(item % n_sl) * SLC;
  const uint32_t row = slot == cur_slot ? ids.row_c : ids.row_n;  // scalars (SlotIds::settle)
  const uint32_t actw = slot == cur_slot ? ids.act_c : ids.act_n;
  const bool act = (actw & 1u) != 0u;
  if (skip_all && (actw & 2u)) return;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)row * (size_t)a.stride;
  L.pre = act ? slice_fetch(a.wws + (size_t)slot * a.ws_stride, a, c0) : 0u;
#pragma unroll
  for (int j = 0; j < ItemLoads<DT>::G; ++j) {
    const int idx0 = c0 + (j * WT + tid) * EPL;
    L.hq[j] = 0u;
    L.A[j] = typename Io<DT>::Raw();
    if (idx0 + EPL <= a.V) L.A[j] = Io<DT>::load(rowp + idx0);
    if (use_hot && idx0 < a.V) L.hq[j] = (as_global(a.hot_bits)[idx0 >> 5] >> ((unsigned)idx0 & 31u)) & ((1u << EPL) - 1u);
  }
}

// ---------------------------------------------------------------- bins ------------------------
template <typename DT>
__global__ __launch_bounds__(WT, (sizeof(DT) == 4 ? 4 : 5)) void wide_bins_kernel(const SampleArgs a) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int G = ItemLoads<DT>::G;
  __shared__ SliceTabs Tb;
  __shared__ u64 lh[NBW + 1];  // the bins, and the mass at or above g
  __shared__ FS S;
  const int tid = threadIdx.x;
  const int V = a.V;
  // mask word and bit of this thread's first column in each of its groups (a group step is whole words)
  const int wbase = (tid * EPL) >> 5;
  const unsigned wsh = (unsigned)(tid * EPL) & 31u;
  static_assert((WT * EPL) % 32 == 0, "group stride in mask words");
  const Items I = my_items(a);
  if (I.i0 >= I.i1) return;
  const unsigned n_wide = min(as_global(a.wq)[a.parity], (unsigned)a.wide_slots);
  int cur = (int)(I.i0 / I.n_sl);
  SlotIds ids;
  ids.request(a, (unsigned)cur, n_wide, ids.row_c, ids.act_c);
  ids.request(a, (unsigned)cur + 1u, n_wide, ids.row_n, ids.act_n);
  WideRow W = load_row(a, (unsigned)cur);
  ids.settle();
  {  // nothing to do for rows without truncation (a workgroup's items lie in at most two slots)
    const int last = (int)((I.i1 - 1u) / I.n_sl);
    if ((ids.act_c & 2u) && (last == cur || (last == cur + 1 && (ids.act_n & 2u)))) return;
  }
  ItemLoads<DT> N;  // the next item's loads
  item_fetch<DT, false, true>(N, a, I.i0, I.n_sl, cur, ids);
  for (int b = tid; b <= NBW; b += WT) lh[b] = 0ull;
  u64 mtop = 0ull;
  unsigned ntop = 0u;      // top-k route: columns at or above g seen by this thread
  float ymax = -INFINITY;  // rows with a min-p cut: largest tempered value seen by this thread
  auto flush = [&]() {
    __syncthreads();
    if (W.mode == WIDE_TOP_P || W.mode == WIDE_TOP_K) {
      u64* gh = reinterpret_cast<u64*>(W.ws + WS_HIST);
      for (int b = tid; b < NBW; b += WT) { const u64 v = lh[b]; if (v) atomicAdd(&gh[b], v); }
      const u64 t = blk_sum_u64<WNW>(S, mtop) + lh[NBW];
      if (tid == 0 && t) atomicAdd(reinterpret_cast<u64*>(W.ws + WS_SCAL), t);
      if (W.mode == WIDE_TOP_K) {
        const unsigned nt = wave_sum(ntop);
        if ((tid & 63) == 0 && nt) atomicAdd(reinterpret_cast<uint32_t*>(W.ws + WS_SCAL) + 7, nt);
      }
    }
    if (W.min_p > 0.0f) {
      const float m = wave_max(ymax);
      if ((tid & 63) == 0 && m > -INFINITY) atomicMax(reinterpret_cast<uint32_t*>(W.ws + WS_SCAL) + 6, fkey(m));
    }
    mtop = 0ull; ntop = 0u; ymax = -INFINITY;
  };
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    const int c0 = sl * SLC;
    const ItemLoads<DT> L = N;
    const bool more = it + 1u < I.i1;
    if (slot != cur) {
      flush();
      cur = slot;
      ids.row_c = ids.row_n; ids.act_c = ids.act_n;
      ids.request(a, (unsigned)slot + 1u, n_wide, ids.row_n, ids.act_n);
      W = load_row(a, (unsigned)slot);
      ids.settle();
      for (int b = tid; b <= NBW; b += WT) lh[b] = 0ull;
    }
    if (W.mode == WIDE_ALL) {  // every column survives: nothing to find in a first pass
      if (more) item_fetch<DT, false, true>(N, a, it + 1u, I.n_sl, cur, ids);
      continue;
    }
    const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
    HistPre<DT> HP;
    if (W.h_active) {
      slice_store(Tb, L.pre, a, c0, W.distinct);
      __syncthreads();
      hist_fetch<DT>(HP, Tb, W.ws, a, rowp, c0, V);  // this item's own loads go first: loads return in order
    } else __syncthreads();  // the zeroed bins are visible
    if (more) item_fetch<DT, false, true>(N, a, it + 1u, I.n_sl, cur, ids);
    auto one = [&](float z, int) {
      if (W.mode == WIDE_MIN_P) { ymax = fmaxf(ymax, tempered(z, W.C)); return; }
      int b; float y;
      const float w = mass_term(z, W.C, b, y);
      ymax = fmaxf(ymax, y);
      // top-k route: a bin also counts its columns, above its mass
      if (z < W.C.g) atomicAdd(&lh[b], mass_fix_below(w) | (W.mode == WIDE_TOP_K ? 1ull << CNT_SHIFT : 0ull));
      else { mtop += mass_fix(fminf(w, W_LIMIT)); ++ntop; }
    };
    if (W.mode == WIDE_MIN_P) {  // the row maximum is all a value cut needs
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int idx0 = c0 + (j * WT + tid) * EPL;
        if (idx0 + EPL <= V) {
          float z[EPL];
          Io<DT>::unpack(L.A[j], z);
          const uint32_t nib = W.h_active ? (Tb.bm[wbase + j * (WT * EPL / 32)] >> wsh) & ((1u << EPL) - 1u) : 0u;
          float zm = -INFINITY;  // the tempered value is monotone in z: one division per group
#pragma unroll
          for (int e = 0; e < EPL; ++e) zm = ((nib >> e) & 1u) ? zm : fmaxf(zm, z[e]);
          ymax = fmaxf(ymax, tempered(zm, W.C));
        } else {
          for (int idx = idx0; idx < V; ++idx)
            if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
        }
      }
    } else {
      auto sweep = [&](auto unit_tau_c, auto top_k_c) {
        constexpr bool UT = decltype(unit_tau_c)::value, TOPK = decltype(top_k_c)::value;
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const int idx0 = c0 + (j * WT + tid) * EPL;
          if (idx0 + EPL <= V) {
            float z[EPL];
            Io<DT>::unpack(L.A[j], z);
            uint32_t nib = 0u;
            if (W.h_active) {  // history columns are handled below: here they count as -inf (no mass)
              nib = (Tb.bm[wbase + j * (WT * EPL / 32)] >> wsh) & ((1u << EPL) - 1u);
#pragma unroll
              for (int e = 0; e < EPL; ++e) z[e] = ((nib >> e) & 1u) ? -INFINITY : z[e];
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) {  // straight-line: the columns at or above g share one more slot
              int b;
              const float w = mass_term<UT>(z[e], W.C, b);
              uint32_t hi, lo;
              float_to_parts(fminf(w, W_LIMIT) * MSCALE, hi, lo);
              const bool below = z[e] < W.C.g;
              u64 v = parts_to_u64(hi, lo);
              if (TOPK) {  // the bin counts the column too (not the history columns, handled below)
                v |= (below && !((nib >> e) & 1u)) ? 1ull << CNT_SHIFT : 0ull;
                ntop += below ? 0u : 1u;
              }
              atomicAdd(&lh[below ? b : NBW], v);
            }
            if (W.min_p > 0.0f) {  // the tempered value is monotone in z: one division per group
              float zm = z[0];
#pragma unroll
              for (int e = 1; e < EPL; ++e) zm = fmaxf(zm, z[e]);
              ymax = fmaxf(ymax, tempered(zm, W.C));
            }
          } else {
            for (int idx = idx0; idx < V; ++idx)
              if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
          }
          __builtin_amdgcn_sched_barrier(0);  // one group at a time: interleaving them costs registers
        }
      };
      const std::true_type yes{};
      const std::false_type no{};
      if (W.mode == WIDE_TOP_K) { if (W.tau == 1.0f) sweep(yes, yes); else sweep(no, yes); }
      else { if (W.tau == 1.0f) sweep(yes, no); else sweep(no, no); }
    }
    if (W.h_active) {  // the history columns, whose logits and counts were requested before the main line
      hist_stage<DT>(Tb, HP, W.ws, a, rowp, c0, V);
      __syncthreads();
      hist_columns<DT>(Tb, W, rowp, c0, V, one);
      __syncthreads();  // the tables are rewritten by the next item
    }
  }
  flush();
}

// ---------------------------------------------------------------- classify --------------------
template <typename DT, bool use_hot>  // use_hot: a hot set is installed (section 5.3): masses are split by class
__global__ __launch_bounds__(WT, 4) void wide_classify_kernel(const SampleArgs a) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int G = ItemLoads<DT>::G;  // a slice is one tile of the draw's walk
  constexpr unsigned EMASK = (1u << EPL) - 1u;
  __shared__ SliceTabs Tb;
  __shared__ u64 lrl[LCAP];  // boundary columns of the current row found by this workgroup, not yet written out
  __shared__ u64 ltile[2];
  __shared__ unsigned l_n, l_base;
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63;
  const int V = a.V;
  // mask word and bit of this thread's first column in each of its groups (a group step is whole words)
  const int wbase = (tid * EPL) >> 5;
  const unsigned wsh = (unsigned)(tid * EPL) & 31u;
  static_assert((WT * EPL) % 32 == 0, "group stride in mask words");
  const Items I = my_items(a);
  if (I.i0 >= I.i1) return;
  const uint32_t* hot_bits = a.hot_bits;
  const unsigned n_wide = min(as_global(a.wq)[a.parity], (unsigned)a.wide_slots);
  int cur = (int)(I.i0 / I.n_sl);
  SlotIds ids;
  ids.request(a, (unsigned)cur, n_wide, ids.row_c, ids.act_c);
  ids.request(a, (unsigned)cur + 1u, n_wide, ids.row_n, ids.act_n);
  ids.settle();
  ItemLoads<DT> N;  // the next item's loads
  item_fetch<DT, use_hot>(N, a, I.i0, I.n_sl, cur, ids);
  WideRow W;
  int bstar = -1;
  float thr_y = -INFINITY;
  bool valid = false;
  ZCut zc = {INFINITY, INFINITY};
  auto enter_row = [&](int slot) {  // barriers inside
    W = load_row(a, (unsigned)slot);
    ids.settle();
    const RowCut rc = row_cut(S, W);
    bstar = rc.bstar; thr_y = rc.thr_y; valid = rc.valid;
    if (valid) zc = z_cut(W, bstar, thr_y);
  };
  // What a thread gathers over this workgroup's slices of one row, reduced when the row ends:
  unsigned n_sure = 0u;    // sure columns
  u64 acc_all = 0ull;      // exact mass of every column (routes without bins)
  float ymax = -INFINITY;  // largest tempered value
  bool bad = false;        // a mass the fixed point cannot carry, or a NaN
  // Writes the staged boundary columns to the row's list.  All threads call, after a barrier that
  // follows the last append; ends with a barrier.
  auto list_out = [&]() {
    const unsigned nb = l_n;
    if (nb == 0u) return;
    uint32_t* sc = reinterpret_cast<uint32_t*>(W.ws + WS_SCAL);
    // more columns than the stage holds: the count is pushed past the limit, so that the finishing
    // kernel hands the row on
    if (tid == 0) l_base = atomicAdd(&sc[3], nb > (unsigned)LCAP ? (unsigned)RCAP + 1u : nb);
    __syncthreads();
    const unsigned base = l_base;
    if (nb <= (unsigned)LCAP)
      for (unsigned t = tid; t < nb; t += WT)
        if (base + t < (unsigned)RCAP) reinterpret_cast<u64*>(W.ws + WS_RL)[base + t] = lrl[t];
    if (tid == 0) l_n = 0u;
    __syncthreads();
  };
  auto leave_row = [&]() {  // barriers inside
    if (!valid) return;
    __syncthreads();
    list_out();
    uint32_t* sc = reinterpret_cast<uint32_t*>(W.ws + WS_SCAL);
    const float m = wave_max(ymax);
    if (lane == 0 && m > -INFINITY) atomicMax(&sc[6], fkey(m));
    if (__ballot(bad) && lane == 0) atomicAdd(&sc[3], (unsigned)RCAP + 1u);  // the finishing kernel hands the row on
    unsigned ns = n_sure, dz = 0u; u64 mx = 0ull, dsum = acc_all;
    blk_reduce<WNW>(S, ns, dz, mx, dsum);
    if (tid == 0) {
      if (ns) atomicAdd(&sc[2], ns);
      if (dsum) atomicAdd(reinterpret_cast<u64*>(W.ws + WS_SCAL + 16), dsum);
    }
    n_sure = 0u; acc_all = 0ull; ymax = -INFINITY; bad = false;
  };
  if (tid == 0) l_n = 0u;
  enter_row(cur);
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    const ItemLoads<DT> L = N;
    const bool more = it + 1u < I.i1;
    if (slot != cur) {
      leave_row();
      cur = slot;
      ids.row_c = ids.row_n; ids.act_c = ids.act_n;
      ids.request(a, (unsigned)slot + 1u, n_wide, ids.row_n, ids.act_n);
      enter_row(slot);
    }
    if (!valid) {  // the finishing kernel hands the row on
      if (more) item_fetch<DT, use_hot>(N, a, it + 1u, I.n_sl, cur, ids);
      continue;
    }
    const int c0 = sl * SLC;
    const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
    if (tid < 2) ltile[tid] = 0ull;
    if (W.h_active) slice_store(Tb, L.pre, a, c0, W.distinct);
    __syncthreads();
    HistPre<DT> HP;
    if (W.h_active) hist_fetch<DT>(HP, Tb, W.ws, a, rowp, c0, V);  // this item's own loads go first: loads return in order
    if (more) item_fetch<DT, use_hot>(N, a, it + 1u, I.n_sl, cur, ids);
    u64 acc_s = 0ull, acc1 = 0ull;  // this slice: mass of the sure columns, and of the hot ones among them
    // one column the slow way: history columns and the ragged end of the row
    auto one = [&](float z, int idx) {
      int b; float y;
      const float w = mass_term(z, W.C, b, y);
      const bool below = z < W.C.g;
      if (!below && !(w <= W_LIMIT)) { bad = true; return; }
      const u64 m = below ? mass_fix_below(w) : mass_fix(w);
      acc_all += m;
      ymax = fmaxf(ymax, y);
      if (!(y >= thr_y)) return;
      if (!below || b < bstar) {
        acc_s += m;
        if (use_hot && hot_bit(hot_bits, (uint32_t)idx)) acc1 += m;
        ++n_sure;
      } else if (b == bstar) {
        const unsigned s = atomicAdd(&l_n, 1u);
        if (s < (unsigned)LCAP) lrl[s] = ((u64)__float_as_uint(z) << 32) | (u64)(uint32_t)idx;
      }
    };
    // The main line: every column's mass, and its class by the logit alone; boundary columns follow
    // under a wave-wide test.
    auto sweep = [&](auto unit_tau_c, auto want_all_c, auto all_sure_c) {
      // UT: tau == 1; WANT_ALL: the row's mass is summed here (no bins); ALL_SURE: no truncation, every column survives
      constexpr bool UT = decltype(unit_tau_c)::value, WANT_ALL = decltype(want_all_c)::value, ALL_SURE = decltype(all_sure_c)::value;
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int idx0 = c0 + (j * WT + tid) * EPL;
        if (idx0 + EPL <= V) {
          float z[EPL];
          Io<DT>::unpack(L.A[j], z);
          bool any_edge = false;
          uint32_t live = ~0u;
          if (W.h_active) {  // history columns are handled below: here they carry no mass
            live = ~((Tb.bm[wbase + j * (WT * EPL / 32)] >> wsh) & EMASK);
#pragma unroll
            for (int e = 0; e < EPL; ++e) z[e] = ((live >> e) & 1u) ? z[e] : -INFINITY;
            // ... but -inf counts as sure when every value does
            if (ALL_SURE || zc.z_sure == -INFINITY) n_sure -= (unsigned)__popc(~live & EMASK);
          }
          // group sums of the masses' two parts (units of 2^24, and the rest): <= 8 terms of <= 2^25
          uint32_t sh = 0u, sl_ = 0u, hh = 0u, hl = 0u, ah = 0u, al = 0u;
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            int b; float y;
            const float w = mass_term<UT>(z[e], W.C, b, y);
            bad = bad || !(w <= W_LIMIT);  // a mass the fixed point cannot carry, or a NaN
            uint32_t hi, lo;
            float_to_parts(w * MSCALE, hi, lo);
            ymax = fmaxf(ymax, y);
            if (ALL_SURE) {
              sh += hi; sl_ += lo;
              if (use_hot) { const uint32_t hm = (uint32_t)(-(int32_t)((L.hq[j] >> e) & 1u)); hh += hi & hm; hl += lo & hm; }
            } else {
              const bool sure = z[e] >= zc.z_sure;
              const uint32_t his = sure ? hi : 0u, los = sure ? lo : 0u;
              sh += his; sl_ += los;
              if (use_hot) { const uint32_t hm = (uint32_t)(-(int32_t)((L.hq[j] >> e) & 1u)); hh += his & hm; hl += los & hm; }
              if (WANT_ALL) { ah += hi; al += lo; }
              n_sure += sure ? 1u : 0u;
              any_edge = any_edge || (z[e] >= zc.z_edge && !sure);
            }
          }
          acc_s += parts_to_u64(sh, sl_);
          if (use_hot) acc1 += parts_to_u64(hh, hl);
          if (ALL_SURE) { acc_all += parts_to_u64(sh, sl_); n_sure += (unsigned)EPL; }
          else if (WANT_ALL) acc_all += parts_to_u64(ah, al);
          if (__ballot(any_edge)) {  // boundary columns: few per wave, element by element
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
              if (((live >> e) & 1u) && z[e] >= zc.z_edge && !(z[e] >= zc.z_sure)) {
                const unsigned s = atomicAdd(&l_n, 1u);
                if (s < (unsigned)LCAP) lrl[s] = ((u64)__float_as_uint(z[e]) << 32) | (u64)(uint32_t)(idx0 + e);
              }
            }
          }
        } else {
          for (int idx = idx0; idx < V; ++idx)
            if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
        }
        __builtin_amdgcn_sched_barrier(0);  // one group at a time: interleaving them costs registers
      }
    };
    // the top-p route has the row's mass from its bins; the other routes sum it here
    const std::true_type yes{};
    const std::false_type no{};
    if (W.tau == 1.0f) {
      if (W.mode == WIDE_TOP_P || W.mode == WIDE_TOP_K) sweep(yes, no, no); else if (W.mode == WIDE_ALL) sweep(yes, yes, yes); else sweep(yes, yes, no);
    } else {
      if (W.mode == WIDE_TOP_P || W.mode == WIDE_TOP_K) sweep(no, no, no); else if (W.mode == WIDE_ALL) sweep(no, yes, yes); else sweep(no, yes, no);
    }
    if (W.h_active) {  // the history columns, whose logits and counts were requested before the main line
      hist_stage<DT>(Tb, HP, W.ws, a, rowp, c0, V);
      __syncthreads();
      hist_columns<DT>(Tb, W, rowp, c0, V, one);
    }
    {
      const u64 s0 = wave_sum(acc_s - acc1);
      if (lane == 0 && s0) atomicAdd(&ltile[0], s0);
      if (use_hot) { const u64 s1 = wave_sum(acc1); if (lane == 0 && s1) atomicAdd(&ltile[1], s1); }
    }
    __syncthreads();  // the tile sums and this slice's appends are complete
    if (tid < 2 && sl < 256) reinterpret_cast<u64*>(W.ws + WS_TILES)[tid * 256 + sl] = ltile[tid];
    // every slice may add ICAP boundary columns before the stage has to be written out
    if (l_n > (unsigned)(LCAP - ICAP)) list_out();
  }
  leave_row();
}

// ---------------------------------------------------------------- finish ----------------------
__device__ inline void hand_on(const SampleArgs& a, int row) {
  const unsigned slot = atomicAdd(&a.pend[a.parity], 1u);
  a.pend[2 + slot] = (uint32_t)row;
  a.out[row] = PENDING;
}

template <typename DT>
__device__ inline bool finish_row(const SampleArgs& a, const WideRow& W, FS& S, SliceTabs& Tb, u64* rcmp, uint32_t* rl,
                                  u64* dmass, u64* tiles, simple_row_diag& dg) {
  constexpr int T = SLC;            // a tile of the draw's walk is a slice
  constexpr int EPT = T / WT;       // its columns per thread, contiguous
  const int tid = threadIdx.x;
  const int V = a.V;
  const StreamCtx& C = W.C;
  const uint32_t* hot_bits = a.hot_bits;
  const bool use_hot = hot_bits != nullptr;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
  double u3[3];
  row_uniforms(a.seed, a.row_offset + (uint64_t)W.row, a.step, u3);
  // every value of the slot this workgroup needs is requested before the first barrier
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(W.ws + WS_SCAL);
  const unsigned n_sure = as_global(sc)[2], n_r = as_global(sc)[3];
  const u64 S_sum = as_global(reinterpret_cast<const u64*>(W.ws + WS_SCAL))[2];  // mass of the row, summed by the classifying pass
  u64 tv[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) tv[k] = as_global(reinterpret_cast<const u64*>(W.ws + WS_TILES))[k * WT + tid];
  const uint32_t kmax = as_global(sc)[6];
  const RowCut rcut = row_cut(S, W);
  const int bstar = rcut.bstar;
  const float thr_y = rcut.thr_y;
  if (!rcut.valid) { return false; }
  const bool top_p_route = W.mode == WIDE_TOP_P, top_k_route = W.mode == WIDE_TOP_K;
  const bool cut_route = top_p_route || top_k_route;  // a cut inside a bin: by mass, or by count
  const u64 S_tot = top_p_route ? rcut.s_tot : S_sum;  // exact mass of the row (from the bins where there are bins)
  // a count past the limit is also how the classifying pass reports a row it could not handle; no
  // collected column on the top-p route means that a min-p cut ended the survivors above the bin
  const bool minp_too = top_p_route && W.min_p > 0.0f;
  if (n_r > (unsigned)RCAP || (!cut_route && n_r != 0u) || (cut_route && n_r == 0u && !minp_too)) { return false; }
  if (tid == 0) { S.bd = -1; S.cut_k = 0ull; S.cut_p = ~0ull; S.out_id = -1; S.out_w = 0ull; }
  tiles[tid] = tv[0]; tiles[WT + tid] = tv[1];
  const u64 msure = tv[0] + tv[1];
  u64 cut_found = 0ull;  // every collected column at or after it in the order survives; 0: no collected columns
  unsigned r_in = 0;
  if (cut_route && n_r == 0u) cut_found = ~0ull;  // nothing of the bin survives
  if (cut_route && n_r != 0u) {
  // exact masses (top-k: counts) from here: the columns surely inside must stay below the target, the
  // collected bin must reach it
  const u64 m_sure = blk_sum_u64<WNW>(S, msure);  // barriers inside
  const u64 m_above = top_k_route ? (u64)n_sure : m_sure;
  const u64 target = top_k_route ? (u64)W.top_k : (u64)__double2ull_ru((double)W.top_p * (double)S_tot);
  if (m_above >= target) { return false; }
  // -- the boundary bin, exactly: shortest prefix in the total order whose mass reaches the target --
  {
    u64 cmax_t = 0ull, cmin_t = ~0ull;
    const u64* grl = reinterpret_cast<const u64*>(W.ws + WS_RL);
    for (unsigned t0 = 0; t0 < n_r; t0 += 4u * WT) {  // four independent loads per thread and round
      u64 e[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) { const unsigned t = t0 + (unsigned)(k * WT + tid); e[k] = (t < n_r) ? as_global(grl)[t] : 0ull; }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const unsigned t = t0 + (unsigned)(k * WT + tid);
        if (t >= n_r) continue;
        const float z = __uint_as_float((uint32_t)(e[k] >> 32));
        int b;
        const float w = mass_term(z, C, b);
        const u64 c = composite(fkey(z / W.tau), (uint32_t)e[k]);
        rcmp[t] = c;
        rl[t] = (uint32_t)mass_fix_below(w);
        cmax_t = (c > cmax_t) ? c : cmax_t; cmin_t = (c < cmin_t) ? c : cmin_t;
      }
    }
    cmax_t = wave_all(cmax_t, [](u64 x, u64 y) { return x > y ? x : y; });
    cmin_t = wave_all(cmin_t, [](u64 x, u64 y) { return x < y ? x : y; });
    if ((tid & 63) == 0) { atomicMax(&S.cut_k, cmax_t); atomicMin(&S.cut_p, cmin_t); }
  }
  __syncthreads();
  // Radix descent, eight bits at a time from the top of (key, ~id): among the columns that share the
  // digits fixed so far, the digit whose mass carries the running total over the target is fixed
  // next.  Digits on which all columns agree are skipped; after the last one the cut column is known.
  {
    const u64 cmax = S.cut_k, differ = S.cut_k ^ S.cut_p;
    u64 prefix = 0ull, mask = 0ull, acc = m_above;
    bool ok = true;
    for (int shift = 56; shift >= 0; shift -= 8) {
      if ((differ >> shift) == 0ull) {  // no column differs here or above
        prefix |= cmax & (0xFFull << shift); mask |= 0xFFull << shift;
        continue;
      }
      dmass[tid] = 0ull;
      if (tid == 0) S.bp = -1;
      __syncthreads();
      for (unsigned t = tid; t < n_r; t += WT) {
        const u64 c = rcmp[t];
        if ((c & mask) == prefix) atomicAdd(&dmass[(unsigned)(c >> shift) & 0xFFu], top_k_route ? 1ull : (u64)rl[t]);
      }
      __syncthreads();
      {  // thread i looks at digit 255 - i: the exclusive scan sums the digits above it
        const u64 m = dmass[255 - tid];
        unsigned ce2, ct2; u64 me2, mt2;
        blk_excl_scan2<WNW>(S, 0u, m, ce2, me2, ct2, mt2);
        if (m > 0ull && acc + me2 < target && acc + me2 + m >= target) { S.bp = 255 - tid; S.mab_p = acc + me2; }
      }
      __syncthreads();
      const int d = S.bp;
      if (d < 0) { ok = false; break; }  // the collected columns do not reach the target: the passes disagree
      acc = S.mab_p;
      prefix |= (u64)(unsigned)d << shift; mask |= 0xFFull << shift;
      __syncthreads();
    }
    if (differ == 0ull && m_above + (top_k_route ? 1ull : (u64)rl[0]) < target) ok = false;  // a single column, and it does not reach the target
    // the collected columns do not reach the target: with a min-p cut those below it were never
    // collected, and the min-p prefix is the shorter one (all collected columns survive)
    if (!ok && !minp_too) { return false; }
    cut_found = ok ? prefix : 1ull;
  }
  if (cut_found == 0ull) { return false; }
  for (unsigned t = tid; t < n_r; t += WT) {
    if (rcmp[t] >= cut_found) {
      const uint32_t id = 0xFFFFFFFFu - (uint32_t)rcmp[t];
      const unsigned hot = use_hot ? hot_bit(hot_bits, id) : 0u;
      atomicAdd(&tiles[hot * 256u + id / (unsigned)T], (u64)rl[t]);
      ++r_in;
    }
  }
  }  // a cut inside a bin
  const u64 cut_c = cut_found;
  unsigned ns = r_in + (tid == 0 ? n_sure : 0u), dz = 0; u64 mx = 0ull, dsum = 0ull;
  blk_reduce<WNW>(S, ns, dz, mx, dsum);  // barriers inside: the tile masses are complete after it
  if (top_k_route && ns != (unsigned)W.top_k) { return false; }  // the passes disagree
  // -- masses of the classes, acceptance (section 5.3), the tile that holds the draw --
  u64 p0 = 0ull, p1 = 0ull;
  for (int i = tid; i < 256; i += WT) { p0 += tiles[i]; p1 += tiles[256 + i]; }
  const u64 S0 = blk_sum_u64<WNW>(S, p0);
  const u64 S1 = blk_sum_u64<WNW>(S, p1);
  const u64 S_K = S0 + S1;
  bool pick_hot = false;
  if (use_hot) {
    pick_hot = (S1 > 0ull) && (u3[1] * (double)S_K <= (double)S1);
    dg.alpha = (double)S1 / (double)S_K;
    dg.flags |= SIMPLE_DIAG_SHVS | (pick_hot ? SIMPLE_DIAG_ACCEPTED : 0u);
  }
  const unsigned cls = pick_hot ? 1u : 0u;
  const u64 S_cls = use_hot ? (pick_hot ? S1 : S0) : S_K;
  const double u = use_hot ? (pick_hot ? u3[0] : u3[2]) : u3[0];
  dg.n_survivors = (int)ns;
  dg.s_k = (double)(top_k_route ? S_K : S_tot) / (double)MSCALE * exp((double)C.y_g - (double)keyf(kmax));
  if (S_cls == 0ull) { return false; }
  u64 tfix = (u64)__double2ull_rd(u * (double)S_cls);
  if (tfix >= S_cls) tfix = S_cls - 1ull;
  {
    const u64 m2 = tiles[cls * 256u + (unsigned)tid];  // WT == 256: one tile per thread
    unsigned ce2, ct2; u64 me2, tot2;
    blk_excl_scan2<WNW>(S, 0u, m2, ce2, me2, ct2, tot2);
    if (m2 > 0ull && me2 <= tfix && me2 + m2 > tfix) { S.bd = tid; S.mab_d = me2; }
  }
  __syncthreads();
  const int tstar = S.bd;
  if (tstar < 0) { return false; }
  // -- the drawn id inside one tile --
  const int c0 = tstar * T;
  float zv[EPT];  // requested before the tables' barriers
#pragma unroll
  for (int e = 0; e < EPT; ++e) { const int idx = c0 + tid * EPT + e; zv[e] = (idx < V) ? Io<DT>::one(rowp + idx) : 0.0f; }
  if (W.h_active) load_slice(Tb, W, a, c0);
  u64 mloc[EPT]; u64 lsum = 0ull;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int idx = c0 + tid * EPT + e;
    mloc[e] = 0ull;
    if (idx < V) {
      float z = zv[e];
      if (W.h_active && slice_bit(idx - c0, Tb)) z = slice_value(z, idx - c0, Tb, W);
      const unsigned hot = use_hot ? hot_bit(hot_bits, (uint32_t)idx) : 0u;
      if (!use_hot || hot == cls) {
        int b; float y;
        const float w = mass_term(z, C, b, y);
        const bool below = z < C.g;
        bool in = !below || b < bstar;
        if (!in && b == bstar) in = composite(fkey(z / W.tau), (uint32_t)idx) >= cut_c;
        if (in && y >= thr_y) mloc[e] = below ? mass_fix_below(w) : mass_fix(w);
      }
    }
    lsum += mloc[e];
  }
  unsigned ce3, ct3; u64 me3, tot3;
  blk_excl_scan2<WNW>(S, 0u, lsum, ce3, me3, ct3, tot3);
  u64 run = S.mab_d + me3;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (mloc[e] > 0ull && run <= tfix && run + mloc[e] > tfix) { S.out_id = c0 + tid * EPT + e; S.out_w = mloc[e]; }
    run += mloc[e];
  }
  __syncthreads();
  dg.p_chosen = (float)((double)S.out_w / (double)S_K);
  return S.out_id >= 0;
}

template <typename DT>
__global__ __launch_bounds__(WT) void wide_finish_kernel(const SampleArgs a) {
  __shared__ SliceTabs Tb;
  __shared__ u64 rcmp[RCAP];
  __shared__ uint32_t rl[RCAP];
  __shared__ u64 dmass[256];
  __shared__ u64 tiles[512];
  __shared__ FS S;
  const int tid = threadIdx.x;
  const unsigned n_wide = min(as_global(a.wq)[a.parity], (unsigned)a.wide_slots);
  for (unsigned slot = blockIdx.x; slot < n_wide; slot += gridDim.x) {
    __syncthreads();
    const WideRow W = load_row(a, slot);
    simple_row_diag dg;
    dg.alpha = __longlong_as_double(0x7FF8000000000000ll);
    dg.s_k = 0.0; dg.p_chosen = 0.0f; dg.n_survivors = 0; dg.reserved = 0u;
    dg.flags = SIMPLE_DIAG_WIDE | W.flags;
    if (a.hot_bits && a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
    const bool ok = finish_row<DT>(a, W, S, Tb, rcmp, rl, dmass, tiles, dg);
    if (tid == 0) {
      if (!ok) hand_on(a, W.row);
      else {
        a.out[W.row] = S.out_id;
        if (a.diag) a.diag[W.row] = dg;
        if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
        write_decision(a, W.row, S.out_id, dg.p_chosen, false);
      }
    }
  }
}

}  // namespace fast


hipError_t launch_wide(const SampleArgs& a, int dtype, hipStream_t st) {
  // One resident round of workgroups each: six (bins) and five (classify) per compute unit fit by
  // registers and LDS; a workgroup then takes a contiguous run of slices, mostly of one row.
  const dim3 bins((unsigned)a.n_cu * 5u), cls((unsigned)a.n_cu * 4u), fin(1024), blk(fast::WT);
  if (dtype == SIMPLE_F32) {
    hipLaunchKernelGGL((fast::wide_bins_kernel<float>), cls, blk, 0, st, a);  // (float32: four workgroups per compute unit, no spilled register)
    if (a.hot_bits) hipLaunchKernelGGL((fast::wide_classify_kernel<float, true>), cls, blk, 0, st, a);
    else hipLaunchKernelGGL((fast::wide_classify_kernel<float, false>), cls, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_finish_kernel<float>), fin, blk, 0, st, a);
  } else {
    hipLaunchKernelGGL((fast::wide_bins_kernel<uint16_t>), bins, blk, 0, st, a);
    if (a.hot_bits) hipLaunchKernelGGL((fast::wide_classify_kernel<uint16_t, true>), cls, blk, 0, st, a);
    else hipLaunchKernelGGL((fast::wide_classify_kernel<uint16_t, false>), cls, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_finish_kernel<uint16_t>), fin, blk, 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace simple
