// Rows whose survivors are not a short prefix that the single-pass kernel's candidate list can hold:
// a nucleus over the whole vocabulary that is wider than the list (top-p over all of V, section 2.1
// Eq. (2)), no truncation at all (every column survives), or a min-p cut below the list's reach.
//
// The single-pass kernel queues such rows with their threshold g.  Their remaining work is two more
// reads of the row, which one workgroup per row would do at the latency of a single compute unit;
// here every queued row is cut into slices of 4096 columns that spread over the whole chip:
//
//   bins      per slice, the penalised, tempered logits below g are binned (bins linear in the
//             tempered logit, 1/64 of a factor two in probability wide) with their masses relative
//             to the mass at g (integers, LDS atomics); the mass at or above g is summed beside
//             them.  This pass points at the bin that holds the cut.
//   classify  that bin follows from the cumulated masses; per tile, the exact (integer) masses of
//             the columns surely inside are summed by class (tail / hot), the columns of the
//             cut's bin are collected, and the exact mass of the whole row is summed.
//   finish    one workgroup per row checks that the cut does lie in the collected bin (else the
//             general kernel takes the row), finds it exactly among those columns by a radix
//             descent over (value, id) weighted by mass, however many of them tie (total order:
//             value descending, id ascending), applies the SHVS acceptance test (section 5.3), walks
//             the per-tile masses of the drawn class in ascending id and reads one tile a last time
//             to locate the drawn id (inverse CDF, step (3) of section 2.1).
//
// Rows without truncation skip the first kernel and have no cut; rows with a min-p cut use the first
// kernel for the row maximum only (the cut is a value).
//
// Penalties (section 2.2) are applied on the fly: the single-pass kernel leaves the row's history
// tables (presence mask, rank directory, counts by rank) in the row's workspace slot, and a slice
// loads its part of them into LDS.  All masses are
// integers, so no result depends on the order of the additions.  A row for which a table overflows
// or the passes disagree is handed to the general kernel.
#include "simple_rowdev.hpp"

namespace simple {
namespace fast {

#ifdef SIMPLE_PHASE_TIMES  // profiling builds only: per-workgroup timestamps of the first kernel (100 MHz wall clock)
__device__ unsigned long long g_wide_phase_times[3 * 8192 * 8];
#define CPHASE(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_wide_phase_times[(16384 + blockIdx.x) * 8 + (i)] = wall_clock64(); } while (0)
#define XPHASE(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_wide_phase_times[(8192 + blockIdx.x) * 8 + (i)] = wall_clock64(); } while (0)
#define XWHY(code, v) do { if (threadIdx.x == 0 && blockIdx.x < 8192) { g_wide_phase_times[(8192 + blockIdx.x) * 8 + 6] = (code); g_wide_phase_times[(8192 + blockIdx.x) * 8 + 7] = (v); } } while (0)
#define WPHASE(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_wide_phase_times[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define WPHASE(i) do { } while (0)
#define XPHASE(i) do { } while (0)
#define CPHASE(i) do { } while (0)
#define XWHY(code, v) do { } while (0)
#endif

constexpr int WT = 256;      // threads per workgroup
constexpr int WNW = WT / 64;
constexpr int SLC = 4096;    // columns per slice
constexpr int ICAP = 1024;   // columns of the boundary bin one slice can stage
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
  W.ws = a.wws + (size_t)slot * a.ws_stride;
  return W;
}

// A slice's part of the row's history tables, in LDS: the mask words of its columns, the
// rank at the start of each of its word pairs (and of the next slice), and the counts of its
// columns, indexed by rank minus the slice's first rank.
struct SliceTabs {
  uint32_t bm[SLC / 32];
  uint32_t dir[SLC / 64 + 2];
  uint16_t cnt[SLC];
};
static_assert(WT == 256, "the finishing kernel maps one tile of each class to a thread");
static_assert(SLC / 32 + SLC / 64 + 1 <= WT, "one mask word or directory entry per thread");
// The tables of the slice that starts at column c0 come in two steps, so that their loads overlap
// with the other loads of an item.  First this thread's mask word or directory entry (the addresses
// follow from the slot alone):
__device__ __forceinline__ uint32_t slice_fetch(const unsigned char* ws, const SampleArgs& a, int c0) {
  const int tid = threadIdx.x;
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
  const int tid = threadIdx.x;
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
// The history columns of a slice, one mask word per thread: f(z', idx) for each, with its penalised
// value.  The streaming loops skip these columns, so their main line carries no table lookups.
template <typename DT, typename F>
__device__ __forceinline__ void for_history_columns(const SliceTabs& T, const WideRow& W, const DT* rowp, int c0, int V, F&& f) {
  const int tid = threadIdx.x;
  if (tid < SLC / 32) {
    uint32_t word = T.bm[tid];
    unsigned r = T.dir[tid >> 1] - T.dir[0] + ((tid & 1) ? (unsigned)__popc(T.bm[tid - 1]) : 0u);
    while (word) {
      const int idx = c0 + 32 * tid + (__ffs((int)word) - 1);
      word &= word - 1u;
      if (idx < V) {
        const float z = apply_penalties(Io<DT>::one(rowp + idx), (uint32_t)T.cnt[min(r, (unsigned)SLC - 1u)], W.rep, W.inv_rep, W.freq, W.pres);
        f(z, idx);
      }
      ++r;
    }
  }
}

// The bin that holds the cut, from the masses of the first pass: cumulative mass from the top
// reaches top_p * total.  bstar < 0 if none.  Ends with a barrier.
__device__ inline int find_cut(FS& S, const WideRow& W) {
  const int tid = threadIdx.x;
  constexpr int BPT = NBW / WT;
  const u64* gh = reinterpret_cast<const u64*>(W.ws + WS_HIST);
  const u64 m_top = as_global(reinterpret_cast<const u64*>(W.ws + WS_SCAL))[0];
  u64 hm[BPT]; u64 loc = 0ull;
#pragma unroll
  for (int j = 0; j < BPT; ++j) { hm[j] = as_global(gh)[tid * BPT + j]; loc += hm[j]; }
  if (tid == 0) S.bk = -1;
  unsigned ce, ct; u64 me, mt;
  blk_excl_scan2<WNW>(S, 0u, loc, ce, me, ct, mt);
  const u64 target = (u64)__double2ull_ru((double)W.top_p * (double)(m_top + mt));
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

// How a column is classified, per route: it surely survives iff its tempered value reaches thr_y and it
// lies at or above g or in a bin before bstar; columns of bin bstar are resolved one by one.
struct RowCut { int bstar; float thr_y; bool valid; };
__device__ inline RowCut row_cut(FS& S, const WideRow& W) {  // every thread calls; barriers inside on one route
  RowCut c;
  c.thr_y = -INFINITY; c.valid = true;
  if (W.mode == WIDE_TOP_P) { c.bstar = find_cut(S, W); c.valid = c.bstar >= 0; }
  else c.bstar = NBW;  // no bin holds a cut
  if (W.mode != WIDE_ALL && W.min_p > 0.0f) {  // min-p, alone or on top of top-p: the shorter prefix wins
    const uint32_t kmax = as_global(reinterpret_cast<const uint32_t*>(W.ws + WS_SCAL))[6];
    c.valid = c.valid && kmax > KEY_NEG_INF;
    c.thr_y = keyf(kmax) + (float)log((double)W.min_p);  // fl(y_max + fl(ln min_p)), as in the list's epilogue
  }
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

// ---------------------------------------------------------------- bins ------------------------
template <typename DT>
__global__ __launch_bounds__(WT, 6) void wide_bins_kernel(const SampleArgs a) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int G = SLC / (WT * EPL);
  typedef typename Io<DT>::Raw Raw;
  __shared__ SliceTabs Tb;
  __shared__ u64 lh[NBW];
  __shared__ FS S;
  const int tid = threadIdx.x;
  const int V = a.V;
  const Items I = my_items(a);
  if (I.i0 >= I.i1) return;
  WPHASE(0);
#ifdef SIMPLE_PHASE_TIMES
  if (threadIdx.x == 0 && blockIdx.x < 8192) { g_wide_phase_times[blockIdx.x * 8 + 5] = __builtin_amdgcn_s_getreg(63492); g_wide_phase_times[blockIdx.x * 8 + 6] = __builtin_amdgcn_s_getreg(63508); }
#endif
  int cur = -1;
  WideRow W;
  u64 mtop = 0ull;
  float ymax = -INFINITY;  // rows with a min-p cut: largest tempered value seen by this thread
  auto flush = [&]() {
    __syncthreads();
    if (W.mode == WIDE_TOP_P) {
      u64* gh = reinterpret_cast<u64*>(W.ws + WS_HIST);
      for (int b = tid; b < NBW; b += WT) { const u64 v = lh[b]; if (v) atomicAdd(&gh[b], v); }
      const u64 t = blk_sum_u64<WNW>(S, mtop);
      if (tid == 0 && t) atomicAdd(reinterpret_cast<u64*>(W.ws + WS_SCAL), t);
    }
    if (W.min_p > 0.0f) {
      const float m = wave_max(ymax);
      if ((tid & 63) == 0 && m > -INFINITY) atomicMax(reinterpret_cast<uint32_t*>(W.ws + WS_SCAL) + 6, fkey(m));
    }
    mtop = 0ull; ymax = -INFINITY;
  };
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    const int c0 = sl * SLC;
    const unsigned char* ws = a.wws + (size_t)slot * a.ws_stride;
    const uint32_t pre = slice_fetch(ws, a, c0);  // in flight while the record arrives
    if (slot != cur) {
      if (cur >= 0) flush();
      W = load_row(a, (unsigned)slot);
      cur = slot;
      for (int b = tid; b < NBW; b += WT) lh[b] = 0ull;
    }
    if (W.mode == WIDE_ALL) continue;  // every column survives: nothing to find in a first pass
    const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
    Raw A[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      if (idx0 + EPL <= V) A[j] = Io<DT>::load(rowp + idx0);
    }
    WPHASE(1);
    slice_store(Tb, pre, a, c0, W.distinct);
    __syncthreads();
    if (W.h_active) slice_counts(Tb, ws, a);
    __syncthreads();
    WPHASE(2);
    auto one = [&](float z, int) {
      if (W.mode == WIDE_MIN_P) { ymax = fmaxf(ymax, tempered(z, W.C)); return; }
      int b; float y;
      const float w = mass_term(z, W.C, b, y);
      ymax = fmaxf(ymax, y);
      if (z < W.C.g) atomicAdd(&lh[b], mass_fix_below(w));
      else mtop += mass_fix(fminf(w, W_LIMIT));
    };
    if (W.h_active) for_history_columns<DT>(Tb, W, rowp, c0, V, one);
    if (W.mode == WIDE_MIN_P) {  // the row maximum is all a value cut needs
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int idx0 = c0 + (j * WT + tid) * EPL;
        if (idx0 + EPL <= V) {
          float z[EPL];
          Io<DT>::unpack(A[j], z);
          const uint32_t nib = W.h_active ? (Tb.bm[(idx0 - c0) >> 5] >> ((unsigned)(idx0 - c0) & 31u)) & ((1u << EPL) - 1u) : 0u;
          float zm = -INFINITY;  // the tempered value is monotone in z: one division per group
#pragma unroll
          for (int e = 0; e < EPL; ++e) zm = ((nib >> e) & 1u) ? zm : fmaxf(zm, z[e]);
          ymax = fmaxf(ymax, tempered(zm, W.C));
        } else {
          for (int idx = idx0; idx < V; ++idx)
            if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
        }
      }
      __syncthreads();
      continue;
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      if (idx0 + EPL <= V) {
        float z[EPL];
        Io<DT>::unpack(A[j], z);
        bool any_top = false;
        if (W.h_active) {  // history columns were handled above: here they count as -inf (no mass)
          const uint32_t nib = (Tb.bm[(idx0 - c0) >> 5] >> ((unsigned)(idx0 - c0) & 31u)) & ((1u << EPL) - 1u);
#pragma unroll
          for (int e = 0; e < EPL; ++e) z[e] = ((nib >> e) & 1u) ? -INFINITY : z[e];
        }
        float zm = -INFINITY;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {  // straight-line: a column at or above g adds zero to its bin
          int b;
          const float w = mass_term(z[e], W.C, b);
          const bool below = z[e] < W.C.g;
          atomicAdd(&lh[b], below ? mass_fix_below(w) : 0ull);
          any_top = any_top || !below;
          zm = fmaxf(zm, z[e]);
        }
        if (W.min_p > 0.0f) ymax = fmaxf(ymax, tempered(zm, W.C));  // the tempered value is monotone in z
        if (__ballot(any_top)) {  // few columns: the 64-bit conversion stays out of the main line
#pragma unroll
          for (int e = 0; e < EPL; ++e)
            if (!(z[e] < W.C.g)) { int b; mtop += mass_fix(fminf(mass_term(z[e], W.C, b), W_LIMIT)); }
        }
      } else {
        for (int idx = idx0; idx < V; ++idx)
          if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
      }
    }
    __syncthreads();  // the tables are reloaded by the next item
    WPHASE(3);
  }
  flush();
  WPHASE(4);
}

// ---------------------------------------------------------------- classify --------------------
template <typename DT, bool use_hot>  // use_hot: a hot set is installed (section 5.3): masses are split by class
__global__ __launch_bounds__(WT, 5) void wide_classify_kernel(const SampleArgs a) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int G = SLC / (WT * EPL);  // 16-byte groups per thread and slice; a slice is one tile of the draw's walk
  constexpr unsigned EMASK = (1u << EPL) - 1u;
  typedef typename Io<DT>::Raw Raw;
  __shared__ SliceTabs Tb;
  __shared__ u64 lrl[ICAP];
  __shared__ u64 ltile[2];
  __shared__ unsigned l_n, l_base;
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63;
  const int V = a.V;
  const Items I = my_items(a);
  if (I.i0 >= I.i1) return;
  const uint32_t* hot_bits = a.hot_bits;
  CPHASE(0);
  int cur = -1;
  WideRow W;
  int bstar = -1;
  float thr_y = -INFINITY;
  bool valid = false;
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    if (slot != cur) {
      W = load_row(a, (unsigned)slot);
      cur = slot;
      const RowCut rc = row_cut(S, W);
      bstar = rc.bstar; thr_y = rc.thr_y; valid = rc.valid;
      CPHASE(1);
    }
    if (!valid) continue;  // the finishing kernel hands the row on
    const int c0 = sl * SLC;
    const uint32_t pre = slice_fetch(W.ws, a, c0);
    const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
    Raw A[G];
    uint32_t hq[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      hq[j] = 0u;
      if (idx0 + EPL <= V) A[j] = Io<DT>::load(rowp + idx0);
      if (use_hot && idx0 < V) hq[j] = (as_global(hot_bits)[idx0 >> 5] >> ((unsigned)idx0 & 31u)) & EMASK;
    }
    if (tid < 2) ltile[tid] = 0ull;
    if (tid == 0) l_n = 0u;
    slice_store(Tb, pre, a, c0, W.distinct);
    __syncthreads();
    if (W.h_active) slice_counts(Tb, W.ws, a);
    __syncthreads();
    CPHASE(2);
    unsigned n_sure = 0u;
    u64 acc_all = 0ull;  // exact mass of every column of the slice
    float ymax = -INFINITY;  // largest tempered value
    bool bad = false;        // a mass the fixed point cannot carry, or a NaN
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
        const unsigned hot = use_hot ? hot_bit(hot_bits, (uint32_t)idx) : 0u;
        atomicAdd(&ltile[hot], m);
        ++n_sure;
      } else if (b == bstar) {
        const unsigned s = atomicAdd(&l_n, 1u);
        if (s < (unsigned)ICAP) lrl[s] = ((u64)__float_as_uint(z) << 32) | (u64)(uint32_t)idx;
      }
    };
    if (W.h_active) for_history_columns<DT>(Tb, W, rowp, c0, V, one);
    CPHASE(3);
    u64 acc0 = 0ull, acc1 = 0ull;
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      if (idx0 + EPL <= V) {
        float z[EPL];
        Io<DT>::unpack(A[j], z);
        bool any_top = false, any_edge = false;
        // history columns were handled above: here they are skipped
        const uint32_t live = W.h_active ? ~((Tb.bm[(idx0 - c0) >> 5] >> ((unsigned)(idx0 - c0) & 31u)) & EMASK) : ~0u;
        uint32_t g0 = 0u, g1 = 0u, gall = 0u;  // group sums: <= 8 masses of <= 2^28
#pragma unroll
        for (int e = 0; e < EPL; ++e) {  // straight-line; the rare cases follow under wave-wide tests
          if (!((live >> e) & 1u)) z[e] = -INFINITY;  // no mass, no bin of interest ...
          int b; float y;
          const float w = mass_term(z[e], W.C, b, y);
          const bool below = z[e] < W.C.g;
          const bool sure = ((live >> e) & 1u) && y >= thr_y && (!below || b < bstar);
          ymax = fmaxf(ymax, y);
          const uint32_t m = below ? (uint32_t)mass_fix_below(w) : 0u;
          const uint32_t ms = sure ? m : 0u;
          const bool hot = use_hot && ((hq[j] >> e) & 1u) != 0u;
          gall += m;
          g0 += hot ? 0u : ms;
          g1 += hot ? ms : 0u;
          n_sure += sure ? 1u : 0u;
          any_top = any_top || !below;
          any_edge = any_edge || (((live >> e) & 1u) && below && b == bstar && y >= thr_y);
        }
        acc0 += (u64)g0; acc1 += (u64)g1; acc_all += (u64)gall;
        if (__ballot(any_top)) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            if (!(z[e] < W.C.g)) {  // not below the list's threshold: inside any top-p nucleus that got here
              int b; float y;
              const float w = mass_term(z[e], W.C, b, y);
              if (!(w <= W_LIMIT)) { bad = true; continue; }
              const u64 m = mass_fix(w);
              acc_all += m;
              if (y >= thr_y) { if (use_hot && ((hq[j] >> e) & 1u)) acc1 += m; else acc0 += m; }
            }
          }
        }
        if (__ballot(any_edge)) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            int b; float y;
            (void)mass_term(z[e], W.C, b, y);
            if (((live >> e) & 1u) && z[e] < W.C.g && b == bstar && y >= thr_y) {
              const unsigned s = atomicAdd(&l_n, 1u);
              if (s < (unsigned)ICAP) lrl[s] = ((u64)__float_as_uint(z[e]) << 32) | (u64)(uint32_t)(idx0 + e);
            }
          }
        }
      } else {
        for (int idx = idx0; idx < V; ++idx)
          if (!(W.h_active && slice_bit(idx - c0, Tb))) one(Io<DT>::one(rowp + idx), idx);
      }
    }
    CPHASE(4);
    {
      const u64 s0 = wave_sum(acc0);
      if (lane == 0 && s0) atomicAdd(&ltile[0], s0);
      if (use_hot) { const u64 s1 = wave_sum(acc1); if (lane == 0 && s1) atomicAdd(&ltile[1], s1); }
    }
    unsigned ns = n_sure, dz = 0u; u64 mx = 0ull, dsum = acc_all;
    blk_reduce<WNW>(S, ns, dz, mx, dsum);  // barriers inside: tile sums and the boundary list are complete
    u64* gt = reinterpret_cast<u64*>(W.ws + WS_TILES);
    uint32_t* sc = reinterpret_cast<uint32_t*>(W.ws + WS_SCAL);
    if (tid < 2 && sl < 256) gt[tid * 256 + sl] = ltile[tid];
    {
      const float m = wave_max(ymax);
      if (lane == 0 && m > -INFINITY) atomicMax(&sc[6], fkey(m));
      if (__ballot(bad) && lane == 0) atomicAdd(&sc[3], (unsigned)RCAP + 1u);  // the finishing kernel hands the row on
    }
    const unsigned nb = l_n;
    if (tid == 0) {
      if (ns) atomicAdd(&sc[2], ns);
      if (dsum) atomicAdd(reinterpret_cast<u64*>(W.ws + WS_SCAL + 16), dsum);
      // more columns of the bin in one slice than the staging list holds: the count is pushed past
      // the limit, so that the finishing kernel hands the row on
      l_base = nb ? atomicAdd(&sc[3], nb > (unsigned)ICAP ? (unsigned)RCAP + 1u : nb) : 0u;
    }
    __syncthreads();
    const unsigned base = l_base;
    for (unsigned t = tid; t < min(nb, (unsigned)ICAP); t += WT)
      if (base + t < (unsigned)RCAP) reinterpret_cast<u64*>(W.ws + WS_RL)[base + t] = lrl[t];
    __syncthreads();
    CPHASE(5);
  }
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
  const u64 S_tot = as_global(reinterpret_cast<const u64*>(W.ws + WS_SCAL))[2];  // exact mass of the row
  u64 tv[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) tv[k] = as_global(reinterpret_cast<const u64*>(W.ws + WS_TILES))[k * WT + tid];
  const uint32_t kmax = as_global(sc)[6];
  XPHASE(0);
  const RowCut rcut = row_cut(S, W);
  const int bstar = rcut.bstar;
  const float thr_y = rcut.thr_y;
  XPHASE(1);
  if (!rcut.valid) { XWHY(1, 0); return false; }
  const bool top_p_route = W.mode == WIDE_TOP_P;
  // a count past the limit is also how the classifying pass reports a row it could not handle; no
  // collected column on the top-p route means that a min-p cut ended the survivors above the bin
  const bool minp_too = top_p_route && W.min_p > 0.0f;
  if (n_r > (unsigned)RCAP || (!top_p_route && n_r != 0u) || (top_p_route && n_r == 0u && !minp_too)) { XWHY(2, n_r); return false; }
  if (tid == 0) { S.bd = -1; S.cut_k = 0ull; S.cut_p = ~0ull; S.out_id = -1; S.out_w = 0ull; }
  tiles[tid] = tv[0]; tiles[WT + tid] = tv[1];
  const u64 msure = tv[0] + tv[1];
  u64 cut_found = 0ull;  // every collected column at or after it in the order survives; 0: no collected columns
  unsigned r_in = 0;
  if (top_p_route && n_r == 0u) cut_found = ~0ull;  // nothing of the bin survives
  if (top_p_route && n_r != 0u) {
  // exact masses from here: the columns surely inside must stay below the target, the collected bin must reach it
  const u64 m_above = blk_sum_u64<WNW>(S, msure);  // barriers inside
  const u64 target = (u64)__double2ull_ru((double)W.top_p * (double)S_tot);
  if (m_above >= target) { XWHY(3, 0); return false; }
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
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const u64 hi = __shfl_xor(cmax_t, o, 64), lo = __shfl_xor(cmin_t, o, 64);
      cmax_t = (hi > cmax_t) ? hi : cmax_t; cmin_t = (lo < cmin_t) ? lo : cmin_t;
    }
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
        if ((c & mask) == prefix) atomicAdd(&dmass[(unsigned)(c >> shift) & 0xFFu], (u64)rl[t]);
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
    if (differ == 0ull && m_above + (u64)rl[0] < target) ok = false;  // a single column, and it does not reach the target
    // the collected columns do not reach the target: with a min-p cut those below it were never
    // collected, and the min-p prefix is the shorter one (all collected columns survive)
    if (!ok && !minp_too) { XWHY(4, 0); return false; }
    cut_found = ok ? prefix : 1ull;
  }
  XPHASE(2);
  if (cut_found == 0ull) { XWHY(6, 0); return false; }
  for (unsigned t = tid; t < n_r; t += WT) {
    if (rcmp[t] >= cut_found) {
      const uint32_t id = 0xFFFFFFFFu - (uint32_t)rcmp[t];
      const unsigned hot = use_hot ? hot_bit(hot_bits, id) : 0u;
      atomicAdd(&tiles[hot * 256u + id / (unsigned)T], (u64)rl[t]);
      ++r_in;
    }
  }
  }  // top-p route
  const u64 cut_c = cut_found;
  unsigned ns = r_in + (tid == 0 ? n_sure : 0u), dz = 0; u64 mx = 0ull, dsum = 0ull;
  blk_reduce<WNW>(S, ns, dz, mx, dsum);  // barriers inside: the tile masses are complete after it
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
  dg.s_k = (double)S_tot / (double)MSCALE * exp((double)C.y_g - (double)keyf(kmax));
  if (S_cls == 0ull) { XWHY(7, 0); return false; }
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
  XPHASE(3);
  if (tstar < 0) { XWHY(8, 0); return false; }
  // -- the drawn id inside one tile --
  const int c0 = tstar * T;
  float zv[EPT];  // requested before the tables' barriers
#pragma unroll
  for (int e = 0; e < EPT; ++e) { const int idx = c0 + tid * EPT + e; zv[e] = (idx < V) ? Io<DT>::one(rowp + idx) : 0.0f; }
  if (W.h_active) load_slice(Tb, W, a, c0);
  XPHASE(4);
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
  XPHASE(5);
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
      }
    }
  }
}

}  // namespace fast

#ifdef SIMPLE_PHASE_TIMES
extern "C" int simple_debug_wide_phase_times(unsigned long long* dst_host, int n) {
  return (int)hipMemcpyFromSymbol(dst_host, HIP_SYMBOL(simple::fast::g_wide_phase_times), sizeof(unsigned long long) * 8 * (size_t)n);  // n <= 3 * 8192
}
#endif

hipError_t launch_wide(const SampleArgs& a, int dtype, hipStream_t st) {
  // One resident round of workgroups each: six (bins) and five (classify) per compute unit fit by
  // registers and LDS; a workgroup then takes a contiguous run of slices, mostly of one row.
  const dim3 bins((unsigned)a.n_cu * 6u), cls((unsigned)a.n_cu * 5u), fin(1024), blk(fast::WT);
  if (dtype == SIMPLE_F32) {
    hipLaunchKernelGGL((fast::wide_bins_kernel<float>), bins, blk, 0, st, a);
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
