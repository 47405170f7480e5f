// Whole-vocabulary nucleus wider than the candidate list (top-p over all of V, section 2.1 Eq. (2)).
//
// The single-pass kernel queues such rows with their threshold g.  Their remaining work is two more
// reads of the row, which one workgroup per row would do at the latency of a single compute unit;
// here every queued row is cut into slices of 4096 columns that spread over the whole chip:
//
//   bins      per slice, the penalised, tempered logits below g are binned (bins linear in the
//             tempered logit, 1/32 of a factor two in probability wide) with their masses relative
//             to the mass at g, as integers; the mass at or above g is summed beside them.
//   classify  the bin that holds the cut follows from the cumulated masses; per tile, the masses of
//             the columns surely inside are summed by class (tail / hot), and the columns of the
//             cut's bin are collected.
//   finish    one workgroup per row finds the cut exactly among the collected columns (total order:
//             value descending, id ascending), applies the SHVS acceptance test (section 5.3), walks
//             the per-tile masses of the drawn class in ascending id and reads one tile a last time
//             to locate the drawn id (inverse CDF, step (3) of section 2.1).
//
// Penalties (section 2.2) are applied on the fly: the single-pass kernel leaves the row's history
// tables (presence mask, rank directory, counts by rank) in the row's workspace slot, and a slice
// loads its part of them into LDS.  All masses are
// integers, so no result depends on the order of the additions.  A row for which a table overflows
// or the passes disagree is handed to the general kernel.
#include "simple_rowdev.hpp"

namespace simple {
namespace fast {

constexpr int WT = 256;      // threads per workgroup
constexpr int WNW = WT / 64;
constexpr int SLC = 4096;    // columns per slice
static_assert(WS_HT == WIDE_SLOT_FIXED, "workspace slot size");
static_assert(sizeof(WideRec) == 64, "queue record size");

// Per-row constants of a queued row, identical in every thread.
struct WideRow {
  int row;
  StreamCtx C;
  float tau, top_p;
  uint32_t kmax, flags;
  bool h_active;
  float rep, freq, pres;
  double inv_rep;
  uint32_t distinct;
  unsigned char* ws;
};

__device__ __forceinline__ WideRow load_row(const SampleArgs& a, unsigned slot) {
  WideRow W;
  const WideRec rec = reinterpret_cast<const WideRec*>(a.wq + WQ_HEAD)[slot];
  W.row = (int)rec.row; W.kmax = rec.kmax; W.flags = rec.flags;
  W.tau = rec.tau; W.top_p = rec.top_p;
  W.C.g = rec.g; W.C.y_g = rec.g / rec.tau; W.C.inv_tau = 1.0 / (double)rec.tau; W.C.need_sum = true;
  W.C.l2e_tau = 0.0f;
  W.rep = rec.rep; W.freq = rec.freq; W.pres = rec.pres;
  W.inv_rep = 1.0 / (double)rec.rep;
  W.h_active = rec.h_active != 0;
  W.distinct = rec.distinct;
  W.ws = a.wws + (size_t)slot * a.ws_stride;
  return W;
}

// A slice's part of the row's history tables, in LDS: the 128 mask words of its 4096 columns, the
// rank at the start of each of its 64 word pairs (and of the next slice), and the counts of its
// columns, indexed by rank minus the slice's first rank.
struct SliceTabs {
  uint32_t bm[SLC / 32];
  uint32_t dir[SLC / 64 + 2];
  uint16_t cnt[SLC];
};
// Loads the tables of the slice that starts at column c0.  Two barriers; ends with one.
__device__ inline void load_slice(SliceTabs& T, const WideRow& W, const SampleArgs& a, int c0) {
  const int tid = threadIdx.x;
  const unsigned char* ht = W.ws + WS_HT;
  const uint32_t* gbm = reinterpret_cast<const uint32_t*>(ht);
  const uint16_t* gdir = reinterpret_cast<const uint16_t*>(ht + a.F.dir);
  const uint16_t* gcnt = reinterpret_cast<const uint16_t*>(ht + a.F.cnt);
  const int n_pairs = (((a.V + 31) >> 5) + 1) >> 1;  // the mask is stored in whole pairs of words
  const int w0 = c0 >> 5, p0 = c0 >> 6;
  if (tid < SLC / 32) T.bm[tid] = (w0 + tid < 2 * n_pairs) ? as_global(gbm)[w0 + tid] : 0u;
  else if (tid < SLC / 32 + SLC / 64 + 1) {
    const int j = tid - SLC / 32;
    T.dir[j] = (p0 + j < n_pairs) ? (uint32_t)as_global(gdir)[p0 + j] : W.distinct;
  }
  __syncthreads();
  const unsigned r0 = T.dir[0];
  const unsigned nc = min(T.dir[SLC / 64] - r0, (unsigned)SLC);
  for (unsigned t = tid; t < nc; t += WT) T.cnt[t] = as_global(gcnt)[r0 + t];
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

// The bin that holds the cut: cumulative mass from the top reaches top_p * total.  bstar < 0 if none.
__device__ inline void find_cut(FS& S, const WideRow& W, int& bstar, u64& m_above, u64& target, u64& S_tot, unsigned& in_bin) {
  const int tid = threadIdx.x;
  constexpr int BPT = NBW / WT;
  const u64* gh = reinterpret_cast<const u64*>(W.ws + WS_HIST);
  const u64 m_top = *reinterpret_cast<const u64*>(W.ws + WS_SCAL);
  u64 hm[BPT]; unsigned hc[BPT]; u64 loc = 0ull;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    const u64 e = as_global(gh)[tid * BPT + j];
    hm[j] = e & ((1ull << 46) - 1ull); hc[j] = (unsigned)(e >> 46); loc += hm[j];
  }
  if (tid == 0) { S.bk = -1; S.mab_k = 0ull; S.need_k = 0u; }
  unsigned ce, ct; u64 me, mt;
  blk_excl_scan2<WNW>(S, 0u, loc, ce, me, ct, mt);
  S_tot = m_top + mt;
  target = (u64)__double2ull_ru((double)W.top_p * (double)S_tot);
  u64 run = m_top + me;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    if (run < target && run + hm[j] >= target) { S.bk = tid * BPT + j; S.mab_k = run; S.need_k = hc[j]; }
    run += hm[j];
  }
  __syncthreads();
  bstar = S.bk; m_above = S.mab_k; in_bin = S.need_k;
  __syncthreads();
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
__global__ __launch_bounds__(WT) void wide_bins_kernel(const SampleArgs a) {
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
  int cur = -1;
  WideRow W;
  u64 mtop = 0ull;
  auto flush = [&]() {
    __syncthreads();
    u64* gh = reinterpret_cast<u64*>(W.ws + WS_HIST);
    for (int b = tid; b < NBW; b += WT) { const u64 v = lh[b]; if (v) atomicAdd(&gh[b], v); }
    const u64 t = blk_sum_u64<WNW>(S, mtop);
    if (tid == 0 && t) atomicAdd(reinterpret_cast<u64*>(W.ws + WS_SCAL), t);
    mtop = 0ull;
  };
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    if (slot != cur) {
      if (cur >= 0) flush();
      W = load_row(a, (unsigned)slot);
      cur = slot;
      __syncthreads();
      for (int b = tid; b < NBW; b += WT) lh[b] = 0ull;
      __syncthreads();
    }
    const int c0 = sl * SLC;
    const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
    Raw A[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      if (idx0 + EPL <= V) A[j] = Io<DT>::load(rowp + idx0);
    }
    if (W.h_active) load_slice(Tb, W, a, c0);
    auto one = [&](float z, int idx) {
      if (W.h_active && slice_bit(idx - c0, Tb)) z = slice_value(z, idx - c0, Tb, W);
      int b;
      const float w = mass_term(z, W.C, b);
      if (z < W.C.g) { if (z > -INFINITY) atomicAdd(&lh[b], hist_entry(w)); }
      else mtop += mass_fix(w);
    };
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      if (idx0 + EPL <= V) {
        float z[EPL];
        Io<DT>::unpack(A[j], z);
        bool any_top = false;
        if (W.h_active) {
          const uint32_t nib = (Tb.bm[(idx0 - c0) >> 5] >> ((unsigned)(idx0 - c0) & 31u)) & ((1u << EPL) - 1u);
          if (nib) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) if ((nib >> e) & 1u) z[e] = slice_value(z[e], idx0 - c0 + e, Tb, W);
          }
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) {  // straight-line: a column at or above g adds zero to its bin
          int b;
          const float w = mass_term(z[e], W.C, b);
          const bool below = z[e] < W.C.g;
          atomicAdd(&lh[b], (below && z[e] > -INFINITY) ? hist_entry(w) : 0ull);
          any_top = any_top || !below;
        }
        if (__ballot(any_top)) {  // few columns: the 64-bit conversion stays out of the main line
#pragma unroll
          for (int e = 0; e < EPL; ++e)
            if (!(z[e] < W.C.g)) { int b; mtop += mass_fix(mass_term(z[e], W.C, b)); }
        }
      } else {
        for (int idx = idx0; idx < V; ++idx) one(Io<DT>::one(rowp + idx), idx);
      }
    }
    __syncthreads();  // the tables are reloaded by the next item
  }
  flush();
}

// ---------------------------------------------------------------- classify --------------------
template <typename DT>
__global__ __launch_bounds__(WT) void wide_classify_kernel(const SampleArgs a) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int G = SLC / (WT * EPL);  // tiles per slice: one 16-byte group per thread covers a tile
  constexpr int T = WT * EPL;
  constexpr unsigned EMASK = (1u << EPL) - 1u;
  typedef typename Io<DT>::Raw Raw;
  __shared__ SliceTabs Tb;
  __shared__ u64 lrl[RCAP];
  __shared__ u64 ltile[2 * G];
  __shared__ unsigned l_n, l_base;
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63;
  const int V = a.V;
  const Items I = my_items(a);
  if (I.i0 >= I.i1) return;
  const uint32_t* hot_bits = a.hot_bits;
  const bool use_hot = hot_bits != nullptr;
  int cur = -1;
  WideRow W;
  int bstar = -1;
  bool valid = false;
  for (unsigned it = I.i0; it < I.i1; ++it) {
    const int slot = (int)(it / I.n_sl), sl = (int)(it % I.n_sl);
    if (slot != cur) {
      W = load_row(a, (unsigned)slot);
      cur = slot;
      u64 m_above, target, S_tot; unsigned in_bin;
      find_cut(S, W, bstar, m_above, target, S_tot, in_bin);
      valid = bstar >= 0 && in_bin <= (unsigned)RCAP;
    }
    if (!valid) continue;  // the finishing kernel hands the row on
    const int c0 = sl * SLC;
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
    if (tid < 2 * G) ltile[tid] = 0ull;
    if (tid == 0) l_n = 0u;
    if (W.h_active) load_slice(Tb, W, a, c0); else __syncthreads();
    unsigned n_sure = 0u;
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int idx0 = c0 + (j * WT + tid) * EPL;
      u64 acc0 = 0ull, acc1 = 0ull;
      auto one = [&](float z, int idx, bool hot) {
        if (W.h_active && slice_bit(idx - c0, Tb)) z = slice_value(z, idx - c0, Tb, W);
        int b;
        const float w = mass_term(z, W.C, b);
        const bool below = z < W.C.g;
        if (!below || b < bstar) {
          const u64 m = below ? mass_fix_below(w) : mass_fix(w);
          if (hot) acc1 += m; else acc0 += m;
          ++n_sure;
        } else if (b == bstar) {
          const unsigned s = atomicAdd(&l_n, 1u);
          if (s < (unsigned)RCAP) lrl[s] = ((u64)__float_as_uint(z) << 32) | (u64)(uint32_t)idx;
        }
      };
      if (idx0 + EPL <= V) {
        float z[EPL];
        Io<DT>::unpack(A[j], z);
        bool any_top = false, any_edge = false;
        if (W.h_active) {
          const uint32_t nib = (Tb.bm[(idx0 - c0) >> 5] >> ((unsigned)(idx0 - c0) & 31u)) & EMASK;
          if (nib) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) if ((nib >> e) & 1u) z[e] = slice_value(z[e], idx0 - c0 + e, Tb, W);
          }
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) {  // straight-line; the rare cases follow under wave-wide tests
          int b;
          const float w = mass_term(z[e], W.C, b);
          const bool below = z[e] < W.C.g;
          const bool sure = !below || b < bstar;
          const u64 m = (sure && below) ? mass_fix_below(w) : 0ull;
          const bool hot = ((hq[j] >> e) & 1u) != 0u;
          acc0 += hot ? 0ull : m;
          acc1 += hot ? m : 0ull;
          n_sure += sure ? 1u : 0u;
          any_top = any_top || !below;
          any_edge = any_edge || (below && b == bstar);
        }
        if (__ballot(any_top)) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            if (!(z[e] < W.C.g)) {
              int b;
              const u64 m = mass_fix(mass_term(z[e], W.C, b));
              if ((hq[j] >> e) & 1u) acc1 += m; else acc0 += m;
            }
          }
        }
        if (__ballot(any_edge)) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            int b;
            (void)mass_term(z[e], W.C, b);
            if (z[e] < W.C.g && b == bstar) {
              const unsigned s = atomicAdd(&l_n, 1u);
              if (s < (unsigned)RCAP) lrl[s] = ((u64)__float_as_uint(z[e]) << 32) | (u64)(uint32_t)(idx0 + e);
            }
          }
        }
      } else {
        for (int idx = idx0; idx < V; ++idx) one(Io<DT>::one(rowp + idx), idx, (hq[j] >> (idx - idx0)) & 1u);
      }
      const u64 s0 = wave_sum(acc0), s1 = wave_sum(acc1);
      if (lane == 0) { if (s0) atomicAdd(&ltile[j], s0); if (s1) atomicAdd(&ltile[G + j], s1); }
    }
    unsigned ns = n_sure, dz = 0u; u64 mx = 0ull, dsum = 0ull;
    blk_reduce<WNW>(S, ns, dz, mx, dsum);  // barriers inside: tile sums and the boundary list are complete
    u64* gt = reinterpret_cast<u64*>(W.ws + WS_TILES);
    uint32_t* sc = reinterpret_cast<uint32_t*>(W.ws + WS_SCAL);
    if (tid < 2 * G) {
      const int tile = c0 / T + (tid % G);
      if (tile < 256) gt[(tid / G) * 256 + tile] = ltile[tid];
    }
    const unsigned nb = l_n;
    if (tid == 0) {
      if (ns) atomicAdd(&sc[2], ns);
      l_base = nb ? atomicAdd(&sc[3], nb) : 0u;
    }
    __syncthreads();
    const unsigned base = l_base;
    for (unsigned t = tid; t < min(nb, (unsigned)RCAP); t += WT)
      if (base + t < (unsigned)RCAP) reinterpret_cast<u64*>(W.ws + WS_RL)[base + t] = lrl[t];
    __syncthreads();
  }
}

// ---------------------------------------------------------------- finish ----------------------
__device__ inline void hand_on(const SampleArgs& a, int row) {
  const unsigned slot = atomicAdd(&a.pend[a.parity], 1u);
  a.pend[2 + slot] = (uint32_t)row;
  a.out[row] = PENDING;
}

template <typename DT>
__device__ inline bool finish_row(const SampleArgs& a, const WideRow& W, FS& S, SliceTabs& Tb, u64* rcmp, u64* rl,
                                  uint32_t* fcnt, u64* fmass, u64* mc, u64* mw, u64* tiles, simple_row_diag& dg) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int T = WT * EPL;
  const int tid = threadIdx.x;
  const int V = a.V;
  const StreamCtx& C = W.C;
  const uint32_t* hot_bits = a.hot_bits;
  const bool use_hot = hot_bits != nullptr;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)W.row * (size_t)a.stride;
  double u3[3];
  row_uniforms(a.seed, a.row_offset + (uint64_t)W.row, a.step, u3);
  int bstar; u64 m_above, target, S_tot; unsigned in_bin;
  find_cut(S, W, bstar, m_above, target, S_tot, in_bin);
  if (bstar < 0 || in_bin > (unsigned)RCAP) return false;
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(W.ws + WS_SCAL);
  const unsigned n_sure = as_global(sc)[2], n_r = as_global(sc)[3];
  if (n_r > (unsigned)RCAP || n_r == 0u) return false;
  if (tid == 0) { S.n2 = 0u; S.cut_k = 0ull; S.bd = -1; S.bp = -1; S.kmax = 0u; S.nunc = 0xFFFFFFFFu; S.out_id = -1; S.out_w = 0ull; }
  for (int i = tid; i < 512; i += WT) tiles[i] = as_global(reinterpret_cast<const u64*>(W.ws + WS_TILES))[i];
  for (int i = tid; i < NBF; i += WT) { fcnt[i] = 0u; fmass[i] = 0ull; }
  __syncthreads();
  // -- the boundary bin, exactly: shortest prefix in the total order whose mass reaches the target --
  for (unsigned t = tid; t < n_r; t += WT) {
    const u64 e = as_global(reinterpret_cast<const u64*>(W.ws + WS_RL))[t];
    const float z = __uint_as_float((uint32_t)(e >> 32));
    int b;
    const float w = mass_term(z, C, b);
    const uint32_t key = fkey(z / W.tau);
    rcmp[t] = composite(key, (uint32_t)e);
    rl[t] = mass_fix_below(w);
    atomicMax(&S.kmax, key);
    atomicMin(&S.nunc, key);
  }
  __syncthreads();
  const uint32_t kmx = S.kmax, kmn = S.nunc;
  const float y_hi = keyf(kmx);
  const float sscale = (float)NBF / fmaxf(y_hi - keyf(kmn), 1e-30f);
  auto sub_bin = [&](u64 c) { return (unsigned)min((int)((y_hi - keyf((uint32_t)(c >> 32))) * sscale), NBF - 1); };
  for (unsigned t = tid; t < n_r; t += WT) {
    const unsigned sb = sub_bin(rcmp[t]);
    atomicAdd(&fcnt[sb], 1u);
    atomicAdd(&fmass[sb], rl[t]);
  }
  __syncthreads();
  {
    const u64 m2 = (tid < NBF) ? fmass[tid] : 0ull;
    unsigned ce2, ct2; u64 me2, mt2;
    blk_excl_scan2<WNW>(S, 0u, m2, ce2, me2, ct2, mt2);
    if (tid < NBF && m2 > 0ull && m_above + me2 < target && m_above + me2 + m2 >= target) { S.bp = tid; S.mab_p = m_above + me2; }
  }
  __syncthreads();
  const int sbp = S.bp;
  if (sbp < 0) return false;  // the masses of the passes disagree
  for (unsigned t = tid; t < n_r; t += WT) {
    if ((int)sub_bin(rcmp[t]) == sbp) {
      const unsigned s = atomicAdd(&S.n2, 1u);
      if (s < (unsigned)MEMB2) { mc[s] = rcmp[t]; mw[s] = rl[t]; }
    }
  }
  __syncthreads();
  const unsigned nm = S.n2;
  if (nm > (unsigned)MEMB2) return false;
  {
    const u64 mab = S.mab_p;
    for (unsigned mi = tid; mi < nm; mi += WT) {
      const u64 cm = mc[mi], wm = mw[mi];
      u64 Gm = mab;
      for (unsigned q = 0; q < nm; ++q) Gm += (mc[q] >= cm) ? mw[q] : 0ull;
      if (Gm >= target && Gm - wm < target) S.cut_k = cm;
    }
  }
  __syncthreads();
  const u64 cut_c = S.cut_k;
  if (cut_c == 0ull) return false;
  unsigned r_in = 0;
  for (unsigned t = tid; t < n_r; t += WT) {
    if (rcmp[t] >= cut_c) {
      const uint32_t id = 0xFFFFFFFFu - (uint32_t)rcmp[t];
      const unsigned hot = use_hot ? hot_bit(hot_bits, id) : 0u;
      atomicAdd(&tiles[hot * 256u + id / (unsigned)T], rl[t]);
      ++r_in;
    }
  }
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
  dg.s_k = (double)S_tot / (double)MSCALE * exp((double)C.y_g - (double)keyf(W.kmax));
  if (S_cls == 0ull) return false;
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
  if (tstar < 0) return false;
  // -- the drawn id inside one tile --
  const int c0 = (tstar * T / SLC) * SLC;
  if (W.h_active) load_slice(Tb, W, a, c0);
  u64 mloc[EPL]; u64 lsum = 0ull;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int idx = tstar * T + tid * EPL + e;
    mloc[e] = 0ull;
    if (idx < V) {
      float z = Io<DT>::one(rowp + idx);
      if (W.h_active && slice_bit(idx - c0, Tb)) z = slice_value(z, idx - c0, Tb, W);
      const unsigned hot = use_hot ? hot_bit(hot_bits, (uint32_t)idx) : 0u;
      if (!use_hot || hot == cls) {
        int b;
        const float w = mass_term(z, C, b);
        const bool below = z < C.g;
        bool in = !below || b < bstar;
        if (!in && b == bstar) in = composite(fkey(z / W.tau), (uint32_t)idx) >= cut_c;
        if (in) mloc[e] = below ? mass_fix_below(w) : mass_fix(w);
      }
    }
    lsum += mloc[e];
  }
  unsigned ce3, ct3; u64 me3, tot3;
  blk_excl_scan2<WNW>(S, 0u, lsum, ce3, me3, ct3, tot3);
  u64 run = S.mab_d + me3;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    if (mloc[e] > 0ull && run <= tfix && run + mloc[e] > tfix) { S.out_id = tstar * T + tid * EPL + e; S.out_w = mloc[e]; }
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
  __shared__ u64 rl[RCAP];
  __shared__ uint32_t fcnt[NBF];
  __shared__ u64 fmass[NBF];
  __shared__ u64 mc[MEMB2];
  __shared__ u64 mw[MEMB2];
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
    const bool ok = finish_row<DT>(a, W, S, Tb, rcmp, rl, fcnt, fmass, mc, mw, tiles, dg);
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

hipError_t launch_wide(const SampleArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(4096), fin(1024), blk(fast::WT);
  if (dtype == SIMPLE_F32) {
    hipLaunchKernelGGL((fast::wide_bins_kernel<float>), grid, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_classify_kernel<float>), grid, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_finish_kernel<float>), fin, blk, 0, st, a);
  } else {
    hipLaunchKernelGGL((fast::wide_bins_kernel<uint16_t>), grid, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_classify_kernel<uint16_t>), grid, blk, 0, st, a);
    hipLaunchKernelGGL((fast::wide_finish_kernel<uint16_t>), fin, blk, 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace simple
