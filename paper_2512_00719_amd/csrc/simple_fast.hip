// Single-pass row kernel for gfx950: one workgroup per logits row, every logit read from HBM once.
//
// A row needs little LDS (one region is shared in time between the history tables and the
// candidate list), so four row workgroups fit a compute unit and their latency-bound phases
// overlap with the streaming of the others.
//
//   history   the row's token history becomes, in LDS, a presence bit per column, a 16-bit count
//             of set bits before each pair of mask words and 16-bit generated-token counts indexed
//             by the rank of the id among the set bits.  The V-wide histograms of section 2.2 are
//             never materialised; a column's penalty is looked up only where its bit is set, so
//             unpenalised columns are never touched (column-wise penalties, section 5.2).
//   sample    every wave's first two tiles (history columns masked) give, by wave-ballot bisection, a
//             value g that is expected to admit a small multiple of the requested prefix length.
//   stream    one coalesced pass of 16-byte loads per lane over the raw logits.  Columns with
//             z >= g go to an LDS candidate list that now occupies the history's region (penalties
//             that only lower a logit keep z >= z', so nothing with z' >= g is missed); rows whose
//             nucleus is taken over the whole vocabulary also accumulate exp((z - g) / tau) below g.
//   epilogue  the list moves to registers, the history tables are rebuilt in the region and the
//             listed columns are penalised; the mass below g is corrected, exactly, for the
//             history columns.  The list then certifies itself: every column whose tempered value
//             exceeds fl(g / tau) is in it, so any prefix of the total order (value descending, id
//             ascending) that ends above that value is known exactly (truncation first, section
//             5.2).  Top-k, top-p and min-p cuts, the survivors' mass and the inverse-CDF draw
//             (Eq. (2), step (3)) use integer (fixed-point) masses, so no result depends on the
//             order in which waves appended candidates.  SHVS (section 5.3): acceptance test on the
//             hot mass, then the draw walks the hot or the tail survivors only.
// A row whose nucleus over the whole vocabulary is wider than the list is queued, with its threshold
// and its history tables, for the sliced kernels that run next on the stream.  Rows the kernel
// cannot certify (threshold missed, list overflow, ties wider than a table, penalties that raise
// logits, parameter errors) are queued for the general kernel, which runs last.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "simple_rowdev.hpp"

namespace simple {
namespace fast {



// A key t with need <= #{keys >= t} among the 64 x N keys held by a wave (N per lane), found by
// bisection between lo and hi with wave ballots; no LDS, no barrier.  Stops as soon as the count is
// within need + slack, else converges to the need-th largest key.  Requires #{keys >= lo} >= need
// and hi >= every key; returns lo unchanged if the interval is empty.
template <int N>
__device__ __forceinline__ uint32_t wave_threshold(const uint32_t (&k)[N], unsigned need, unsigned slack, uint32_t lo, uint32_t hi) {
#pragma unroll 1
  for (int it = 0; it < 34 && lo < hi; ++it) {
    const uint32_t mid = lo + ((hi - lo + 1u) >> 1);
    unsigned c = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) c += (unsigned)__popcll(__ballot(k[j] >= mid));
    if (c >= need) { lo = mid; if (c <= need + slack) break; } else hi = mid - 1u;
  }
  return lo;
}

// Fixed-point weight exp(y - y_max) * 2^44 (stable softmax numerator, section 2.1 Eq. (2)).  The
// exponential is float32 with a split log2(e): relative error about 1e-7, far inside the 1e-5
// tolerance on probabilities; the sums are exact integers.
__device__ __forceinline__ u64 wfix(uint32_t key, float y_max) {
  const float d = keyf(key) - y_max;
  const float t = fmaf(d, L2E_HI, d * L2E_LO);
  return float_to_u64(__builtin_amdgcn_exp2f(t) * 0x1p44f);  // the scaling is exact
}

// Unpacks one 16-byte group of a sample tile; columns that are in the history are masked out, so
// the threshold comes from unpenalised columns only (history columns can only add to the prefix).
template <typename DT>
__device__ __forceinline__ void sample_group(const typename Io<DT>::Raw& A, int idx0, const Hist& H, float (&z)[Io<DT>::EPL]) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr unsigned EMASK = (1u << EPL) - 1u;
  Io<DT>::unpack(A, z);
  if (H.active) {
    const uint32_t nib = (H.bm[idx0 >> 5] >> ((unsigned)idx0 & 31u)) & EMASK;
#pragma unroll
    for (int e = 0; e < EPL; ++e) z[e] = (nib & (1u << e)) ? -INFINITY : z[e];
  }
}

// Appends the flagged elements of one 16-byte group per lane with a single list reservation.
// m[e]: the wave's ballot of "element e is at or above g".
template <int EPL>
__device__ __forceinline__ void append_group(FS& S, uint32_t* lz, uint32_t* li, unsigned cap, const float (&z)[EPL], float g,
                                             const u64 (&m)[EPL], int idx0) {
  const int lane = lane_id();
  unsigned pre[EPL], tot = 0;
#pragma unroll
  for (int e = 0; e < EPL; ++e) { pre[e] = tot; tot += (unsigned)__popcll(m[e]); }
  unsigned base = 0;
  if (lane == 0) base = atomicAdd(&S.cand_count, tot);
  base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    if (!(z[e] < g)) {  // the lanes of m[e]
      const unsigned slot = base + pre[e] + lanes_before(m[e]);
      if (slot < cap) { lz[slot] = __float_as_uint(z[e]); li[slot] = (uint32_t)(idx0 + e); }
    }
  }
}

// One tile of the stream: raw logits against g; rows that need it also sum the mass below g (per lane).
template <typename DT>
__device__ __forceinline__ void stream_tile(const typename Io<DT>::Raw (&A)[UNR], int tb, const StreamCtx& C,
                                            FS& S, uint32_t* lz, uint32_t* li, unsigned cap, u64& below_mass) {
  constexpr int EPL = Io<DT>::EPL;
  const int lane = lane_id();
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
    float z[EPL];
    Io<DT>::unpack(A[u], z);
    const int idx0 = tb + u * 64 * EPL + lane * EPL;
    if (C.need_sum) {
      uint32_t grp = 0u;  // straight-line: a column at or above g adds 2^28 (taken off after the stream); <= 8 terms
#pragma unroll
      for (int e = 0; e < EPL; ++e) grp += below_term_clamped(z[e], C);
      below_mass += (u64)grp;
    }
    u64 m[EPL], any = 0ull;  // one compare per element, straight into the wave's mask; the rest is scalar
#pragma unroll
    for (int e = 0; e < EPL; ++e) { m[e] = __ballot(!(z[e] < C.g)); any |= m[e]; }
    if (any) append_group<EPL>(S, lz, li, cap, z, C.g, m, idx0);
  }
}

// ---------------------------------------------------------------- epilogue --------------------
enum { FIN_DONE = 0, FIN_PENDING = 1, FIN_WIDE = 2 };

__device__ __forceinline__ u64 pick8(const u64 (&a)[8], int j) {
  u64 v = 0ull;
#pragma unroll
  for (int i = 0; i < 8; ++i) v = (i == j) ? a[i] : v;
  return v;
}

// Mass of the top-k prefix when top-k is off: the whole row (list, uncertified entries, below g).
__device__ __forceinline__ u64 whole_row_mass(u64 total_m, unsigned n_unc, uint32_t key_g, float y_max, float g, float tau,
                                              double S_below) {
  (void)g; (void)tau;
  const double f0 = exp((double)keyf(key_g) - (double)y_max);  // S_below is relative to the mass at y_g
  return total_m + (u64)n_unc * wfix(key_g, y_max) + (u64)__double2ull_rn(S_below * f0 * WSCALE);
}

// Survivors, masses and the draw for at most MEMB certified entries (the usual case).  The entries
// arrive as composites in mc[0, n); they are ranked by counting, laid out in sorted order and one
// wave takes every decision of Eq. (2) on that order; then all threads locate the drawn id.
template <int NTHR>
__device__ __forceinline__ int finalize_small(FS& S, const RowCfg& R, unsigned n, unsigned n_unc, uint32_t kmax, uint32_t key_g,
                                              float g, double S_below, const u64* mc, u64* sc, u64* sw, uint32_t* sid,
                                              const uint32_t* __restrict__ hot_bits, simple_row_diag& dg) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float y_max = keyf(kmax);
  for (unsigned t = tid; t < n; t += NTHR) {
    const u64 c = mc[t];
    const unsigned r = count_greater(mc, n, c);
    sc[r] = c;
    sw[r] = R.greedy ? 0ull : wfix((uint32_t)(c >> 32), y_max);
  }
  __syncthreads();
  if (wave == 0) {
    int rc = FIN_DONE;
    if (R.greedy) {
      if (lane == 0) { S.out_id = (int)(0xFFFFFFFFu - (uint32_t)sc[0]); S.out_w = 0ull; S.e_n = 1u; S.e_SK = 1ull; S.e_skfix = 0ull; S.e_SH = 0ull; S.e_acc = 0; }
    } else {
      u64 wl[8], cum[8];
      uint32_t kl[8], il[8];
      u64 loc = 0ull;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned r = (unsigned)lane * 8u + (unsigned)j;
        const u64 c = (r < n) ? sc[r] : 0ull;
        wl[j] = (r < n) ? sw[r] : 0ull;
        kl[j] = (uint32_t)(c >> 32); il[j] = 0xFFFFFFFFu - (uint32_t)c;
        loc += wl[j];
      }
      const u64 incl = wave_incl_scan(loc);
      const u64 total_m = read_lane(incl, 63);
      u64 run = incl - loc;
#pragma unroll
      for (int j = 0; j < 8; ++j) { run += wl[j]; cum[j] = run; }
      const unsigned n_k = R.k_on ? (unsigned)R.top_k : n;  // n >= top_k was checked by the caller
      const u64 S_klist = __shfl(pick8(cum, (int)((n_k - 1u) & 7u)), (int)((n_k - 1u) >> 3), 64);
      const u64 S_k_fix = R.k_on ? S_klist : whole_row_mass(total_m, n_unc, key_g, y_max, g, R.tau, S_below);
      u64 target = 0ull;
      bool p_found = false;
      if (R.p_le0) p_found = true;
      else if (R.p_on) {
        target = (u64)__double2ull_ru((double)R.top_p * (double)S_k_fix);
        if (target == 0ull) target = 1ull;
        p_found = S_klist >= target;
      }
      uint32_t key_thr = 0u;
      bool m_cert = false;
      if (R.minp_on) {
        const float thr = y_max + (float)log((double)R.min_p);
        key_thr = fkey(thr);
        m_cert = key_thr > key_g;
      }
      const bool known = R.k_on || p_found || m_cert;
      if (!known) rc = (R.need_sum || (!R.k_on && !R.p_on && R.minp_on)) ? FIN_WIDE : FIN_PENDING;
      // every cut is a prefix of the sorted order; the first entry always survives
      const bool use_hot = hot_bits != nullptr;
      unsigned okm = 0u, hotm = 0u;
      unsigned cl = 0; u64 ml = 0ull, hl = 0ull;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned r = (unsigned)lane * 8u + (unsigned)j;
        bool o = r < n_k;
        if (R.p_le0) o = o && (r == 0u);
        else if (R.p_on && p_found) o = o && (cum[j] - wl[j] < target);
        if (m_cert) o = o && (kl[j] >= key_thr);
        o = (o || r == 0u) && (r < n);
        if (o) {
          okm |= 1u << j; ++cl; ml += wl[j];
          if (use_hot && hot_bit(hot_bits, il[j])) { hotm |= 1u << j; hl += wl[j]; }
        }
      }
      const unsigned ns = wave_sum(cl);
      const u64 S_K = wave_sum(ml);
      const u64 S_H = use_hot ? wave_sum(hl) : 0ull;
      bool pick_hot = false;
      if (use_hot) pick_hot = (S_H > 0ull) && (R.u_acc * (double)S_K <= (double)S_H);
      const u64 S_cls = use_hot ? (pick_hot ? S_H : S_K - S_H) : S_K;
      const double u = use_hot ? (pick_hot ? R.u_draw : R.u_tail) : R.u_draw;
      if (rc == FIN_DONE && S_cls == 0ull) rc = FIN_PENDING;  // the chosen class holds no mass here: general kernel
      u64 tfix = (u64)__double2ull_rd(u * (double)S_cls);
      if (S_cls > 0ull && tfix >= S_cls) tfix = S_cls - 1ull;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned r = (unsigned)lane * 8u + (unsigned)j;
        const bool in_cls = ((okm >> j) & 1u) && (!use_hot || (((hotm >> j) & 1u) != 0u) == pick_hot);
        if (r < n) sid[r] = in_cls ? il[j] : 0xFFFFFFFFu;
      }
      if (lane == 0) { S.e_n = ns; S.e_SK = S_K; S.e_SH = S_H; S.e_tfix = tfix; S.e_skfix = S_k_fix; S.e_acc = pick_hot ? 1 : 0; }
    }
    if (lane == 0) S.e_rc = rc;
  }
  __syncthreads();
  if (S.e_rc != FIN_DONE) return S.e_rc;
  dg.n_survivors = (int)S.e_n;
  if (R.greedy) { dg.p_chosen = 1.0f; return FIN_DONE; }
  dg.s_k = (double)S.e_skfix / WSCALE;
  if (hot_bits != nullptr) {
    dg.alpha = (double)S.e_SH / (double)S.e_SK;
    dg.flags |= SIMPLE_DIAG_SHVS | (S.e_acc ? SIMPLE_DIAG_ACCEPTED : 0u);
  }
  // inverse CDF in ascending token id over the survivors of the chosen class (they lie in [0, e_n))
  const unsigned n_s = S.e_n;
  const u64 tfix = S.e_tfix;
  for (unsigned t = tid; t < n_s; t += NTHR) {
    const uint32_t my = sid[t];
    if (my == 0xFFFFFFFFu) continue;
    unsigned dummy;
    const u64 C = sum_where<false>(sid, sw, n_s, my, dummy);
    if (C > tfix && C - sw[t] <= tfix) { S.out_id = (int)my; S.out_w = sw[t]; }
  }
  __syncthreads();
  dg.p_chosen = (float)((double)S.out_w / (double)S.e_SK);
  return (S.out_id >= 0) ? FIN_DONE : FIN_PENDING;
}

// Long lists (more than MEMB certified entries, in LDS as keys lk[] / ids li[]): bucket tables over
// the key range locate each cut; only the bucket that holds a cut is resolved entry by entry.
// Same decisions as finalize_small.
template <int NTHR>
__device__ __forceinline__ int finalize_long(FS& S, const RowCfg& R, unsigned n, unsigned n_unc, uint32_t kmax,
                                             uint32_t key_g, float g, double S_below, const uint32_t* lk, const uint32_t* li,
                                             unsigned char* tables, const uint32_t* __restrict__ hot_bits, simple_row_diag& dg) {
  constexpr int NWV = NTHR / 64;
  const int tid = threadIdx.x;
  uint32_t* fcnt = reinterpret_cast<uint32_t*>(tables);             // NBF * 4
  u64* fmass = reinterpret_cast<u64*>(tables + NBF * 4);             // NBF * 8
  u64* mc = reinterpret_cast<u64*>(tables + NBF * 12);               // MEMB2 * 8
  u64* mw = reinterpret_cast<u64*>(tables + NBF * 12 + MEMB2 * 8);   // MEMB2 * 8
  const float y_max = keyf(kmax);
  // buckets are linear in the tempered value (key space is logarithmic around zero); monotone in the key
  const float bscale = (float)NBF / fmaxf(y_max - keyf(key_g), 1e-30f);
  auto bucket_of = [&](uint32_t k) { return (unsigned)min((int)((y_max - keyf(k)) * bscale), NBF - 1); };
  u64 cl = 0ull;
  for (unsigned i = tid; i < n; i += NTHR) { const u64 c = composite(lk[i], li[i]); cl = (c > cl) ? c : cl; }
  unsigned da = 0, db = 0; u64 cmax = cl, dd = 0ull;
  blk_reduce<NWV>(S, da, db, cmax, dd);
  for (int i = tid; i < NBF; i += NTHR) { fcnt[i] = 0u; fmass[i] = 0ull; }
  __syncthreads();
  for (unsigned i = tid; i < n; i += NTHR) {
    const uint32_t k = lk[i];
    const unsigned b = bucket_of(k);
    atomicAdd(&fcnt[b], 1u);
    atomicAdd(&fmass[b], wfix(k, y_max));
  }
  __syncthreads();
  const unsigned c = (tid < NBF) ? fcnt[tid] : 0u;
  const u64 m = (tid < NBF) ? fmass[tid] : 0ull;
  unsigned ce, total_c; u64 me, total_m;
  blk_excl_scan2<NWV>(S, c, m, ce, me, total_c, total_m);
  const unsigned n_k = R.k_on ? (unsigned)R.top_k : (unsigned)R.V;
  // ---- top-k cut: the bucket that holds the n_k-th entry, then its members exactly ----
  const bool kcut = R.k_on && n > n_k;
  if (kcut && tid < NBF && c > 0u && ce < n_k && n_k <= ce + c) { S.bk = tid; S.need_k = n_k - ce; S.cab_k = ce; S.mab_k = me; }
  __syncthreads();
  u64 cut_k = 0ull, S_klist = total_m;
  int bk = -1;
  if (kcut) {
    bk = S.bk;
    for (unsigned i = tid; i < n; i += NTHR) {
      const uint32_t k = lk[i];
      if ((int)bucket_of(k) == bk) {
        const unsigned slot = atomicAdd(&S.memb, 1u);
        if (slot < (unsigned)MEMB2) { mc[slot] = composite(k, li[i]); mw[slot] = wfix(k, y_max); }
      }
    }
    __syncthreads();
    const unsigned nm = S.memb;
    if (nm > (unsigned)MEMB2) return FIN_PENDING;  // ties wider than the member table
    const unsigned need = S.need_k;
    for (unsigned mi = tid; mi < nm; mi += NTHR) {
      const u64 cm = mc[mi];
      const unsigned r = count_greater(mc, nm, cm);
      if (r == need - 1u) S.cut_k = cm;
    }
    __syncthreads();
    cut_k = S.cut_k;
    u64 part = 0ull;
    for (unsigned mi = tid; mi < nm; mi += NTHR) if (mc[mi] >= cut_k) part += mw[mi];
    S_klist = S.mab_k + blk_sum_u64<NWV>(S, part);
    if (tid == 0) S.memb = 0u;
    __syncthreads();
  }
  // ---- mass of the top-k prefix (all of V when top-k is off) ----
  const u64 S_k_fix = R.k_on ? S_klist : whole_row_mass(total_m, n_unc, key_g, y_max, g, R.tau, S_below);
  // ---- nucleus cut: shortest prefix whose mass reaches top_p * S_k ----
  u64 cut_p = 0ull;
  bool p_found = false;
  if (R.p_le0) { cut_p = cmax; p_found = true; }
  else if (R.p_on) {
    u64 target = (u64)__double2ull_ru((double)R.top_p * (double)S_k_fix);
    if (target == 0ull) target = 1ull;
    if (tid < NBF && c > 0u && (bk < 0 || tid <= bk)) {
      const u64 incl = (tid == bk) ? S_klist : me + m;
      if (me < target && incl >= target) { S.bp = tid; S.mab_p = me; S.cab_p = ce; }
    }
    __syncthreads();
    const int bp = S.bp;
    if (bp >= 0) {
      for (unsigned i = tid; i < n; i += NTHR) {
        const uint32_t k = lk[i];
        if ((int)bucket_of(k) == bp && composite(k, li[i]) >= cut_k) {
          const unsigned slot = atomicAdd(&S.memb, 1u);
          if (slot < (unsigned)MEMB2) { mc[slot] = composite(k, li[i]); mw[slot] = wfix(k, y_max); }
        }
      }
      __syncthreads();
      const unsigned nm = S.memb;
      if (nm > (unsigned)MEMB2) return FIN_PENDING;
      const u64 mab = S.mab_p;
      for (unsigned mi = tid; mi < nm; mi += NTHR) {
        const u64 cm = mc[mi], wm = mw[mi];
        unsigned r;
        const u64 G = mab + sum_where<true>(mc, mw, nm, cm, r);
        if (G >= target && G - wm < target) { S.cut_p = cm; S.n_p = S.cab_p + r + 1u; }
      }
      __syncthreads();
      cut_p = S.cut_p;
      p_found = true;
      if (tid == 0) S.memb = 0u;
      __syncthreads();
    }
  }
  // ---- min-p cut: y >= fl32(y_max + fl32(ln min_p)) ----
  u64 cut_m = 0ull;
  bool m_cert = false;
  if (R.minp_on) {
    const float thr = y_max + (float)log((double)R.min_p);
    const uint32_t key_thr = fkey(thr);
    if (key_thr > key_g) { cut_m = (u64)key_thr << 32; m_cert = true; }
  }
  const bool known = R.k_on || p_found || m_cert;
  if (!known) return (R.need_sum || (!R.k_on && !R.p_on && R.minp_on)) ? FIN_WIDE : FIN_PENDING;
  if (R.k_on && R.p_on && !p_found) { return FIN_PENDING; }  // cannot happen: the top-k prefix holds its own mass
  u64 cut = cut_k;
  if (p_found && cut_p > cut) cut = cut_p;
  if (m_cert && cut_m > cut) cut = cut_m;
  if (cut > cmax) cut = cmax;  // never empty
  // ---- survivors K_b, their mass, the hot split (Eq. (7)) ----
  const bool use_hot = hot_bits != nullptr;
  unsigned ns = 0, nh = 0; u64 sk = 0ull, sh = 0ull, cdum = 0ull;
  for (unsigned i = tid; i < n; i += NTHR) {
    const uint32_t k = lk[i];
    if (composite(k, li[i]) >= cut) {
      const u64 w = wfix(k, y_max);
      ++ns; sk += w;
      if (use_hot && hot_bit(hot_bits, li[i])) { ++nh; sh += w; }
    }
  }
  blk_reduce<NWV>(S, ns, nh, cdum, sk);
  const u64 S_K = sk;
  u64 S_H = 0ull;
  if (use_hot) S_H = blk_sum_u64<NWV>(S, sh);
  bool pick_hot = false;
  if (use_hot) {
    pick_hot = (S_H > 0ull) && (R.u_acc * (double)S_K <= (double)S_H);
    dg.alpha = (double)S_H / (double)S_K;
    dg.flags |= SIMPLE_DIAG_SHVS | (pick_hot ? SIMPLE_DIAG_ACCEPTED : 0u);
  }
  const u64 S_cls = use_hot ? (pick_hot ? S_H : S_K - S_H) : S_K;
  const double u = use_hot ? (pick_hot ? R.u_draw : R.u_tail) : R.u_draw;
  dg.n_survivors = (int)ns;
  dg.s_k = (double)S_k_fix / WSCALE;
  if (S_cls == 0ull) { return FIN_PENDING; }  // the chosen class holds no mass here: general kernel
  // ---- inverse CDF in ascending token id: first id whose running mass exceeds u * S ----
  u64 tfix = (u64)__double2ull_rd(u * (double)S_cls);
  if (tfix >= S_cls) tfix = S_cls - 1ull;
  const int ishift = max(0, 32 - (int)__clz((unsigned)(R.V - 1) | 1u) - 8);
  for (int i = tid; i < NBF; i += NTHR) fmass[i] = 0ull;
  __syncthreads();
  auto in_class = [&](uint32_t k, uint32_t id) {
    if (composite(k, id) < cut) return false;
    if (!use_hot) return true;
    return (hot_bit(hot_bits, id) != 0u) == pick_hot;
  };
  for (unsigned i = tid; i < n; i += NTHR) if (in_class(lk[i], li[i])) atomicAdd(&fmass[li[i] >> ishift], wfix(lk[i], y_max));
  __syncthreads();
  {
    const u64 m2 = (tid < NBF) ? fmass[tid] : 0ull;
    unsigned ce2, ct2; u64 me2, mt2;
    blk_excl_scan2<NWV>(S, 0u, m2, ce2, me2, ct2, mt2);
    if (tid < NBF && m2 > 0ull && me2 <= tfix && me2 + m2 > tfix) { S.bd = tid; S.mab_d = me2; }
  }
  __syncthreads();
  const int bd = S.bd;
  if (bd < 0) { return FIN_PENDING; }  // cannot happen: tfix < S_cls
  for (unsigned i = tid; i < n; i += NTHR) {
    if (in_class(lk[i], li[i]) && (int)(li[i] >> ishift) == bd) {
      const unsigned slot = atomicAdd(&S.memb, 1u);
      if (slot < (unsigned)MEMB2) { mc[slot] = (u64)li[i]; mw[slot] = wfix(lk[i], y_max); }
    }
  }
  __syncthreads();
  {
    const unsigned nm = S.memb;
    if (nm > (unsigned)MEMB2) return FIN_PENDING;
    const u64 mab = S.mab_d;
    for (unsigned mi = tid; mi < nm; mi += NTHR) {
      const u64 im = mc[mi], wm = mw[mi];
      unsigned dummy;
      const u64 C = mab + sum_where<false>(mc, mw, nm, im, dummy);
      if (C > tfix && C - wm <= tfix) { S.out_id = (int)im; S.out_w = wm; }
    }
  }
  __syncthreads();
  dg.p_chosen = (float)((double)S.out_w / (double)S_K);
  return (S.out_id >= 0) ? FIN_DONE : FIN_PENDING;
}

__device__ inline void queue_pending(const SampleArgs& a, int row) {
  const unsigned slot = atomicAdd(&a.pend[a.parity], 1u);
  a.pend[2 + slot] = (uint32_t)row;
  a.out[row] = PENDING;
}

// ---------------------------------------------------------------- the kernel ------------------
// (The second launch bound is HIP's: waves per SIMD, not workgroups per compute unit.  Four waves per
// SIMD, 128 registers each, are sixteen waves per compute unit at every workgroup size: four
// workgroups of 256 threads, two of 512, one of 1024.)
// STATEFUL: the rows' histories come from an incremental penalty state (its own instantiation, so
// that the stateless kernel carries none of that code).
template <typename DT, int NTHR, bool STATEFUL>
__global__ __launch_bounds__(NTHR, 4) void fast_rows_kernel(const SampleArgs a) {
  constexpr int NWV = NTHR / 64;
  constexpr int EPL = Io<DT>::EPL;
  constexpr int T = 64 * EPL * UNR;
  constexpr int PER = CAPF_PER_THREAD;
  typedef typename Io<DT>::Raw Raw;
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;  // (rows with long epilogues first: see order_rows_kernel)
  const int V = a.V;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)row * (size_t)a.stride;
  // the pattern-count kernel, when it ran before this one, has left NOT_TAKEN on every row that is still to do
  if (a.pattern_on && a.out[row] != NOT_TAKEN) {
    if (blockIdx.x == 0 && tid == 0) { a.pend[a.parity ^ 1] = 0u; a.wq[a.parity ^ 1] = 0u; }  // the previous launch's counts
    return;
  }
  // this wave's first two tiles (its threshold sample): issued before anything else
  const int nfull = V / T;  // the host guarantees nfull >= 2 * NWV
  const int t0 = (int)(((long long)wave * nfull) / NWV);
  Raw A[UNR], Bf[UNR];
#pragma unroll
  for (int u = 0; u < UNR; ++u) A[u] = Io<DT>::load(rowp + (size_t)t0 * T + u * 64 * EPL + lane * EPL);
#pragma unroll
  for (int u = 0; u < UNR; ++u) Bf[u] = Io<DT>::load(rowp + (size_t)(t0 + 1) * T + u * 64 * EPL + lane * EPL);
  const simple_row_params par = a.params[row];
  if (blockIdx.x == 0 && tid == 0) { a.pend[a.parity ^ 1] = 0u; a.wq[a.parity ^ 1] = 0u; }  // the previous launch's counts
  uint32_t* samp = reinterpret_cast<uint32_t*>(lds + a.F.samp);

  // ---- row configuration (identical in every thread) ----
  const bool bad_par = !(par.temperature >= 0.0f) || !(par.rep_penalty > 0.0f);
  RowCfg R;
  R.greedy = par.temperature == 0.0f;
  R.k_on = par.top_k >= 1 && par.top_k < V;
  R.top_k = par.top_k; R.V = V;
  R.tau = R.greedy ? 1.0f : par.temperature;
  R.top_p = par.top_p; R.min_p = par.min_p;
  R.p_on = par.top_p < 1.0f;
  R.p_le0 = par.top_p <= 0.0f;
  R.minp_on = par.min_p > 0.0f;
  R.need_sum = !R.greedy && !R.k_on && R.p_on && !R.p_le0;
  // the call's CSR arrays, or the row's slot of an incremental state
  const RowHist rh = STATEFUL ? row_history_state(a, row, par.n_prompt) : row_history_csr(a, row, par.n_prompt);
  const int nnz = rh.nnz;
  constexpr bool stateful = STATEFUL;
  const bool too_long = nnz > a.max_nnz;
  const bool pen_on = par.rep_penalty != 1.0f || par.freq_penalty != 0.0f || par.pres_penalty != 0.0f;
  const bool lowering = par.rep_penalty >= 1.0f && par.freq_penalty >= 0.0f && par.pres_penalty >= 0.0f;
  const bool h_active = (nnz > 0) && pen_on;
  const bool no_trunc = !R.greedy && !R.k_on && !R.p_on && !R.minp_on;
  // Rows that keep no candidate list and only pass through here on their way to the kernels of the
  // whole-vocabulary routes, which apply any penalties column by column: rows without any
  // truncation, and rows without top-k whose penalties raise logits (the list's threshold test on
  // raw logits would miss columns).
  // ... and rows with top-k alone beyond the list's reach (any penalties).
  const bool big_k = !R.greedy && R.k_on && par.top_k > KMAXF && !R.p_on && !R.minp_on;
  const bool straight = no_trunc || big_k || (!R.greedy && !R.k_on && !R.p_le0 && h_active && !lowering);
  const uint32_t straight_mode = no_trunc ? (uint32_t)WIDE_ALL : big_k ? (uint32_t)WIDE_TOP_K
                                          : (R.p_on ? (uint32_t)WIDE_TOP_P : (uint32_t)WIDE_MIN_P);
  const bool eligible = straight ? (!bad_par && !too_long)
                                 : (!bad_par && !too_long && (!h_active || lowering) &&
                                    (R.greedy || !R.k_on || par.top_k <= KMAXF));
  if (!eligible) {  // the general kernel takes the row (it also reports parameter errors)
    if (tid == 0) queue_pending(a, row);
    return;
  }
  // (top-k beyond the list: the threshold is only the reference of the masses and must leave fewer
  // than top_k columns above it, so it aims at a quarter of them)
  const int k_sel = R.greedy ? 1 : (R.k_on ? (big_k ? par.top_k / 4 : par.top_k) : (R.p_le0 ? 1 : KMAXF));
  if (tid == 0) {
    S.cand_count = 0u; S.flags = 0u; S.kmax = 0u; S.memb = 0u; S.bk = -1; S.bp = -1; S.bd = -1;
    S.need_k = 0u; S.cut_k = 0ull; S.cut_p = 0ull; S.n_p = 0u; S.out_id = -1; S.out_w = 0ull;
    S.n2 = 0u; S.nunc = 0u; S.e_rc = FIN_PENDING; S.e_n = 0u; S.tile_ctr = 0u;
  }
  // ---- loads first: history ids, then this wave's two sample tiles ----
  const int32_t* hist = rh.ids;
  // With a state the tables come ready-made from the row's slot (section 5.2: carried from step to
  // step, not rebuilt): `whole` = mask, rank directory and counts, else the mask alone.  Ends with a barrier.
  auto load_tables = [&](bool whole) {
    const unsigned n_pairs = (unsigned)((((V + 31) >> 5) + 1) >> 1);
    const unsigned units = whole ? (a.F.cnt + (unsigned)((nnz + 3) / 2) * 4u + 15u) / 16u : (n_pairs * 8u + 15u) / 16u;
    const u32x4* src = reinterpret_cast<const u32x4*>(a.st_tables + (size_t)rh.slot * a.st_stride);
    u32x4* dst = reinterpret_cast<u32x4*>(lds);
    for (unsigned i = tid; i < units; i += NTHR) dst[i] = as_global(src)[i];
    if (tid == 0) { S.distinct = (unsigned)a.st_rec[rh.slot].distinct; if (rh.flags) atomicOr(&S.flags, rh.flags); }
    __syncthreads();
  };
  Hist H;
  H.bm = reinterpret_cast<uint32_t*>(lds + a.F.bitmap);
  H.dir = reinterpret_cast<uint16_t*>(lds + a.F.dir);
  H.cnt32 = reinterpret_cast<uint32_t*>(lds + a.F.cnt);
  H.n_words = (V + 31) >> 5;
  H.rep = par.rep_penalty; H.freq = par.freq_penalty; H.pres = par.pres_penalty;
  H.inv_rep = 1.0 / (double)par.rep_penalty;
  H.active = h_active;
  {
    int ids[IDR];
#pragma unroll
    for (int j = 0; j < IDR; ++j) { const int i = tid + j * NTHR; ids[j] = (h_active && !stateful && i < nnz) ? hist[i] : -1; }
    {
      double u[3];
      row_uniforms(a.seed, a.row_offset + (uint64_t)row, a.step, u);
      R.u_draw = u[0]; R.u_acc = u[1]; R.u_tail = u[2];
    }
    __syncthreads();
    // ---- presence mask of the history (in the shared region); all tables for a row that leaves early ----
    if (H.active) {
      if (stateful) load_tables(straight);
      else if (straight) { unsigned own; build_history<NTHR>(S, H, ids, hist, nnz, rh.n_prompt, V, own); }
      else build_bitmap<NTHR>(S, H, ids, hist, nnz, V);
    }
  }
  const uint32_t* hot_bits = R.greedy ? nullptr : a.hot_bits;

  // ---- threshold from the sample: three largest penalised values per lane, wave select, merge ----
  float a1 = -INFINITY, a2 = -INFINITY, a3 = -INFINITY;  // branch-free insertion; a NaN is ignored here
#define SIMPLE_TAKE3(v) do { const float v_ = (v); const float m1_ = fmaxf(a1, v_), l1_ = fminf(a1, v_); \
    const float m2_ = fmaxf(a2, l1_), l2_ = fminf(a2, l1_); a3 = fmaxf(a3, l2_); a2 = m2_; a1 = m1_; } while (0)
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
    float z[EPL];
    sample_group<DT>(A[u], t0 * T + u * 64 * EPL + lane * EPL, H, z);
#pragma unroll
    for (int e = 0; e < EPL; ++e) SIMPLE_TAKE3(z[e]);
    sample_group<DT>(Bf[u], (t0 + 1) * T + u * 64 * EPL + lane * EPL, H, z);
#pragma unroll
    for (int e = 0; e < EPL; ++e) SIMPLE_TAKE3(z[e]);
  }
#undef SIMPLE_TAKE3
  // rank in the sample whose value leaves, with high probability, >= k_sel columns above it in the row
  const float m_exp = (float)k_sel * (float)(NWV * 2 * T) / (float)V;
  const unsigned r_samp = (unsigned)ceilf(1.15f * m_exp + 3.2f * sqrtf(m_exp) + 3.5f);
  {
    const float r_w = (float)r_samp / (float)NWV;
    const unsigned q = min((unsigned)(SPW * 3 / 4), (unsigned)ceilf(r_w + 3.0f * sqrtf(r_w) + 2.0f));
    const uint32_t k3[3] = {fkey(a1), fkey(a2), fkey(a3)};
    // every lane's largest is >= the smallest of the lanes' largest: at least 64 >= q keys qualify
    const uint32_t Kw = wave_threshold<3>(k3, q, q / 4u + 1u, wave_min_u32(k3[0]), wave_max_u32(k3[0]));
    if (lane < SPW) samp[wave * SPW + lane] = 0u;
    unsigned have = 0;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const u64 m = __ballot(k3[j] >= Kw);
      const unsigned p = have + lanes_before(m);
      if (((m >> lane) & 1ull) && p < (unsigned)SPW) samp[wave * SPW + p] = k3[j];
      have = min(have + (unsigned)__popcll(m), (unsigned)SPW);
    }
    const float wp = wave_max(a1);
    if (lane == 0) { S.wmax[wave] = wp; S.wcnt[wave] = have; }
  }
  __syncthreads();
  StreamCtx C;
  {
    constexpr int NS = (NWV * SPW) / 64;
    uint32_t ks[NS];
    unsigned total = 0;
    float Mp = S.wmax[0];
#pragma unroll
    for (int w = 0; w < NWV; ++w) { total += S.wcnt[w]; Mp = fmaxf(Mp, S.wmax[w]); }
    uint32_t kmn = 0xFFFFFFFFu, kmx = 0u;
#pragma unroll
    for (int j = 0; j < NS; ++j) { ks[j] = samp[j * 64 + lane]; kmx = max(kmx, ks[j]); if (ks[j]) kmn = min(kmn, ks[j]); }
    kmn = wave_min_u32(kmn); kmx = wave_max_u32(kmx);
    const unsigned need = max(1u, min(r_samp, total));
    float g = keyf(wave_threshold<NS>(ks, need, need / 8u + 1u, min(kmn, kmx), kmx));
    if (!R.greedy && !R.k_on && R.minp_on) {
      // min-p survivors lie within ln(min_p) of the row maximum, which is at least the sample's
      const float thr_lb = Mp / R.tau + (float)log((double)R.min_p);
      float gm = thr_lb * R.tau;
      gm = gm - fabsf(gm) * 1e-6f - 1e-30f;
      g = fmaxf(g, gm);
    }
    C.g = g;
    C.y_g = R.greedy ? g : g / R.tau;
    C.inv_tau = 1.0 / (double)R.tau;
    C.need_sum = R.need_sum;
    C.l2e_tau = (float)(1.4426950408889634 / (double)R.tau);
  }
  // Hands the row to the kernels of the whole-vocabulary routes: a queue record, a cleared workspace
  // slot and the row's history tables (rebuilt first if the region no longer holds them).  False if
  // no slot is free.  All threads call.
  auto queue_wide = [&](uint32_t mode, bool tables_live) -> bool {
    __syncthreads();
    if (H.active && !tables_live) {
      if (stateful) load_tables(true);
      else {
        int ids2[IDR];
#pragma unroll
        for (int j = 0; j < IDR; ++j) { const int i = tid + j * NTHR; ids2[j] = (i < nnz) ? hist[i] : -1; }
        unsigned own;
        build_history<NTHR>(S, H, ids2, hist, nnz, rh.n_prompt, V, own);
      }
    }
    if (tid == 0) S.e_n = atomicAdd(&a.wq[a.parity], 1u);
    __syncthreads();
    const unsigned slot = S.e_n;
    const unsigned hb = H.active ? (a.F.cnt + (unsigned)((nnz + 3) / 2) * 4u + 15u) / 16u : 0u;  // 16-byte units of history tables
    if (slot >= (unsigned)a.wide_slots || WS_HT + hb * 16u > a.ws_stride) return false;
    u32x4* ws = reinterpret_cast<u32x4*>(a.wws + (size_t)slot * a.ws_stride);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (unsigned i = tid; i < WS_RL / 16u; i += NTHR) ws[i] = zero;
    if (H.active) {
      const u32x4* src = reinterpret_cast<const u32x4*>(lds);
      for (unsigned i = tid; i < hb; i += NTHR) ws[WS_HT / 16u + i] = src[i];
    }
    if (tid == 0) {
      WideRec rec;
      rec.row = (uint32_t)row; rec.g = C.g; rec.mode = mode; rec.flags = S.flags & 0x3FFFFFFFu;
      rec.tau = R.tau; rec.top_p = R.top_p; rec.rep = par.rep_penalty; rec.freq = par.freq_penalty;
      rec.pres = par.pres_penalty; rec.nnz = nnz; rec.n_prompt = min(max(rh.n_prompt, 0), nnz); rec.h_active = h_active ? 1 : 0;
      rec.min_p = R.min_p; rec.top_k = par.top_k; rec.distinct = H.active ? S.distinct : 0u; rec.reserved1 = 0u;
      reinterpret_cast<WideRec*>(a.wq + WQ_HEAD)[slot] = rec;
      a.out[row] = PENDING;
    }
    return true;
  };
  if (straight) {  // nothing to select here (without truncation every column survives)
    if (!queue_wide(straight_mode, true) && tid == 0) queue_pending(a, row);
    return;
  }
  const bool minp_only = !R.greedy && !R.k_on && !R.p_on && R.minp_on;
  // the history mask is dead from here (every wave passed the barrier above after its last lookup):
  // the region becomes the candidate list
  uint32_t* lz = reinterpret_cast<uint32_t*>(lds);
  const unsigned cap = (unsigned)a.F.list_cap;
  uint32_t* li = lz + cap;
  u64 below_mass = 0ull;  // this thread's share of the mass below g (integer: the total is order-free)
  // ---- the stream (raw logits) ----
  // Every wave starts with its two sample tiles (in registers).  With four waves per row each then
  // takes the rest of its contiguous share of the row; with more, the other tiles are handed out one
  // at a time from a counter, so that the waves finish together whatever each of them met (measured:
  // 1 % slower at four waves, 1.5 to 3 % faster at eight).  No result depends on which wave took
  // which tile (the list is ranked by value and id, the masses are integers).
  constexpr bool HAND_OUT = NWV > 4;
  const int t_end = (int)(((long long)(wave + 1) * nfull) / NWV);
  const unsigned n_dyn = (unsigned)(nfull - 2 * NWV);
  int t_own = t0 + 2;  // contiguous shares: this wave's next tile
  auto grab = [&]() -> int {  // the next tile for this wave, -1 if none; the same in every lane
    if constexpr (!HAND_OUT) {
      const int t = t_own++;
      return t < t_end ? t : -1;
    } else {
      unsigned c = 0u;
      if (lane == 0) c = atomicAdd(&S.tile_ctr, 1u);
      c = (unsigned)__builtin_amdgcn_readfirstlane((int)c);
      if (c >= n_dyn) return -1;
      int t = (int)c;  // the c-th tile that is no wave's sample tile
#pragma unroll
      for (int w = 0; w < NWV; ++w) { const int s0 = (int)(((long long)w * nfull) / NWV); if (s0 <= t) t += 2; }
      return t;
    }
  };
  auto fill = [&](Raw (&X)[UNR], int t) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) X[u] = Io<DT>::load(rowp + (size_t)t * T + u * 64 * EPL + lane * EPL);
  };
  {
    int tA = t0, tB = t0 + 1;
    int nx = grab();
    if constexpr (sizeof(DT) == 2) {
      // two buffers in turn, each refilled as soon as it has been consumed, so no registers are
      // copied (bf16: 7 % faster on C5 than the rotation below, which in turn is 1.5 % faster for
      // float32 on C3)
      while (tA >= 0) {
        stream_tile<DT>(A, tA * T, C, S, lz, li, cap, below_mass);
        tA = nx;
        if (tA >= 0) { fill(A, tA); nx = grab(); }
        if (tB < 0) continue;
        stream_tile<DT>(Bf, tB * T, C, S, lz, li, cap, below_mass);
        tB = nx;
        if (tB >= 0) { fill(Bf, tB); nx = grab(); }
      }
    } else {
      stream_tile<DT>(A, tA * T, C, S, lz, li, cap, below_mass);
      while (tB >= 0) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) A[u] = Bf[u];
        tA = tB;
        tB = nx;
        if (tB >= 0) { fill(Bf, tB); nx = grab(); }
        stream_tile<DT>(A, tA * T, C, S, lz, li, cap, below_mass);
      }
    }
  }
  // the epilogue rebuilds the history tables: fetch the ids while the other waves finish
  int ids[IDR];
#pragma unroll
  for (int j = 0; j < IDR; ++j) { const int i = tid + j * NTHR; ids[j] = (h_active && (!stateful || R.need_sum) && i < nnz) ? hist[i] : -1; }
  // ragged tail, element by element
  for (int idx = nfull * T + tid; idx < V; idx += NTHR) {
    const float zz = Io<DT>::one(rowp + idx);
    if (C.need_sum) below_mass += (u64)below_term_clamped(zz, C);
    if (!(zz < C.g)) {
      const unsigned slot = atomicAdd(&S.cand_count, 1u);
      if (slot < cap) { lz[slot] = __float_as_uint(zz); li[slot] = (uint32_t)idx; }
    }
  }
  __syncthreads();

  // ---- epilogue ----
  simple_row_diag dg;
  dg.alpha = __longlong_as_double(0x7FF8000000000000ll);
  dg.s_k = 0.0; dg.p_chosen = 0.0f; dg.n_survivors = 0; dg.flags = 0u; dg.reserved = 0u;
  if (a.hot_bits && a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
  int rc = FIN_PENDING;
  const unsigned n = S.cand_count;
  // the stream added 2^28 for every column at or above g: all of them were counted for the list
  if (C.need_sum && tid == 0) below_mass -= (u64)n << 28;
  if (n > cap && (R.need_sum || minp_only)) {
    // more columns at or above g than the list holds, and a cut that the whole-vocabulary routes
    // find without the list
    if (queue_wide(R.need_sum ? WIDE_TOP_P : WIDE_MIN_P, false)) return;
  }
  if (n <= cap) {
    // the list moves to registers; the region takes the history tables again
    float ez[PER]; uint32_t eid[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const unsigned i = (unsigned)tid + (unsigned)j * NTHR;
      ez[j] = (i < n) ? __uint_as_float(lz[i]) : -INFINITY;
      eid[j] = (i < n) ? li[i] : 0u;
    }
    __syncthreads();
    if (H.active) {
      unsigned own = 0u;
      if (stateful) load_tables(true);
      else build_history<NTHR>(S, H, ids, hist, nnz, rh.n_prompt, V, own);
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const unsigned i = (unsigned)tid + (unsigned)j * NTHR;
        if (i < n) ez[j] = H.penalised_at(ez[j], (int)eid[j]);
      }
      if (R.need_sum) {
        // exact correction of the mass below g for the history columns (the stream summed their raw
        // values), once per distinct column: by the thread that first marked it when all ids sit in
        // registers, else by the thread that first claims the column's rank
        const bool by_claim = stateful || nnz > IDR * NTHR;  // (ready-made tables come without first-marker flags)
        uint32_t* claim = reinterpret_cast<uint32_t*>(lds + a.F.claim);
        if (by_claim) {
          zero16(claim, ((nnz + 31) / 32) * 4, tid, NTHR);
          __syncthreads();
        }
        auto claims = [&](int id) -> bool {  // true for exactly one of the entries that name this column
          if ((unsigned)id >= (unsigned)V) return false;
          const unsigned r = H.rank(id, H.bm[id >> 5]);
          const uint32_t bit = 1u << (r & 31u);
          return !(atomicOr(&claim[r >> 5], bit) & bit);
        };
        auto correct = [&](float z_raw, int id) {  // columns at or above g are in the list: their terms are settled there
          if (z_raw < C.g) {
            below_mass -= (u64)below_term(z_raw, C);
            below_mass += (u64)below_term(H.penalised_at(z_raw, id), C);
          }
        };
        if (by_claim) {
          own = 0u;
#pragma unroll
          for (int j = 0; j < IDR; ++j) if (tid + j * NTHR < nnz && claims(ids[j])) own |= 1u << j;
        }
        float zr[IDR];
#pragma unroll
        for (int j = 0; j < IDR; ++j) zr[j] = ((own >> j) & 1u) ? Io<DT>::one(rowp + ids[j]) : 0.0f;
#pragma unroll
        for (int j = 0; j < IDR; ++j) if ((own >> j) & 1u) correct(zr[j], ids[j]);
        // entries beyond the registers, four at a time (their trips to memory overlap)
        for (int i0 = tid + IDR * NTHR; i0 < nnz; i0 += 4 * NTHR) {
          int id4[4]; bool mine[4]; float z4[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) id4[k] = (i0 + k * NTHR < nnz) ? hist[i0 + k * NTHR] : -1;
#pragma unroll
          for (int k = 0; k < 4; ++k) mine[k] = claims(id4[k]);
#pragma unroll
          for (int k = 0; k < 4; ++k) z4[k] = mine[k] ? Io<DT>::one(rowp + id4[k]) : 0.0f;
#pragma unroll
          for (int k = 0; k < 4; ++k) if (mine[k]) correct(z4[k], id4[k]);
        }
      }
      __syncthreads();
    }
    // keys of the tempered values; listed columns that fell below g return to the mass below g
    uint32_t key[PER];
    bool err = false, peaked = false;
    uint32_t kloc = 0u;
    u64 mlist = 0ull, mcert = 0ull;  // mass (relative to the one at y_g) of the listed / certified columns
    const uint32_t key_g = fkey(C.y_g);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const unsigned i = (unsigned)tid + (unsigned)j * NTHR;
      key[j] = 0u;
      if (i < n) {
        const float z = ez[j];
        if (z != z || z == INFINITY) err = true;
        else if (!(z < C.g)) {
          const float y = R.greedy ? z : tempered(z, C);  // the IEEE quotient z / tau
          if (y == INFINITY) err = true;
          else {
            key[j] = fkey(y);
            if (R.need_sum) {
              int b;
              const float w = mass_term(z, C, b);
              if (w > 2097152.0f) peaked = true;  // 2^21: far too peaked for a wide nucleus
              mlist += mass_fix(w);
              if (key[j] > key_g) mcert += mass_fix(w);
            }
          }
        } else if (R.need_sum) below_mass += (u64)below_term(z, C);
      }
      kloc = max(kloc, key[j]);
    }
    if (kloc) atomicMax(&S.kmax, kloc);
    if (err) atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
    if (peaked) atomicOr(&S.flags, 1u << 30);
    __syncthreads();
    // mass below g (integer, exact) and the decision between the list and the kernels that follow
    u64 S_below_int = 0ull, M_list = 0ull, M_cert = 0ull;
    bool wide = false;
    if (R.need_sum) {
      S_below_int = blk_sum_u64<NWV>(S, below_mass);
      M_list = blk_sum_u64<NWV>(S, mlist);
      M_cert = blk_sum_u64<NWV>(S, mcert);
      const u64 target = (u64)__double2ull_ru((double)R.top_p * (double)(M_list + S_below_int));
      wide = !R.minp_on && M_cert < target;
    }
    const double S_below = (double)S_below_int / (double)MSCALE;
    const uint32_t kmax = S.kmax;
    bool tables_live = false;  // the region still holds the history tables
    if (S.flags & SIMPLE_DIAG_ERROR) rc = FIN_DONE;
    else if (kmax <= key_g || kmax <= KEY_NEG_INF) rc = FIN_PENDING;
    else if (wide) {
      rc = ((S.flags >> 30) & 1u) ? FIN_PENDING : FIN_WIDE;
      tables_live = true;
    } else {
      // certified entries (tempered value strictly above fl(g / tau)) as composites
      u64* mc = reinterpret_cast<u64*>(lds);                       // MEMB * 8
      u64* sc = mc + MEMB;
      u64* sw = sc + MEMB;
      uint32_t* sid = reinterpret_cast<uint32_t*>(sw + MEMB);      // ends at 14 KB
      unsigned nul = 0;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        if (!key[j]) continue;
        if (key[j] > key_g) {
          const unsigned slot = atomicAdd(&S.n2, 1u);
          if (slot < (unsigned)MEMB) mc[slot] = composite(key[j], eid[j]);
        } else { ++nul; key[j] = 0u; }
      }
      if (nul) atomicAdd(&S.nunc, nul);
      __syncthreads();
      const unsigned n_cert = S.n2, n_unc = S.nunc;
      if (R.k_on && !R.greedy && n_cert < (unsigned)R.top_k) rc = FIN_PENDING;  // the sampled threshold admitted too few
      else if (n_cert <= (unsigned)MEMB) {
        rc = finalize_small<NTHR>(S, R, n_cert, n_unc, kmax, key_g, C.g, S_below, mc, sc, sw, sid, hot_bits, dg);
      } else if (n_cert <= (unsigned)a.F.long_cap) {
        // long list: keys and ids go back to the region, the bucket tables behind them
        const unsigned lcap = (unsigned)a.F.long_cap;
        uint32_t* lk = reinterpret_cast<uint32_t*>(lds);
        uint32_t* lid = lk + lcap;
        __syncthreads();
        if (tid == 0) S.n2 = 0u;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < PER; ++j) {
          if (key[j]) { const unsigned slot = atomicAdd(&S.n2, 1u); lk[slot] = key[j]; lid[slot] = eid[j]; }
        }
        __syncthreads();
        rc = finalize_long<NTHR>(S, R, n_cert, n_unc, kmax, key_g, C.g, S_below, lk, lid, lds + (size_t)lcap * 8u, hot_bits, dg);
      }
      if (rc == FIN_WIDE && ((S.flags >> 30) & 1u)) rc = FIN_PENDING;
    }

    // ---- a cut below the list's reach: the row goes to the kernels that follow ----
    if (rc == FIN_WIDE) {
      if (queue_wide(R.need_sum ? WIDE_TOP_P : WIDE_MIN_P, tables_live)) return;
      rc = FIN_PENDING;  // no free slot: the general kernel takes the row
    }
  }
  if (tid == 0) {
    if (rc != FIN_DONE) {
      queue_pending(a, row);
    } else {
      const unsigned f = S.flags & 0x3FFFFFFFu;
      const bool err = (f & SIMPLE_DIAG_ERROR) != 0u;
      a.out[row] = err ? -1 : S.out_id;
      dg.flags |= f | (R.greedy ? SIMPLE_DIAG_GREEDY : 0u);
      if (err) dg.p_chosen = 0.0f;
      if (a.diag) a.diag[row] = dg;
      if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
      write_decision(a, row, err ? -1 : S.out_id, dg.p_chosen, R.greedy);
    }
  }
}

}  // namespace fast

}  // namespace simple
namespace simple {

template <bool STATEFUL>
static hipError_t launch_fast_instance(const SampleArgs& a, int dtype, hipStream_t st) {
  const dim3 grid((unsigned)a.B);
  if (a.F.threads == 256) {
    if (dtype == SIMPLE_F32) hipLaunchKernelGGL((fast::fast_rows_kernel<float, 256, STATEFUL>), grid, dim3(256), a.F.total, st, a);
    else hipLaunchKernelGGL((fast::fast_rows_kernel<uint16_t, 256, STATEFUL>), grid, dim3(256), a.F.total, st, a);
  } else if (a.F.threads == 512) {
    if (dtype == SIMPLE_F32) hipLaunchKernelGGL((fast::fast_rows_kernel<float, 512, STATEFUL>), grid, dim3(512), a.F.total, st, a);
    else hipLaunchKernelGGL((fast::fast_rows_kernel<uint16_t, 512, STATEFUL>), grid, dim3(512), a.F.total, st, a);
  } else {
    if (dtype == SIMPLE_F32) hipLaunchKernelGGL((fast::fast_rows_kernel<float, 1024, STATEFUL>), grid, dim3(1024), a.F.total, st, a);
    else hipLaunchKernelGGL((fast::fast_rows_kernel<uint16_t, 1024, STATEFUL>), grid, dim3(1024), a.F.total, st, a);
  }
  return hipGetLastError();
}
// The order in which the single-pass kernel's workgroups take the rows of a launch: rows with long
// epilogues first, the others behind them, each group in row order.  Workgroups are handed to the
// compute units in turn, so that a compute unit holds workgroups b, b + (number of compute units),
// ...: with the long rows at the front every compute unit gets its share of them instead of some
// holding four (measured on the heterogeneous batch: a compute unit with four such rows finishes
// 20 us after one with two), and a launch of several rounds starts its longest rows first.
constexpr int ORD_T = 1024;
__global__ __launch_bounds__(ORD_T) void order_rows_kernel(const SampleArgs a) {
  __shared__ unsigned wsum[ORD_T / 64];
  order_rows_body<ORD_T>(a, wsum);
}

hipError_t launch_order(const SampleArgs& a, hipStream_t st) {
  if (!a.order || a.B <= 0 || a.B > WIDE_SLOTS) return hipErrorInvalidValue;
  hipLaunchKernelGGL(order_rows_kernel, dim3(1), dim3(ORD_T), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fast(const SampleArgs& a, int dtype, hipStream_t st) {
  return a.st_rec ? launch_fast_instance<true>(a, dtype, st) : launch_fast_instance<false>(a, dtype, st);
}

hipError_t set_max_lds_fast(unsigned bytes) {
  const void* fns[12] = {
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 256, false>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 256, false>),
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 512, false>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 512, false>),
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 1024, false>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 1024, false>),
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 256, true>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 256, true>),
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 512, true>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 512, true>),
    reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 1024, true>), reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 1024, true>)};
  for (int i = 0; i < 12; ++i) {
    const hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace simple
