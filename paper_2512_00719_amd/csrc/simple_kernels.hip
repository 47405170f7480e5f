// Row sampling kernel for gfx950: one workgroup per logits row.
//
// Route taken by a row (all inside one launch):
//   history state (bitmap + rank directory + counts in LDS)            -- penalties, section 2.2 / 5.2
//   a few sample tiles spread over the row fix a threshold that is expected to admit a small
//   multiple of the top-k prefix; one coalesced stream over the rest of the row keeps, in an LDS
//   candidate list, every element at or above it, and, for rows whose nucleus is taken over the
//   whole vocabulary, the row's exp-sum                                 -- truncation first, 5.2
//   exact selection, softmax and inverse-CDF draw on the candidate list -- Eq. (2), step (3)
//   SHVS accept / hot draw / tail draw on the same survivors            -- section 5.3
// The list certifies its own completeness (every element at or above the threshold is in it).
// When the sampled threshold admitted too few or too many elements the row is streamed again
// with a threshold that rises monotonically and cannot fail; rows whose survivor set does not
// fit the list at all (top-k above KMAX, a very wide nucleus, no truncation) take a multi-pass
// radix descent over the row, which is exact for every input.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "simple_device.hpp"
#include "simple_kernels.hpp"

namespace simple {


typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ element access -------------
// The pointers are into the logits, device memory, and the loads say so (global-typed pointers): a
// generic load also counts as an LDS access, and every wait for an LDS result would wait for it.
template <typename DT> struct Elem;
template <> struct Elem<float> {
  static constexpr int EPL = 4;
  typedef __attribute__((address_space(1))) const float Glob;
  typedef __attribute__((address_space(1))) const f32x4 GlobVec;
  __device__ static __forceinline__ float one(const float* p) { return *(Glob*)p; }
  template <bool VEC>
  __device__ static __forceinline__ void vec(const float* p, float (&z)[4]) {
    if (VEC) {  // streamed once: non-temporal so the row does not displace what the L2 should keep
      const f32x4 v = __builtin_nontemporal_load((GlobVec*)p);
      z[0] = v.x; z[1] = v.y; z[2] = v.z; z[3] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) z[e] = ((Glob*)p)[e];
    }
  }
};
template <> struct Elem<uint16_t> {  // bfloat16 bit patterns; the upcast to float32 is exact
  static constexpr int EPL = 8;
  typedef __attribute__((address_space(1))) const uint16_t Glob;
  typedef __attribute__((address_space(1))) const u32x4 GlobVec;
  __device__ static __forceinline__ float one(const uint16_t* p) { return __uint_as_float((uint32_t)(*(Glob*)p) << 16); }
  template <bool VEC>
  __device__ static __forceinline__ void vec(const uint16_t* p, float (&z)[8]) {
    if (VEC) {
      const u32x4 v = __builtin_nontemporal_load((GlobVec*)p);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = __uint_as_float(w[i] << 16);
        z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) z[e] = one(p + e);
    }
  }
};

// ------------------------------------------------------------------ shared row state -----------
struct Shared {
  float tau, c_hi, c_lo;
  int greedy, k_on, k_sel, top_k;
  float top_p, min_p;
  unsigned cand_count, n_conv, min_key, max_key;
  float g_pass;
  unsigned flags;
  unsigned sel_digit, sel_need, sel_cnt, sel_found;
  unsigned long long sel_above_mass;
  unsigned sel_above_cnt;
  unsigned scan_u32[NW + 1];
  unsigned long long scan_u64[NW + 1];
  double scan_d[NW + 1];
  float red_f[NW + 1];
  unsigned flag_ws;
  unsigned found_lo, found_hi;
  int walk_chunk, tie_chunk;
  unsigned long long walk_base;
  unsigned walk_ties_before, adm_split[2];
  unsigned list_n;  // keys the descent has set aside for its last level
  int out_id;
  float out_p;
};

// Smallest float z (by bisection over the orderable keys) whose tempered value
// y = (greedy ? z : z / tau) satisfies y > yk (strict) or y >= yk (!strict); the map z -> fl(z/tau)
// is monotone.  yk is finite or -inf.
__device__ inline float min_z_reaching(float yk, float tau, bool greedy, bool strict) {
  uint32_t lo = KEY_NEG_INF, hi = KEY_POS_INF;  // predicate false at lo (unless yk = -inf, !strict), true at hi
  auto pred = [&](uint32_t k) {
    const float z = keyf(k);
    const float y = greedy ? z : z / tau;
    return strict ? (y > yk) : (y >= yk);
  };
  if (pred(lo)) return keyf(lo);
  const float guess = greedy ? yk : yk * tau;
  if (guess > -INFINITY && guess < INFINITY) {  // gallop around the algebraic inverse first
    const uint32_t c = fkey(guess);
    uint32_t step = 2;
    uint32_t a = c, b = c;
    while (true) {  // walk down until the predicate is false
      a = (a - KEY_NEG_INF > step) ? a - step : KEY_NEG_INF;
      if (!pred(a) || a == KEY_NEG_INF) break;
      step <<= 1;
    }
    step = 2;
    while (true) {  // walk up until it is true
      b = (KEY_POS_INF - b > step) ? b + step : KEY_POS_INF;
      if (pred(b) || b == KEY_POS_INF) break;
      step <<= 1;
    }
    lo = a; hi = b;
  }
  while (hi - lo > 1u) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (pred(mid)) hi = mid; else lo = mid;
  }
  return keyf(hi);
}

// ------------------------------------------------------------------ the stream -----------------
// Appends the lanes flagged in the wave mask `m` to the candidate list as (float bits, id).
__device__ __forceinline__ void append_lanes(Shared& S, uint32_t* ck, uint32_t* ci,
                                             unsigned long long m, float z, int idx) {
  const int lane = lane_id();
  unsigned base = 0;
  if (lane == 0) base = atomicAdd(&S.cand_count, (unsigned)__popcll(m));
  base = __shfl(base, 0, 64);
  if ((m >> lane) & 1ull) {
    const unsigned slot = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (slot < (unsigned)CAP) { ck[slot] = __float_as_uint(z); ci[slot] = (uint32_t)idx; }
  }
}

// Running (max, exp-sum) of one thread, in logit space: s = sum exp2((z - m) * c), c = log2(e)/tau
// split into c_hi + c_lo so the product keeps ~48 bits.
struct ExpSum {
  float m; double s; float c_hi, c_lo;
  __device__ __forceinline__ float w(float z) const { const float d = z - m; return __builtin_amdgcn_exp2f(fmaf(d, c_hi, d * c_lo)); }
  __device__ __forceinline__ void raise(float vmax) {
    if (vmax > m) { const float d = m - vmax; s *= (double)__builtin_amdgcn_exp2f(fmaf(d, c_hi, d * c_lo)); m = vmax; }
  }
};

// Processes one tile of the row (64 lanes x UNROLL loads x EPL elements, columns [tb, min(tb+T, V))).
// FULL: columns that are in the history are masked out here (they are handled from the history
// side afterwards) and the thread's (max, exp-sum) is updated.  ALL: every valid element is
// appended (sample tiles); otherwise only elements with !(z < g).
template <typename DT, bool VEC, bool FULL, bool ALL>
__device__ __forceinline__ void process_tile(const DT* __restrict__ rowp, int tb, int V, float g,
                                             const History& H, bool do_sum, ExpSum& E, Shared& S,
                                             uint32_t* ck, uint32_t* ci) {
  constexpr int EPL = Elem<DT>::EPL;
  constexpr int T = 64 * EPL * UNROLL;
  const int lane = lane_id();
  float z[UNROLL][EPL];
  const bool full = (tb + T <= V);
  if (full) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) Elem<DT>::template vec<VEC>(rowp + tb + u * 64 * EPL + lane * EPL, z[u]);
  } else {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int idx = tb + u * 64 * EPL + lane * EPL + e;
        z[u][e] = (idx < V) ? Elem<DT>::one(rowp + idx) : -INFINITY;
      }
    }
  }
  unsigned skip[UNROLL];  // bit e set: element is not a candidate here (masked or out of range)
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const int idx0 = tb + u * 64 * EPL + lane * EPL;
    unsigned sk = 0u;
    if (!full) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sk |= (idx0 + e < V) ? 0u : (1u << e);
    }
    if (FULL) {
      if (H.active && idx0 < V) sk |= (H.bits[idx0 >> 5] >> (idx0 & 31)) & ((1u << EPL) - 1u);
      if (sk) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) if ((sk >> e) & 1u) z[u][e] = -INFINITY;
      }
      if (do_sum) {
        float vmax = z[u][0];
#pragma unroll
        for (int e = 1; e < EPL; ++e) vmax = fmaxf(vmax, z[u][e]);
        E.raise(vmax);
        float ps = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) ps += E.w(z[u][e]);
        E.s += (double)ps;
      }
    }
    skip[u] = sk;
  }
  if (ALL || !full) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const bool pass = !((skip[u] >> e) & 1u) && (ALL || !(z[u][e] < g));
        const unsigned long long m = __ballot(pass);
        if (m) append_lanes(S, ck, ci, m, z[u][e], tb + u * 64 * EPL + lane * EPL + e);
      }
    }
  } else {
    // masked elements are -inf and fail the test unless g is -inf, which only happens when the
    // whole row was sampled (no tile reaches this branch then)
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const unsigned long long m = __ballot(!(z[u][e] < g));
        if (m) append_lanes(S, ck, ci, m, z[u][e], tb + u * 64 * EPL + lane * EPL + e);
      }
    }
  }
}

// Sample tiles: NS tiles spread evenly over the row (all tiles when the row has at most NS).
__device__ __forceinline__ bool is_sample_tile(int ti, int ntiles, int NS) {
  if (ntiles <= NS) return true;
  const int stride = ntiles / NS;
  return (ti % stride == 0) && (ti / stride < NS);
}

// Streams columns [seg0, seg1) of the row once in ascending tiles (used by the monotone-threshold
// replay).  FULL here applies the penalties element by element.
template <typename DT, bool VEC, bool FULL>
__device__ inline void stream_range(const DT* __restrict__ rowp, int seg0, int seg1, float g,
                                    const History& H, bool do_sum, ExpSum& E, Shared& S,
                                    uint32_t* ck, uint32_t* ci) {
  constexpr int EPL = Elem<DT>::EPL;
  constexpr int T = 64 * EPL * UNROLL;
  const int lane = lane_id();
  for (int tb = seg0 + wave_id() * T; tb < seg1; tb += NW * T) {
    float z[UNROLL][EPL];
    const bool full = (tb + T <= seg1);
    if (full) {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) Elem<DT>::template vec<VEC>(rowp + tb + u * 64 * EPL + lane * EPL, z[u]);
    } else {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int idx = tb + u * 64 * EPL + lane * EPL + e;
          z[u][e] = (idx < seg1) ? Elem<DT>::one(rowp + idx) : -INFINITY;
        }
      }
    }
    if (FULL) {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int idx0 = tb + u * 64 * EPL + lane * EPL;
        if (H.active && idx0 < seg1) {
          const unsigned bits = (H.bits[idx0 >> 5] >> (idx0 & 31)) & ((1u << EPL) - 1u);
          if (bits) {
#pragma unroll
            for (int e = 0; e < EPL; ++e)
              if (((bits >> e) & 1u) && idx0 + e < seg1) z[u][e] = H.penalise(z[u][e], idx0 + e);
          }
        }
        if (do_sum) {
          float vmax = z[u][0];
#pragma unroll
          for (int e = 1; e < EPL; ++e) vmax = fmaxf(vmax, z[u][e]);
          E.raise(vmax);
          float ps = 0.0f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) ps += E.w(z[u][e]);
          E.s += (double)ps;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int idx = tb + u * 64 * EPL + lane * EPL + e;
        const unsigned long long m = __ballot(!(z[u][e] < g) && (full || idx < seg1));
        if (m) append_lanes(S, ck, ci, m, z[u][e], idx);
      }
    }
  }
}

// Element-at-a-time replay of [p0, p1) used only after the candidate list overflowed.
template <typename DT, bool FULL>
__device__ inline void stream_careful(const DT* __restrict__ rowp, int p0, int p1, float g,
                                      const History& H, Shared& S, uint32_t* ck, uint32_t* ci) {
  for (int idx = p0 + (int)threadIdx.x; idx < p1; idx += NT) {
    float z = Elem<DT>::one(rowp + idx);
    if (FULL && H.active && H.test(idx)) z = H.penalise(z, idx);
    if (!(z < g)) {
      const unsigned slot = atomicAdd(&S.cand_count, 1u);
      if (slot < (unsigned)CAP) { ck[slot] = __float_as_uint(z); ci[slot] = (uint32_t)idx; }
    }
  }
}

// ------------------------------------------------------------------ candidate list -------------
__device__ __forceinline__ unsigned long long composite(uint32_t key, uint32_t id) {
  return ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - id);
}

// Turns entries [from, to) from (logit bits, id) into (orderable key of y = z'/tau, id); 0 marks a
// dropped entry.  apply_pen: the stream tested raw logits, so the penalty is applied here.
// Returns the number of valid entries among them (all threads).
__device__ inline unsigned convert_entries(Shared& S, uint32_t* ck, const uint32_t* ci, unsigned from,
                                           unsigned to, const History& H, bool apply_pen) {
  unsigned my_valid = 0;
  for (unsigned i = from + threadIdx.x; i < to; i += NT) {
    float z = __uint_as_float(ck[i]);
    const int id = (int)ci[i];
    if (apply_pen && H.active && H.test(id)) z = H.penalise(z, id);
    uint32_t key = 0u;
    if (z != z || z == INFINITY) {
      atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
    } else {
      const float y = S.greedy ? z : z / S.tau;
      if (y == INFINITY) atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
      else key = fkey(y);
    }
    ck[i] = key;
    my_valid += (key != 0u);
  }
  return block_sum(my_valid, S.scan_u32);
}

// Radix select over the 64-bit composite (key, ~id) of the valid entries [0, n): returns the cut
// (prefix, shift) such that exactly `need` entries satisfy (composite >> shift) >= prefix.
// Requires need <= number of valid entries.  `hist` holds NBINS words.
__device__ inline void select_composite(Shared& S, const uint32_t* ck, const uint32_t* ci, unsigned n,
                                        unsigned need, uint32_t* hist, unsigned long long& prefix, int& shift) {
  const int tid = threadIdx.x;
  prefix = 0ull; shift = 64;
  const int widths[6] = {11, 11, 10, 11, 11, 10};
  for (int lvl = 0; lvl < 6; ++lvl) {
    const int w = widths[lvl];
    shift -= w;
    for (int i = tid; i < NBINS; i += NT) hist[i] = 0u;
    __syncthreads();
    for (unsigned i = tid; i < n; i += NT) {
      const uint32_t key = ck[i];
      if (!key) continue;
      const unsigned long long c = composite(key, ci[i]);
      if (lvl == 0 || (c >> (shift + w)) == prefix) atomicAdd(&hist[(unsigned)(c >> shift) & ((1u << w) - 1u)], 1u);
    }
    __syncthreads();
    unsigned local[4], tsum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) { local[j] = hist[4 * tid + j]; tsum += local[j]; }
    unsigned total;
    const unsigned incl = block_incl_scan(tsum, S.scan_u32, total);
    unsigned above = total - incl;
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      if (above < need && need <= above + local[j]) {
        S.sel_digit = 4 * tid + j; S.sel_need = need - above; S.sel_cnt = local[j];
      }
      above += local[j];
    }
    __syncthreads();
    prefix = (prefix << w) | S.sel_digit;
    need = S.sel_need;
    const bool take_all = (S.sel_cnt == need);
    __syncthreads();
    if (take_all) break;
  }
}

// Keeps the entries of [0, n) for which pred(key, id) holds, packed to the front in their
// original order; returns how many were kept (all threads).  Also leaves the smallest and the
// largest kept key in S.min_key / S.max_key.  Each thread owns CAP / NT consecutive entries.
template <class P>
__device__ inline unsigned keep_entries(Shared& S, uint32_t* ck, uint32_t* ci, unsigned n, P pred) {
  constexpr int PER = CAP / NT;
  const int tid = threadIdx.x;
  uint32_t k[PER], d[PER];
  unsigned cnt = 0, lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const unsigned i = (unsigned)tid * PER + j;
    k[j] = 0u; d[j] = 0u;
    if (i < n) { k[j] = ck[i]; d[j] = ci[i]; }
    if (k[j] && !pred(k[j], d[j])) k[j] = 0u;
    if (k[j]) { ++cnt; lo = min(lo, k[j]); hi = max(hi, k[j]); }
  }
  if (tid == 0) { S.min_key = 0xFFFFFFFFu; S.max_key = 0u; }
  unsigned total;
  const unsigned incl = block_incl_scan(cnt, S.scan_u32, total);  // barriers inside: all reads done
  if (cnt) { atomicMin(&S.min_key, lo); atomicMax(&S.max_key, hi); }
  unsigned pos = incl - cnt;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (k[j]) { ck[pos] = k[j]; ci[pos] = d[j]; ++pos; }
  }
  __syncthreads();
  return total;
}

// Monotone-threshold list maintenance: converts the new entries, keeps exactly the best
// min(k_sel, valid) in the order (y descending, id ascending) and raises the stream threshold to
// the smallest logit that can still beat the worst kept entry.  Entries arrive in ascending id,
// so a later element never wins a tie: the threshold is strict.
__device__ inline void compact(Shared& S, uint32_t* ck, uint32_t* ci, uint32_t* hist,
                               const History& H, bool apply_pen) {
  __syncthreads();
  const unsigned n = min(S.cand_count, (unsigned)CAP);
  const unsigned n_conv = S.n_conv;
  const unsigned n_valid = n_conv + convert_entries(S, ck, ci, n_conv, n, H, apply_pen);
  const unsigned k_sel = (unsigned)S.k_sel;
  unsigned long long prefix = 0ull;
  int shift = 64;
  if (n_valid > k_sel) select_composite(S, ck, ci, n, k_sel, hist, prefix, shift);
  const unsigned kept = keep_entries(S, ck, ci, n, [&](uint32_t key, uint32_t id) {
    return shift == 64 || (composite(key, id) >> shift) >= prefix;
  });
  if (threadIdx.x == 0) {
    S.cand_count = kept; S.n_conv = kept;
    S.g_pass = (kept == k_sel) ? min_z_reaching(keyf(S.min_key), S.tau, S.greedy, true) : -INFINITY;
  }
  __syncthreads();
}

// Bitonic sort of n (power of two) entries by composite; descending when `desc`.
__device__ inline void bitonic_sort(uint32_t* key, uint32_t* id, unsigned n, bool desc) {
  for (unsigned k = 2; k <= n; k <<= 1) {
    for (unsigned j = k >> 1; j > 0; j >>= 1) {
      for (unsigned i = threadIdx.x; i < n; i += NT) {
        const unsigned p = i ^ j;
        if (p > i) {
          const unsigned long long a = composite(key[i], id[i]), b = composite(key[p], id[p]);
          const bool up = ((i & k) == 0) == desc;  // this pair wants the larger composite first
          if (up ? (a < b) : (a > b)) {
            const uint32_t tk = key[i], ti = id[i];
            key[i] = key[p]; id[i] = id[p]; key[p] = tk; id[p] = ti;
          }
        }
      }
      __syncthreads();
    }
  }
}

struct Draws { double u_draw, u_acc, u_tail; };

// Exact selection, softmax and draw on the compacted candidate list (<= KMAX entries, the best of
// the row; `complete`: they are all of the prefix that matters).  Returns false when the list cannot certify the survivor set K_b.
__device__ inline bool finalize_small(Shared& S, uint32_t* ck, uint32_t* ci, bool complete, double S_total,
                                      const Draws& U, const uint32_t* __restrict__ hot_bits,
                                      simple_row_diag& dg) {
  const int tid = threadIdx.x;
  const unsigned n_c = S.cand_count;
  if (n_c == 0u || (S.flags & SIMPLE_DIAG_ERROR)) { if (tid == 0) S.flags |= SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT; return true; }
  unsigned npad = 2;
  while (npad < n_c) npad <<= 1;
  for (unsigned i = n_c + tid; i < npad; i += NT) { ck[i] = 0u; ci[i] = 0xFFFFFFFFu; }
  __syncthreads();
  bitonic_sort(ck, ci, npad, true);
  if (ck[0] == KEY_NEG_INF) { if (tid == 0) S.flags |= SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT; return true; }
  if (S.greedy) {
    if (tid == 0) { S.out_id = (int)ci[0]; S.out_p = 1.0f; }
    dg.n_survivors = 1;
    return true;
  }
  double* wv = reinterpret_cast<double*>(ck + KMAX);  // weights in sorted order (8 KB)
  const float y0 = keyf(ck[0]);
  // two consecutive entries per thread
  const unsigned i0 = 2u * tid, i1 = i0 + 1u;
  const double w0 = (i0 < n_c) ? exp((double)keyf(ck[i0]) - (double)y0) : 0.0;
  const double w1 = (i1 < n_c) ? exp((double)keyf(ck[i1]) - (double)y0) : 0.0;
  if (i0 < n_c) wv[i0] = w0;
  if (i1 < n_c) wv[i1] = w1;
  double tot;
  const double incl = block_incl_scan(w0 + w1, S.scan_d, tot);
  const double cum0 = incl - w1, cum1 = incl;  // inclusive prefix masses in sorted order
  const double S_k = complete ? tot : S_total;
  // min-p: how many listed entries satisfy y >= fl32(y_max + fl32(ln min_p))
  unsigned n_m = n_c;
  bool known = complete;
  if (S.min_p > 0.0f) {
    const float thr = y0 + (float)log((double)S.min_p);
    unsigned c = 0;
    if (i0 < n_c && keyf(ck[i0]) >= thr) ++c;
    if (i1 < n_c && keyf(ck[i1]) >= thr) ++c;
    n_m = block_sum(c, S.scan_u32);
    if (n_m < n_c) known = true;
  }
  unsigned n_p = n_c;
  if (S.top_p < 1.0f) {
    if (S.top_p <= 0.0f) { n_p = 1; known = true; }
    else {
      const double target = (double)S.top_p * S_k;
      unsigned c = 0;
      if (i0 < n_c && cum0 < target) ++c;
      if (i1 < n_c && cum1 < target) ++c;
      const unsigned n_lt = block_sum(c, S.scan_u32);
      if (n_lt < n_c) { n_p = n_lt + 1u; known = true; }
    }
  }
  if (!known) return false;
  const unsigned n = max(1u, min(n_c, min(n_m, n_p)));
  dg.n_survivors = (int)n;
  dg.s_k = S_k;
  // survivors -> ascending token id, payload = position in the sorted order
  __syncthreads();
  unsigned np2 = 2;
  while (np2 < n) np2 <<= 1;
  for (unsigned i = tid; i < np2; i += NT) {
    if (i < n) ck[i] = i; else { ck[i] = 0u; ci[i] = 0xFFFFFFFFu; }
  }
  __syncthreads();
  // ascending id == ascending composite of (key = 0, id) inverted: sort on id only
  for (unsigned k = 2; k <= np2; k <<= 1) {
    for (unsigned j = k >> 1; j > 0; j >>= 1) {
      for (unsigned i = tid; i < np2; i += NT) {
        const unsigned p = i ^ j;
        if (p > i) {
          const bool asc = ((i & k) == 0);
          const uint32_t a = ci[i], b = ci[p];
          if (asc ? (a > b) : (a < b)) {
            ci[i] = b; ci[p] = a;
            const uint32_t t = ck[i]; ck[i] = ck[p]; ck[p] = t;
          }
        }
      }
      __syncthreads();
    }
  }
  const bool use_hot = hot_bits != nullptr;
  double a0 = 0.0, a1 = 0.0;  // weights of this thread's two entries, ascending id
  bool h0 = false, h1 = false;
  if (i0 < n) { a0 = wv[ck[i0]]; if (use_hot) h0 = (hot_bits[ci[i0] >> 5] >> (ci[i0] & 31)) & 1u; }
  if (i1 < n) { a1 = wv[ck[i1]]; if (use_hot) h1 = (hot_bits[ci[i1] >> 5] >> (ci[i1] & 31)) & 1u; }
  double S_K;
  block_incl_scan(a0 + a1, S.scan_d, S_K);
  bool pick_hot = false;
  double S_H = 0.0, S_T = 0.0;
  if (use_hot) {
    block_incl_scan((h0 ? a0 : 0.0) + (h1 ? a1 : 0.0), S.scan_d, S_H);
    block_incl_scan((h0 ? 0.0 : a0) + (h1 ? 0.0 : a1), S.scan_d, S_T);
    pick_hot = (S_H > 0.0) && (U.u_acc * S_K <= S_H);
    dg.alpha = S_H / S_K;
    dg.flags |= SIMPLE_DIAG_SHVS | (pick_hot ? SIMPLE_DIAG_ACCEPTED : 0u);
  }
  // the walk: entries of the chosen class in ascending id, first running mass above the target
  const bool in0 = use_hot ? (h0 == pick_hot) : true, in1 = use_hot ? (h1 == pick_hot) : true;
  const double b0 = in0 ? a0 : 0.0, b1 = in1 ? a1 : 0.0;
  double cls_total;
  const double inclw = block_incl_scan(b0 + b1, S.scan_d, cls_total);
  const double total = use_hot ? (pick_hot ? S_H : S_T) : S_K;
  const double target = (use_hot ? (pick_hot ? U.u_draw : U.u_tail) : U.u_draw) * total;
  if (tid == 0) { S.found_lo = 0xFFFFFFFFu; S.found_hi = 0u; }
  __syncthreads();
  const double c0 = inclw - b1, c1 = inclw;
  if (i0 < n && in0 && b0 > 0.0) { if (c0 > target) atomicMin(&S.found_lo, i0); atomicMax(&S.found_hi, i0 + 1u); }
  if (i1 < n && in1 && b1 > 0.0) { if (c1 > target) atomicMin(&S.found_lo, i1); atomicMax(&S.found_hi, i1 + 1u); }
  __syncthreads();
  if (tid == 0) {
    unsigned pos = S.found_lo;
    if (pos == 0xFFFFFFFFu) pos = S.found_hi ? S.found_hi - 1u : 0u;  // rounding: last id of positive weight
    S.out_id = (int)ci[pos];
    S.out_p = (float)(wv[ck[pos]] / S_K);
  }
  return true;
}

// ------------------------------------------------------------------ sampled-threshold route ----
enum { ROUTE_DONE = 0, ROUTE_UNCERTIFIED = 1, ROUTE_RETRY = 2 };

// Columns that are in the history, taken from the history side (FULL rows mask them out of the
// stream): gather the raw logit, apply the penalties, add to the exp-sum and to the candidates.
template <typename DT>
__device__ inline void history_columns(const DT* __restrict__ rowp, const History& H, float g, bool do_sum,
                                       ExpSum& E, Shared& S, uint32_t* ck, uint32_t* ci) {
  for (int w = threadIdx.x; w < H.n_words; w += NT) {
    uint32_t bits = H.bits[w];
    if (!bits) continue;
    int r = H.grp[w >> 3];
    for (int j = w & ~7; j < w; ++j) r += __popc(H.bits[j]);
    while (bits) {
      const int b = __ffs((int)bits) - 1;
      bits &= bits - 1u;
      const int id = w * 32 + b;
      const uint32_t c = H.count_at(r++);
      float z = Elem<DT>::one(rowp + id);
      z = (z > 0.0f) ? z / H.rep : z * H.rep;
      if (c > 0u) { const float t = H.freq * (float)c; z = z - t; z = z - H.pres; }
      if (do_sum) { E.raise(z); E.s += (double)E.w(z); }
      if (!(z < g)) {
        const unsigned slot = atomicAdd(&S.cand_count, 1u);
        if (slot < (unsigned)CAP) { ck[slot] = __float_as_uint(z); ci[slot] = (uint32_t)id; }
      }
    }
  }
}

__device__ inline double combine_exp_sums(Shared& S, const ExpSum& E) {
  const float M = block_max(E.m, S.red_f);
  const float d = E.m - M;
  const double sc = (double)__builtin_amdgcn_exp2f(fmaf(d, E.c_hi, d * E.c_lo));
  return block_sum(E.s * sc, S.scan_d);
}

// One pass over the row with a threshold fixed from sample tiles.  The list ends up holding every
// element whose tempered value is >= y_f, so any prefix of the total order that ends at or above
// y_f is known exactly.  ROUTE_RETRY: the sampled threshold admitted fewer than k_sel elements or
// overflowed the list; ROUTE_UNCERTIFIED: K_b reaches below what the list holds.
template <typename DT, bool VEC, bool FULL>
__device__ inline int sampled_route(const DT* __restrict__ rowp, int V, const History& H, bool need_sum,
                                    Shared& S, uint32_t* ck, uint32_t* ci, uint32_t* hist, const Draws& U,
                                    const uint32_t* __restrict__ hot_bits, simple_row_diag& dg) {
  constexpr int EPL = Elem<DT>::EPL;
  constexpr int T = 64 * EPL * UNROLL;
  constexpr int NS = CAP / T;
  const int tid = threadIdx.x, wave = wave_id();
  const int ntiles = (V + T - 1) / T;
  const bool sampled_all = ntiles <= NS;
  ExpSum E{-3.4028234663852886e38f, 0.0, S.c_hi, S.c_lo};
  if (wave < min(NS, ntiles)) {
    const int ti = sampled_all ? wave : wave * (ntiles / NS);
    process_tile<DT, VEC, FULL, true>(rowp, ti * T, V, 0.0f, H, need_sum, E, S, ck, ci);
  }
  __syncthreads();
  const unsigned n_s = S.cand_count;  // <= NS * T = CAP
  const unsigned n_valid = convert_entries(S, ck, ci, 0u, n_s, H, !FULL);
  uint32_t key_f = 0u;
  float g = -INFINITY;
  unsigned kept;
  if (!sampled_all) {
    // rank of the threshold element in the sample: 1.5 x the expected rank of the k_sel-th largest
    // plus three standard deviations, so that the whole row holds >= k_sel elements above it
    const float m = (float)S.k_sel * (float)n_s / (float)V;
    const unsigned r = (unsigned)ceilf(1.5f * m + 3.0f * sqrtf(m) + 4.0f);
    if (n_valid <= r) return (S.flags & SIMPLE_DIAG_ERROR) ? ROUTE_DONE : ROUTE_RETRY;
    unsigned long long prefix; int shift;
    select_composite(S, ck, ci, n_s, r, hist, prefix, shift);
    key_f = (shift >= 32) ? (uint32_t)(prefix << (shift - 32)) : (uint32_t)(prefix >> (32 - shift));
    if (key_f <= KEY_NEG_INF) return ROUTE_RETRY;
    kept = keep_entries(S, ck, ci, n_s, [&](uint32_t key, uint32_t) { return key >= key_f; });
    if (!S.k_on && !S.greedy && S.min_p > 0.0f) {
      // min-p survivors lie within ln(min_p) of the row maximum, which is at least the sample's
      const float thr_lb = keyf(S.max_key) + (float)log((double)S.min_p);
      if (fkey(thr_lb) > key_f) {
        key_f = fkey(thr_lb);
        kept = keep_entries(S, ck, ci, kept, [&](uint32_t key, uint32_t) { return key >= key_f; });
      }
    }
    if (tid == 0) S.g_pass = min_z_reaching(keyf(key_f), S.tau, S.greedy, false);
  } else {
    kept = keep_entries(S, ck, ci, n_s, [&](uint32_t, uint32_t) { return true; });
    if (tid == 0) S.g_pass = -INFINITY;
  }
  if (tid == 0) { S.cand_count = kept; S.n_conv = kept; }
  __syncthreads();
  g = S.g_pass;
  if (!sampled_all) {
    for (int ti = wave; ti < ntiles; ti += NW) {
      if (is_sample_tile(ti, ntiles, NS)) continue;
      process_tile<DT, VEC, FULL, false>(rowp, ti * T, V, g, H, need_sum, E, S, ck, ci);
    }
  }
  if (FULL && H.active) history_columns<DT>(rowp, H, g, need_sum, E, S, ck, ci);
  __syncthreads();
  const unsigned total = S.cand_count;
  if (total > (unsigned)CAP) return ROUTE_RETRY;
  convert_entries(S, ck, ci, kept, total, H, !FULL);
  unsigned L = keep_entries(S, ck, ci, total, [&](uint32_t key, uint32_t) { return key >= key_f; });
  if (S.flags & SIMPLE_DIAG_ERROR) L = 0u;  // finalize reports the error
  const bool exact_k = S.k_on || S.greedy;
  if (!(S.flags & SIMPLE_DIAG_ERROR) && exact_k && L < (unsigned)S.k_sel) return ROUTE_RETRY;
  const unsigned n_keep = exact_k ? min(L, (unsigned)S.k_sel) : min(L, (unsigned)KMAX);
  if (L > n_keep) {
    unsigned long long prefix; int shift;
    select_composite(S, ck, ci, L, n_keep, hist, prefix, shift);
    keep_entries(S, ck, ci, L, [&](uint32_t key, uint32_t id) { return (composite(key, id) >> shift) >= prefix; });
  }
  if (tid == 0) { S.cand_count = n_keep; S.n_conv = n_keep; }
  const double S_total = need_sum ? combine_exp_sums(S, E) : 0.0;
  __syncthreads();
  const bool complete = exact_k || (sampled_all && L <= (unsigned)KMAX);
  return finalize_small(S, ck, ci, complete, S_total, U, hot_bits, dg) ? ROUTE_DONE : ROUTE_UNCERTIFIED;
}

// ------------------------------------------------------------------ multi-pass route -----------
template <typename DT>
struct RowReader {
  const DT* p; int V; float tau; bool greedy; const History* H;
  __device__ __forceinline__ float load(int idx) const { return Elem<DT>::one(p + idx); }
  // Sixteen bytes from column idx on (a multiple of Elem<DT>::EPL, the row 16-byte aligned).
  __device__ __forceinline__ u32x4 load16(int idx) const {
    typedef __attribute__((address_space(1))) const DT GlobDT;
    typedef __attribute__((address_space(1))) const u32x4 GlobVec;
    return *(GlobVec*)((GlobDT*)p + idx);
  }
  static __device__ __forceinline__ void unpack(const u32x4& q, float (&z)[Elem<DT>::EPL]) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if constexpr (sizeof(DT) == 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = __uint_as_float(w[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) { z[2 * i] = __uint_as_float(w[i] << 16); z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
  }
  // Key of the tempered value z / tau; 0 for NaN / +inf.
  __device__ __forceinline__ uint32_t key_plain(float z) const {
    if (z != z || z == INFINITY) return 0u;
    const float y = greedy ? z : z / tau;
    return (y == INFINITY) ? 0u : fkey(y);
  }
  // The same for column idx whose raw logit is z, after the penalties of a history column.  The
  // penalty is inlined: a call would wait for every load the caller has in flight.
  __device__ __forceinline__ uint32_t key_of(float z, int idx) const {
    if (H->active && H->test(idx)) z = H->penalise_inline(z, idx);
    return key_plain(z);
  }
  // Bit j set: column base + 64 j + lane is a history column (or lies beyond the row).
  template <int N>
  __device__ __forceinline__ uint32_t history_mask(int base, int lane) const {
    uint32_t m = 0u;
    if (H->active) {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int c = min(base + j * 64 + lane, V - 1);
        m |= ((H->bits[c >> 5] >> (c & 31)) & 1u) << j;
      }
    }
    return m;
  }
  // g(z', idx) for the history columns, z' the penalised logit, one column per thread at a time.  A
  // penalised column costs a rank (up to eight mask words), a count and a division; met inside the
  // stream, one such column holds up the 64 lanes of its wave, and with a few thousand distinct ids
  // most groups of 64 columns hold one.
  template <class G>
  __device__ __forceinline__ void history_columns_raw(G g) const {
    if (!H->active) return;
    for (int w = threadIdx.x; w < H->n_words; w += NT) {
      uint32_t b = H->bits[w];
      while (b) {
        const int idx = (w << 5) + __builtin_ctz(b);
        b &= b - 1u;
        if (idx < V) g(H->penalise_inline(load(idx), idx), idx);
      }
    }
  }
  template <class F>
  __device__ __forceinline__ void history_columns(F f) const {
    history_columns_raw([&](float z, int idx) { f(key_plain(z), idx); });
  }
  // The smallest logit after penalties (as a key) whose tempered key is >= K, KEY_POS_INF if no finite
  // one is: tempering is monotone, so {key >= K} is {z' >= keyf(result)} and a pass can sort columns
  // by a float compare, dividing by tau only for those it keeps.  (A quotient that overflows counts
  // as above K; rows that hold one never get this far.)
  __device__ __noinline__ uint32_t z_lower_bound(uint32_t K) const {
    uint32_t lo = KEY_NEG_INF, hi = KEY_POS_INF;
    while (lo < hi) {
      const uint32_t mid = lo + ((hi - lo) >> 1);
      const uint32_t k = key_plain(keyf(mid));
      if (k == 0u || k >= K) hi = mid; else lo = mid + 1u;
    }
    return lo;
  }
  __device__ __forceinline__ uint32_t ykey(int idx) const { return key_of(load(idx), idx); }
};
// The reader reaches these functions by reference, that is through memory; every element would pay
// for a chain of dependent loads (reader -> history -> mask word).  The routes below therefore work
// on a copy whose fields are wave-uniform values held in scalar registers (every thread of the
// workgroup serves the same row).
template <class T> __device__ __forceinline__ T* uni_ptr(T* q) {
  const unsigned long long v = (unsigned long long)q;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}
// For a pointer into the workgroup's LDS: the same, with the address space stated, so that accesses
// through it are LDS instructions and wait on no global load in flight.
template <class T> __device__ __forceinline__ T* uni_lds_ptr(T* q) {
  T* const u = uni_ptr(q);
#if defined(__HIP_DEVICE_COMPILE__)  // the builtin exists in the device pass only
  __builtin_assume(__builtin_amdgcn_is_shared(u));
#endif
  return u;
}
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint32_t uni(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ float uni(float x) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x))); }
__device__ __forceinline__ History uniform_copy(const History& h) {
  History o;
  o.bits = uni_lds_ptr(h.bits); o.grp = uni_lds_ptr(h.grp); o.cnt = uni_lds_ptr(h.cnt);
  o.n_words = uni(h.n_words); o.distinct = uni(h.distinct);
  o.rep = uni(h.rep); o.freq = uni(h.freq); o.pres = uni(h.pres);
  o.active = uni((int)h.active) != 0;
  return o;
}
template <typename DT>
__device__ __forceinline__ RowReader<DT> uniform_copy(const RowReader<DT>& r, const History* h) {
  return RowReader<DT>{uni_ptr(r.p), uni(r.V), uni(r.tau), uni((int)r.greedy) != 0, h};
}

// Stream of a 16-byte aligned row in groups of VGROUP columns, wave w taking groups w, w + NW, ...:
// g(z, idx) for every column of the full groups that is outside the history, then after_group(grp)
// with all lanes active.  A lane reads 16 bytes at a time and two groups are in flight per wave, in
// two register sets that take turns (no copy between them, so nothing waits for the group just
// requested).  The columns past the last full group are the caller's.
constexpr int VGROUP = 1024;
template <typename DT, class G, class AG>
__device__ __forceinline__ void scan_groups_vec(const RowReader<DT>& R, G g, AG after_group) {
  constexpr int EPL = Elem<DT>::EPL, NV = VGROUP / (64 * EPL);
  const int lane = lane_id();
  const int n_full = R.V / VGROUP;
  const History& H = *R.H;
  u32x4 qa[NV], qb[NV];
  auto fetch = [&](u32x4 (&q)[NV], int grp) {
#pragma unroll
    for (int j = 0; j < NV; ++j) q[j] = R.load16(grp * VGROUP + (j * 64 + lane) * EPL);
  };
  auto work = [&](const u32x4 (&q)[NV], int grp) {
    uint32_t hm[NV];  // history bits of the lane's columns (EPL consecutive columns share a mask word)
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx0 = grp * VGROUP + (j * 64 + lane) * EPL;
      hm[j] = H.active ? (H.bits[idx0 >> 5] >> (idx0 & 31)) : 0u;
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx0 = grp * VGROUP + (j * 64 + lane) * EPL;
      float z[EPL];
      RowReader<DT>::unpack(q[j], z);
#pragma unroll
      for (int e = 0; e < EPL; ++e)
        if (!((hm[j] >> e) & 1u)) g(z[e], idx0 + e);
    }
    after_group(grp);
  };
  int grp = uni(wave_id());
  if (grp >= n_full) return;
  fetch(qa, grp);
  for (;;) {
    const bool more_b = grp + NW < n_full;
    if (more_b) fetch(qb, grp + NW);
    work(qa, grp);
    if (!more_b) break;
    grp += NW;
    const bool more_a = grp + NW < n_full;
    if (more_a) fetch(qa, grp + NW);
    work(qb, grp);
    if (!more_a) break;
    grp += NW;
  }
}

// g(z', idx) for every column of the row, z' the logit after the penalties, in no particular order:
// the columns outside the history from the stream, then the history columns.  Each lane keeps two
// groups of SCAN_U loads going: the next group is requested before the current one is worked on.
// A group that lies inside the row (all but the last) runs without per-column bounds checks.
constexpr int SCAN_U = 8;
template <typename DT, bool VEC, class G>
__device__ __forceinline__ void scan_row_raw(const RowReader<DT>& R, G g) {
  const int lane = lane_id(), V = R.V;
  if constexpr (VEC) {  // aligned rows: 16-byte loads; the columns past the last full group one per thread
    scan_groups_vec(R, g, [](int) {});
    for (int idx = (V / VGROUP) * VGROUP + (int)threadIdx.x; idx < V; idx += NT)
      if (!(R.H->active && R.H->test(idx))) g(R.load(idx), idx);
    R.history_columns_raw(g);
    return;
  }
  constexpr int GROUP = 64 * SCAN_U, STEP = NW * GROUP;
  float cur[SCAN_U], nxt[SCAN_U];
  auto fetch = [&](float (&z)[SCAN_U], int b) {
    if (b + GROUP <= V) {
#pragma unroll
      for (int j = 0; j < SCAN_U; ++j) z[j] = R.load(b + j * 64 + lane);
    } else {
#pragma unroll
      for (int j = 0; j < SCAN_U; ++j) {
        const int idx = b + j * 64 + lane;
        z[j] = (idx < V) ? R.load(idx) : 0.0f;
      }
    }
  };
  int base = uni(wave_id() * GROUP);
  if (base < V) fetch(cur, base);
  for (; base < V; base += STEP) {
    if (base + STEP < V) fetch(nxt, base + STEP);
    const uint32_t hm = R.template history_mask<SCAN_U>(base, lane);
    if (base + GROUP <= V) {
#pragma unroll
      for (int j = 0; j < SCAN_U; ++j)
        if (!((hm >> j) & 1u)) g(cur[j], base + j * 64 + lane);
    } else {
#pragma unroll
      for (int j = 0; j < SCAN_U; ++j) {
        const int idx = base + j * 64 + lane;
        if (idx < V && !((hm >> j) & 1u)) g(cur[j], idx);
      }
    }
#pragma unroll
    for (int j = 0; j < SCAN_U; ++j) cur[j] = nxt[j];
  }
  R.history_columns_raw(g);
}
// f(key, idx) for every column, key that of the tempered value (0 for NaN / +inf).
template <typename DT, bool VEC, class F>
__device__ __forceinline__ void scan_row(const RowReader<DT>& R, F f) {
  scan_row_raw<DT, VEC>(R, [&](float z, int idx) { f(R.key_plain(z), idx); });
}

struct Cut {  // the prefix {key > t} plus the first r (by id) of {key == t}
  uint32_t t; uint32_t cnt_gt; unsigned long long mass_gt; uint32_t cnt_eq; uint32_t r; unsigned long long q_t;
};

// Fixed-point mass of a column, the nearest integer to exp(y - ymax) * 2^QBITS, as a function of the
// key alone (every pass must give a column the same mass).  The exponential is 2^n * 2^f with
// n = rint(x log2 e) and a degree-10 polynomial for 2^f on [-1/2, 1/2]: relative error below 1e-12,
// five orders under the tolerance on probabilities, at a quarter of the library routine's
// double-precision instructions.  Below x = -44 the mass rounds to zero.
__device__ __forceinline__ unsigned long long qmass(uint32_t key, float ymax) {
  const double x = (double)keyf(key) - (double)ymax;
  if (!(x >= -44.0)) return 0ull;
  const double t = x * 1.4426950408889634;
  const double n = rint(t), f = t - n;
  double p = 7.054911620801121e-09;
  p = fma(p, f, 1.0178086009239696e-07);
  p = fma(p, f, 1.3215486790144305e-06);
  p = fma(p, f, 1.5252733804059838e-05);
  p = fma(p, f, 0.00015403530393381606);
  p = fma(p, f, 0.0013333558146428441);
  p = fma(p, f, 0.009618129107628477);
  p = fma(p, f, 0.055504108664821576);
  p = fma(p, f, 0.2402265069591007);
  p = fma(p, f, 0.6931471805599453);
  p = fma(p, f, 1.0);
  // below 2^(QBITS + 1) for x <= 0; adding 2^52 rounds it to the nearest integer (ties to even) and
  // leaves that integer in the low 52 bits of the sum
  const double v = ldexp(p, (int)n + QBITS) + 0x1p52;
  return (unsigned long long)__double_as_longlong(v) & 0x000FFFFFFFFFFFFFull;
}

// Radix descent over the 32-bit key of y (three levels: 11, 11, 10 bits) with exact integer
// histograms.  BY_MASS = false: counts only; finds the key of the need_cnt-th largest element (the
// cut's masses stay 0).  BY_MASS = true: fixed-point masses too; finds the key at which the running
// mass (largest first) reaches top_p times the mass of everything the descent covers, and stores
// that mass in *covered.  `lim` (optional) restricts the descent to the prefix described by
// another cut.  When the bin chosen at the first level holds no more than LIST_CAP keys, the second
// level's pass sets them aside in LDS (the 16 KB after the mass histogram) and the third level reads
// them there instead of the row.
constexpr unsigned LIST_CAP = 4096u;
template <typename DT, bool VEC, bool BY_MASS>
__device__ __noinline__ Cut descend(const RowReader<DT>& R_in, Shared& S, uint32_t* hcnt_in,
                              unsigned long long* hmass_in, float ymax_in,
                              uint32_t need_cnt, float top_p, unsigned long long* covered, const Cut* lim_in) {
  constexpr bool by_mass = BY_MASS;
  double T = 0.0;
  const int tid = threadIdx.x;
  const History Hs = uniform_copy(*R_in.H);
  const RowReader<DT> R = uniform_copy(R_in, &Hs);
  uint32_t* const hcnt = uni_lds_ptr(hcnt_in);
  unsigned long long* const hmass = uni_lds_ptr(hmass_in);
  const float ymax = uni(ymax_in);
  Cut lim_copy = {0u, 0u, 0ull, 0u, 0u, 0ull};
  if (lim_in) { lim_copy = *lim_in; lim_copy.t = uni(lim_copy.t); }
  const Cut* const lim = lim_in ? &lim_copy : nullptr;
  uint32_t* const list = reinterpret_cast<uint32_t*>(hmass + NBINS);
  typedef __attribute__((address_space(3))) unsigned LdsU32;
  LdsU32* const list_n = (LdsU32*)&S.list_n;  // LDS-typed: the add must not count as a global access
  uint32_t prefix = 0u, base_c = 0u;
  unsigned long long base_m = 0ull;
  uint32_t need = need_cnt;
  const int widths[3] = {11, 11, 10};
  int shift = 32;
  unsigned in_bin = 0xFFFFFFFFu;  // keys in the bin the level before chose
  bool listed = false;
  for (int lvl = 0; lvl < 3; ++lvl) {
    const int w = widths[lvl];
    shift -= w;
    for (int i = tid; i < NBINS; i += NT) { hcnt[i] = 0u; if (by_mass) hmass[i] = 0ull; }
    // (S.sel_found is not cleared between levels: a wave may still be reading the level before's
    // verdict when thread 0 gets here, so each level marks its hit with its own number instead)
    if (tid == 0) { if (lvl == 0) S.sel_found = 0u; if (lvl == 1) S.list_n = 0u; }
    __syncthreads();
    auto tally = [&](uint32_t key) {
      const unsigned d = (key >> shift) & ((1u << w) - 1u);
      atomicAdd(&hcnt[d], 1u);
      if (by_mass) atomicAdd(&hmass[d], qmass(key, ymax));
    };
    if (listed) {  // third level, from the keys the second set aside (all of them inside the limit)
      const unsigned n_list = S.list_n;
      for (unsigned i = tid; i < n_list; i += NT) {
        const uint32_t key = list[i];
        if ((key >> (shift + w)) == prefix) tally(key);
      }
    } else {
      const bool collect = (lvl == 1) && (in_bin <= LIST_CAP);
      // the keys this level looks at, [prefix << (shift + w), (prefix + 1) << (shift + w)) and not
      // below the limit, as a range of z'
      float z_from = -INFINITY, z_below = INFINITY;
      if (lvl > 0) {
        const unsigned long long k_end = (unsigned long long)(prefix + 1u) << (shift + w);
        z_from = uni(keyf(R.z_lower_bound(prefix << (shift + w))));
        if (k_end <= 0xFFFFFFFFull) z_below = uni(keyf(R.z_lower_bound((uint32_t)k_end)));
      }
      if (lim) z_from = fmaxf(z_from, uni(keyf(R.z_lower_bound(lim->t))));
      scan_row_raw<DT, VEC>(R, [&](float z, int) {
        if (!(z >= z_from && z < z_below)) return;
        const uint32_t key = R.key_plain(z);
        if (!key) return;
        tally(key);
        if (collect) {  // (ties the limit leaves out are met here too, so the count can pass in_bin)
          const unsigned slot = __hip_atomic_fetch_add(list_n, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if (slot < LIST_CAP) list[slot] = key;
        }
      });
      __syncthreads();
      listed = collect && (S.list_n <= LIST_CAP);
    }
    __syncthreads();
    if (lim && tid == 0 && (lvl == 0 || (lim->t >> (shift + w)) == prefix)) {
      const unsigned d = (lim->t >> shift) & ((1u << w) - 1u);  // ties beyond the limit's r do not count
      hcnt[d] -= (lim->cnt_eq - lim->r);
      if (by_mass) hmass[d] -= (unsigned long long)(lim->cnt_eq - lim->r) * lim->q_t;
    }
    __syncthreads();
    unsigned lc[4], tc = 0;
    unsigned long long lm[4], tm = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lc[j] = hcnt[4 * tid + j]; lm[j] = by_mass ? hmass[4 * tid + j] : 0ull;
      tc += lc[j]; tm += lm[j];
    }
    unsigned totc; unsigned long long totm = 0ull;
    const unsigned ic = block_incl_scan(tc, S.scan_u32, totc);
    const unsigned long long im = by_mass ? block_incl_scan(tm, S.scan_u64, totm) : 0ull;
    if (by_mass && lvl == 0) {  // the first level's histogram holds everything the descent covers
      T = (double)top_p * (double)totm;
      if (covered) *covered = totm;
    }
    unsigned above_c = totc - ic;
    unsigned long long above_m = totm - im;
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      bool hit;
      if (by_mass) hit = ((double)(base_m + above_m) < T) && (T <= (double)(base_m + above_m + lm[j]));
      else hit = (above_c < need) && (need <= above_c + lc[j]);
      if (hit) {
        S.sel_digit = 4 * tid + j; S.sel_above_cnt = above_c; S.sel_above_mass = above_m;
        S.sel_cnt = lc[j]; S.sel_found = (unsigned)lvl + 1u;
      }
      above_c += lc[j]; above_m += lm[j];
    }
    __syncthreads();
    if (S.sel_found != (unsigned)lvl + 1u) {  // cannot happen for consistent inputs; fail the row rather than guess
      if (tid == 0) S.flags |= SIMPLE_DIAG_ERROR;
      __syncthreads();  // (the caller reads the flag in every thread)
      Cut bad = {KEY_POS_INF, 0u, 0ull, 0u, 0u, 0ull};
      return bad;
    }
    prefix = (prefix << w) | uni((uint32_t)S.sel_digit);
    in_bin = uni((uint32_t)S.sel_cnt);
    base_c += S.sel_above_cnt;
    base_m += S.sel_above_mass;
    if (!by_mass) need -= S.sel_above_cnt;
  }
  Cut c;
  c.t = prefix; c.cnt_gt = base_c; c.mass_gt = base_m; c.cnt_eq = S.sel_cnt; c.q_t = qmass(prefix, ymax);
  c.r = 0u;
  __syncthreads();
  return c;
}

// Exact route for any row: survivor set as a cut (t, r), then the inverse-CDF walk in ascending
// id through per-chunk masses.  `lds` is the candidate-list region (32 KB), free on this route.
// Bit idx of the hot-set mask (device memory), read through a global-typed pointer.
__device__ __forceinline__ int hot_bit(const uint32_t* hot_bits, int idx) {
  typedef __attribute__((address_space(1))) const uint32_t GlobU32;
  return (int)((*((GlobU32*)hot_bits + (idx >> 5)) >> (idx & 31)) & 1u);
}

template <typename DT, bool VEC>
__device__ __noinline__ void wide_route(const RowReader<DT>& R_in, Shared& S, uint32_t* hist, unsigned char* lds_in,
                                  const Draws& U, const uint32_t* __restrict__ hot_bits_in,
                                  simple_row_diag& dg, const bool want_s_k) {
  const History Hs = uniform_copy(*R_in.H);
  const RowReader<DT> R = uniform_copy(R_in, &Hs);
  unsigned char* const lds = uni_lds_ptr(lds_in);
  const uint32_t* const hot_bits = uni_ptr(hot_bits_in);
  const int tid = threadIdx.x, lane = lane_id(), V = R.V;
  unsigned long long* hmass = reinterpret_cast<unsigned long long*>(lds);  // 16 KB
  // pass A: row maximum and validity
  // (tempering is monotone and rounds correctly, so the largest key is the key of the largest z')
  float mz = -INFINITY; unsigned bad = 0u;
  scan_row_raw<DT, VEC>(R, [&](float z, int) { if (z != z || z == INFINITY) bad = 1u; mz = fmaxf(mz, z); });
  const uint32_t mk = R.key_plain(mz);
  if (!mk) bad = 1u;  // z' / tau overflows
  {
    __syncthreads();
    if (tid == 0) { S.found_hi = 0u; S.flag_ws = 0u; }
    __syncthreads();
    atomicMax(&S.found_hi, mk);
    if (bad) atomicOr(&S.flag_ws, 1u);
    __syncthreads();
  }
  const uint32_t maxkey = uni((uint32_t)S.found_hi);
  if (S.flag_ws || maxkey <= KEY_NEG_INF) { if (tid == 0) S.flags |= SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT; return; }
  const float ymax = uni(keyf(maxkey));
  if (S.greedy) {  // lowest id attaining the maximum
    if (tid == 0) S.found_lo = 0xFFFFFFFFu;
    __syncthreads();
    scan_row<DT, VEC>(R, [&](uint32_t key, int idx) { if (key == maxkey) atomicMin(&S.found_lo, (unsigned)idx); });
    __syncthreads();
    if (tid == 0) { S.out_id = (int)S.found_lo; S.out_p = 1.0f; }
    dg.n_survivors = 1;
    return;
  }
  // pass D: size of the min-p prefix (every column is a valid key here, so without min-p it is V)
  const uint32_t thr_key = uni((S.min_p > 0.0f) ? fkey(ymax + (float)log((double)S.min_p)) : KEY_NEG_INF);
  unsigned n_m = (unsigned)V;
  if (S.min_p > 0.0f) {
    const float z_thr = uni(keyf(R.z_lower_bound(thr_key)));
    unsigned c_ge = 0;
    scan_row_raw<DT, VEC>(R, [&](float z, int) { if (z >= z_thr) ++c_ge; });
    n_m = block_sum(c_ge, S.scan_u32);
  }
  // top-k prefix
  Cut ck_;
  if (S.k_on) {
    ck_ = descend<DT, VEC, false>(R_in, S, hist, hmass, ymax, (uint32_t)S.top_k, 0.0f, nullptr, nullptr);
    if (S.flags & SIMPLE_DIAG_ERROR) return;
    ck_.r = (uint32_t)S.top_k - ck_.cnt_gt;
  }
  const unsigned n_k = S.k_on ? (unsigned)S.top_k : (unsigned)V;
  // nucleus inside the top-k prefix; the descent also measures S_k, the mass of that prefix
  Cut cp_; unsigned n_p = n_k;
  bool have_p = false;
  unsigned long long S_k = 0ull;
  if (S.top_p < 1.0f && S.top_p > 0.0f) {
    cp_ = descend<DT, VEC, true>(R_in, S, hist, hmass, ymax, 0u, S.top_p, &S_k, S.k_on ? &ck_ : nullptr);
    if (S.flags & SIMPLE_DIAG_ERROR) return;
    const double T = (double)S.top_p * (double)S_k;
    // smallest r >= 1 with mass_gt + r * q_t >= T
    double rr = ceil((T - (double)cp_.mass_gt) / (double)cp_.q_t);
    unsigned r = (rr < 1.0) ? 1u : (rr > (double)cp_.cnt_eq ? cp_.cnt_eq : (unsigned)rr);
    while (r > 1u && (double)(cp_.mass_gt + (unsigned long long)(r - 1u) * cp_.q_t) >= T) --r;
    while (r < cp_.cnt_eq && (double)(cp_.mass_gt + (unsigned long long)r * cp_.q_t) < T) ++r;
    cp_.r = r;
    n_p = cp_.cnt_gt + r;
    have_p = true;
  } else {
    if (S.top_p <= 0.0f) n_p = 1u;
    if (want_s_k) {  // reported only: the mass above the top-k cut plus its admitted ties, or of the whole row
      const float z_k = uni(S.k_on ? keyf(R.z_lower_bound(ck_.t)) : -INFINITY);
      const uint32_t t_k = uni(S.k_on ? ck_.t : 0u);
      unsigned long long m_gt = 0ull;
      scan_row_raw<DT, VEC>(R, [&](float z, int) {
        if (!(z >= z_k)) return;
        const uint32_t key = R.key_plain(z);
        if (key > t_k) m_gt += qmass(key, ymax);
      });
      S_k = block_sum(m_gt, S.scan_u64) + (S.k_on ? (unsigned long long)ck_.r * ck_.q_t : 0ull);
    }
  }
  const unsigned n = max(1u, min(n_k, min(n_m, n_p)));
  Cut cut;
  if (n == 1u && !(have_p && n_p == 1u) && !(S.k_on && n_k == 1u)) {
    // the single best token: lowest id at the maximum; how many columns tie there is not known, so the
    // count is set past any r and the walk below looks for the first of them
    cut = Cut{maxkey, 0u, 0ull, 0xFFFFFFFFu, 1u, 1ull << QBITS};
  } else if (have_p && n == n_p) {
    cut = cp_;
  } else if (S.k_on && n == n_k) {
    cut = ck_;
  } else {  // the min-p prefix {key >= thr_key}, or everything
    cut = Cut{thr_key - 1u, n_m, 0ull, 0u, 0u, 0ull};
  }
  cut.t = uni(cut.t); cut.r = uni(cut.r); cut.cnt_eq = uni(cut.cnt_eq);
  dg.n_survivors = (int)n;
  dg.s_k = (double)S_k * (1.0 / (double)(1ull << QBITS));
  __syncthreads();
  // pass F1: per-chunk survivor mass (class 0 = tail / everything, class 1 = hot) and tie counts
  const bool use_hot = hot_bits != nullptr;
  // (an aligned row of up to 2^20 columns: a chunk is one group of the vector stream)
  const bool by_groups = VEC && V <= VGROUP * 1024;
  int J = by_groups ? VGROUP / 64 : 8;
  while ((long long)64 * J * 1024 < (long long)V) J <<= 1;
  const int CH = 64 * J, NC = (V + CH - 1) / CH;
  unsigned long long* cm = reinterpret_cast<unsigned long long*>(lds);  // [2][NC]
  unsigned* ct = reinterpret_cast<unsigned*>(lds + (size_t)16 * NC);   // [2][NC]
  const float z_cut = uni(keyf(R.z_lower_bound(cut.t)));  // {key >= cut.t} as a compare of z'
  if (by_groups) {
    unsigned long long m[2] = {0ull, 0ull}; unsigned t[2] = {0u, 0u};
    auto column = [&](float z, int idx) {
      if (!(z >= z_cut)) return;
      const uint32_t key = R.key_plain(z);
      if (key >= cut.t && key) {
        const int cls = use_hot ? hot_bit(hot_bits, idx) : 0;
        if (key > cut.t) m[cls] += qmass(key, ymax); else t[cls] += 1u;
      }
    };
    auto chunk_done = [&](int c) {
#pragma unroll
      for (int x = 0; x < 2; ++x) { m[x] = wave_sum(m[x]); t[x] = wave_sum(t[x]); }
      if (lane == 0) { cm[c] = m[0]; cm[NC + c] = m[1]; ct[c] = t[0]; ct[NC + c] = t[1]; }
      m[0] = m[1] = 0ull; t[0] = t[1] = 0u;
    };
    scan_groups_vec(R, column, chunk_done);
    if (V % VGROUP != 0 && wave_id() == 0) {  // the columns past the last full group: the last chunk
      for (int idx = (V / VGROUP) * VGROUP + lane; idx < V; idx += 64)
        if (!(R.H->active && R.H->test(idx))) column(R.load(idx), idx);
      chunk_done(NC - 1);
    }
  } else
  for (int c = wave_id(); c < NC; c += NW) {
    unsigned long long m[2] = {0ull, 0ull}; unsigned t[2] = {0u, 0u};
    for (int j0 = 0; j0 < J; j0 += 8) {  // J is a multiple of 8; the eight loads go out together
      float z[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int idx = c * CH + (j0 + j) * 64 + lane;
        z[j] = (idx < V) ? R.load(idx) : 0.0f;
      }
      const uint32_t hm = R.template history_mask<8>(c * CH + j0 * 64, lane);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int idx = c * CH + (j0 + j) * 64 + lane;
        if (idx < V && !((hm >> j) & 1u) && z[j] >= z_cut) {
          const uint32_t key = R.key_plain(z[j]);
          if (key >= cut.t && key) {
            const int cls = use_hot ? hot_bit(hot_bits, idx) : 0;
            if (key > cut.t) m[cls] += qmass(key, ymax); else t[cls] += 1u;
          }
        }
      }
    }
#pragma unroll
    for (int x = 0; x < 2; ++x) { m[x] = wave_sum(m[x]); t[x] = wave_sum(t[x]); }
    if (lane == 0) { cm[c] = m[0]; cm[NC + c] = m[1]; ct[c] = t[0]; ct[NC + c] = t[1]; }
  }
  __syncthreads();
  R.history_columns([&](uint32_t key, int idx) {  // the history columns join their chunks
    if (key >= cut.t && key) {
      const int cls = use_hot ? hot_bit(hot_bits, idx) : 0, c = idx / CH;
      if (key > cut.t) atomicAdd(&cm[cls * NC + c], qmass(key, ymax)); else atomicAdd(&ct[cls * NC + c], 1u);
    }
  });
  __syncthreads();
  // which chunk holds the r-th tie (ties are admitted in ascending id)
  if (tid == 0) {
    int tc = NC;  // all ties admitted
    unsigned seen = 0;
    if (cut.r < cut.cnt_eq) {
      tc = -1;
      for (int c = 0; c < NC; ++c) {
        const unsigned here = ct[c] + ct[NC + c];
        if (seen + here > cut.r) { tc = c; break; }
        seen += here;
      }
      if (tc < 0) tc = NC;
    }
    S.tie_chunk = tc; S.walk_ties_before = seen; S.adm_split[0] = 0u; S.adm_split[1] = 0u;
  }
  __syncthreads();
  const int tie_chunk = S.tie_chunk;
  if (tie_chunk < NC && wave_id() == 0) {  // split of the admitted ties of that chunk by class
    unsigned left = cut.r - S.walk_ties_before, a[2] = {0u, 0u};
    for (int j = 0; j < J; ++j) {
      const int idx = tie_chunk * CH + j * 64 + lane;
      const bool tie = (idx < V) && (R.ykey(idx) == cut.t);
      const unsigned long long mask = __ballot(tie);
      const unsigned rank = __popcll(mask & ((1ull << lane) - 1ull));
      if (tie && rank < left) {
        const int cls = use_hot ? hot_bit(hot_bits, idx) : 0;
        a[cls] += 1u;
      }
      const unsigned here = __popcll(mask);
      left = (here >= left) ? 0u : left - here;
    }
    a[0] = wave_sum(a[0]); a[1] = wave_sum(a[1]);
    if (lane == 0) { S.adm_split[0] = a[0]; S.adm_split[1] = a[1]; }
  }
  __syncthreads();
  unsigned long long part[2] = {0ull, 0ull};
  for (int c = tid; c < NC; c += NT) {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const unsigned adm = (c < tie_chunk) ? ct[x * NC + c] : (c == tie_chunk ? S.adm_split[x] : 0u);
      const unsigned long long tot = cm[x * NC + c] + (unsigned long long)adm * cut.q_t;
      cm[x * NC + c] = tot;
      part[x] += tot;
    }
  }
  const unsigned long long S0 = block_sum(part[0], S.scan_u64);
  const unsigned long long S1 = block_sum(part[1], S.scan_u64);
  const unsigned long long SK = S0 + S1;
  int cls = 0;
  double u = U.u_draw;
  if (use_hot) {
    const bool acc = (S1 > 0ull) && (U.u_acc * (double)SK <= (double)S1);
    cls = acc ? 1 : 0;
    u = acc ? U.u_draw : U.u_tail;
    dg.alpha = (double)S1 / (double)SK;
    dg.flags |= SIMPLE_DIAG_SHVS | (acc ? SIMPLE_DIAG_ACCEPTED : 0u);
  }
  const unsigned long long Scls = cls ? S1 : S0;
  const double target = u * (double)Scls;
  if (tid == 0) {
    unsigned long long cum = 0ull; unsigned ties = 0u;
    int wc = -1, last_c = 0; unsigned long long last_cum = 0ull; unsigned last_ties = 0u;
    for (int c = 0; c < NC; ++c) {
      const unsigned long long here = cm[cls * NC + c];
      if (here > 0ull) { last_c = c; last_cum = cum; last_ties = ties; }
      if ((double)(cum + here) > target) { wc = c; break; }
      cum += here;
      ties += ct[c] + ct[NC + c];
    }
    if (wc < 0) { wc = last_c; cum = last_cum; ties = last_ties; }  // rounding: last chunk with mass
    S.walk_chunk = wc; S.walk_base = cum; S.walk_ties_before = ties; S.out_id = -1;
  }
  __syncthreads();
  if (wave_id() == 0) {  // pass F2: walk inside one chunk
    const int wc = S.walk_chunk;
    unsigned long long base = S.walk_base;
    unsigned ties_before = S.walk_ties_before;
    bool done = false;
    int last_id = -1; unsigned long long last_q = 0ull;
    for (int j = 0; j < J && !done; ++j) {
      const int idx = wc * CH + j * 64 + lane;
      uint32_t key = 0u;
      if (idx < V) key = R.ykey(idx);
      const bool tie = key && (key == cut.t);
      const unsigned long long tmask = __ballot(tie);
      const unsigned trank = ties_before + __popcll(tmask & ((1ull << lane) - 1ull));
      unsigned long long q = 0ull;
      if (key) {
        const int c = use_hot ? hot_bit(hot_bits, idx) : 0;
        if (c == cls) {
          if (key > cut.t) q = qmass(key, ymax);
          else if (tie && trank < cut.r) q = cut.q_t;
        }
      }
      const unsigned long long incl = wave_incl_scan(q);
      const bool hit = (q > 0ull) && ((double)(base + incl) > target);
      const unsigned long long hmask = __ballot(hit);
      if (hmask) {
        const int src = __ffsll((long long)hmask) - 1;
        const int id = __shfl(idx, src, 64);
        const unsigned long long qq = __shfl(q, src, 64);
        if (lane == 0) { S.out_id = id; S.out_p = (float)((double)qq / (double)SK); }
        done = true;
      } else {
        const unsigned long long pmask = __ballot(q > 0ull);
        if (pmask) {
          const int src = 63 - __clzll((long long)pmask);
          last_id = __shfl(idx, src, 64); last_q = __shfl(q, src, 64);
        }
        base += __shfl(incl, 63, 64);
        ties_before += __popcll(tmask);
      }
    }
    if (!done && lane == 0 && last_id >= 0) { S.out_id = last_id; S.out_p = (float)((double)last_q / (double)SK); }
  }
  __syncthreads();
  if (S.out_id < 0 && tid == 0) S.flags |= SIMPLE_DIAG_ERROR;
}

// ------------------------------------------------------------------ the kernel -----------------
// One row, start to finish (all threads of the workgroup call it with the same row).
template <typename DT, bool VEC>
__device__ inline void sample_row_body(const SampleArgs& a, const int row, unsigned char* lds, Shared& S) {
  const int tid = threadIdx.x;
  const int V = a.V;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)row * (size_t)a.stride;
  const simple_row_params par = a.params[row];
  uint32_t* ck = reinterpret_cast<uint32_t*>(lds + a.L.cand);
  uint32_t* ci = ck + CAP;
  uint32_t* hist = reinterpret_cast<uint32_t*>(lds + a.L.hist);

  simple_row_diag dg;
  dg.alpha = __longlong_as_double(0x7FF8000000000000ll);
  dg.s_k = 0.0; dg.p_chosen = 0.0f; dg.n_survivors = 0; dg.flags = a.gated ? SIMPLE_DIAG_GENERAL : 0u; dg.reserved = 0u;

  // ---- row configuration (identical in every thread) ----
  const bool bad_par = !(par.temperature >= 0.0f) || !(par.rep_penalty > 0.0f);
  const bool greedy = par.temperature == 0.0f;
  const bool k_on = par.top_k >= 1 && par.top_k < V;
  const RowHist rh = row_history(a, row, par.n_prompt);  // the call's CSR arrays, or the row's slot of an incremental state
  const int nnz = rh.nnz;
  const bool too_long = nnz > a.max_nnz;
  const bool pen_on = par.rep_penalty != 1.0f || par.freq_penalty != 0.0f || par.pres_penalty != 0.0f;
  const bool lowering = par.rep_penalty >= 1.0f && par.freq_penalty >= 0.0f && par.pres_penalty >= 0.0f;
  if (tid == 0) {
    S.tau = greedy ? 1.0f : par.temperature;
    S.greedy = greedy; S.k_on = k_on; S.top_k = par.top_k;
    S.k_sel = greedy ? 1 : (k_on ? min(par.top_k, KMAX) : KMAX);
    S.top_p = par.top_p; S.min_p = par.min_p;
    S.cand_count = 0u; S.n_conv = 0u; S.g_pass = -INFINITY; S.flags = 0u; S.out_id = -1; S.out_p = 0.0f;
    const double c = 1.4426950408889634 / (double)(greedy ? 1.0f : par.temperature);
    float chi = (float)c;
    if ((double)chi > c) chi = __uint_as_float(__float_as_uint(chi) - 1u);  // round down (c > 0)
    S.c_hi = chi; S.c_lo = fmaxf((float)(c - (double)chi), 1e-30f);
  }
  __syncthreads();
  if (bad_par || too_long) {
    if (tid == 0) {
      a.out[row] = -1;
      dg.flags |= SIMPLE_DIAG_ERROR | (bad_par ? SIMPLE_DIAG_BAD_PARAM : 0u) | (too_long ? SIMPLE_DIAG_HISTORY_TOO_LONG : 0u);
      if (a.diag) a.diag[row] = dg;
      if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
      write_decision(a, row, -1, 0.0f, false);
    }
    return;
  }
  // ---- history state ----
  History H;
  H.bits = reinterpret_cast<uint32_t*>(lds + a.L.bitmap);
  H.grp = reinterpret_cast<uint32_t*>(lds + a.L.grp);
  H.cnt = reinterpret_cast<uint32_t*>(lds + a.L.counts);
  H.n_words = (V + 31) >> 5;
  H.distinct = 0;
  H.rep = par.rep_penalty; H.freq = par.freq_penalty; H.pres = par.pres_penalty;
  H.active = (nnz > 0) && pen_on;
  if (H.active) {
    if (!build_history(H, rh.ids, nnz, rh.n_prompt, V, S.scan_u32, &S.flag_ws)) dg.flags |= SIMPLE_DIAG_BAD_HISTORY_ID;
  }
  if (a.hot_bits && a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
  const uint32_t* hot_bits = greedy ? nullptr : a.hot_bits;

  Draws U;
  { double u[3]; row_uniforms(a.seed, a.row_offset + (uint64_t)row, a.step, u); U.u_draw = u[0]; U.u_acc = u[1]; U.u_tail = u[2]; }

  const bool need_sum = !greedy && !k_on && par.top_p < 1.0f && par.top_p > 0.0f;
  const bool full_mode = need_sum || (H.active && !lowering);
  const bool list_ok = greedy || (k_on && par.top_k <= KMAX) ||
                       (!k_on && (par.top_p < 1.0f || par.min_p > 0.0f || V <= KMAX));
  bool done = false;
  if (list_ok) {
    int rc = full_mode ? sampled_route<DT, VEC, true>(rowp, V, H, need_sum, S, ck, ci, hist, U, hot_bits, dg)
                       : sampled_route<DT, VEC, false>(rowp, V, H, need_sum, S, ck, ci, hist, U, hot_bits, dg);
    if (rc == ROUTE_RETRY) {
      // the threshold only rises here (strict, ids ascending), so this pass cannot fail
      constexpr int T = 64 * Elem<DT>::EPL * UNROLL;
      dg.flags |= SIMPLE_DIAG_REPLAY;
      __syncthreads();
      if (tid == 0) { S.cand_count = 0u; S.n_conv = 0u; S.g_pass = -INFINITY; }
      __syncthreads();
      ExpSum E{-3.4028234663852886e38f, 0.0, S.c_hi, S.c_lo};
      int pos = 0;
      bool careful_used = false;
      while (pos < V) {
        const unsigned count0 = S.cand_count;
        const int k_sel = S.k_sel;
        // segment length: expected appends (k_sel * len / seen) stay below half the free space
        long long len;
        if (pos == 0) len = CAP;
        else len = (long long)(CAP - (int)count0) * (long long)pos / (2ll * (long long)k_sel);
        len = max((len / T) * T, (long long)T);
        const int seg1 = (int)min((long long)V, (long long)pos + len);
        const float g = S.g_pass;
        if (full_mode) stream_range<DT, VEC, true>(rowp, pos, seg1, g, H, need_sum, E, S, ck, ci);
        else stream_range<DT, VEC, false>(rowp, pos, seg1, g, H, false, E, S, ck, ci);
        __syncthreads();
        if (S.cand_count > (unsigned)CAP) {  // overflow: replay the segment in pieces that cannot overflow
          careful_used = true;
          __syncthreads();
          if (tid == 0) S.cand_count = count0;
          __syncthreads();
          int p0 = pos;
          while (p0 < seg1) {
            const int p1 = min(seg1, p0 + (CAP - (int)S.cand_count));
            const float g2 = S.g_pass;
            if (full_mode) stream_careful<DT, true>(rowp, p0, p1, g2, H, S, ck, ci);
            else stream_careful<DT, false>(rowp, p0, p1, g2, H, S, ck, ci);
            compact(S, ck, ci, hist, H, !full_mode);
            p0 = p1;
          }
        } else {
          compact(S, ck, ci, hist, H, !full_mode);
        }
        pos = seg1;
      }
      if (careful_used) dg.flags |= SIMPLE_DIAG_CAREFUL;
      const double S_total = need_sum ? combine_exp_sums(S, E) : 0.0;
      __syncthreads();
      const bool complete = k_on || greedy || (S.cand_count == (unsigned)V);
      done = finalize_small(S, ck, ci, complete, S_total, U, hot_bits, dg);
    } else {
      done = (rc == ROUTE_DONE);
    }
    __syncthreads();
  }
  if (!done) {
    dg.flags |= SIMPLE_DIAG_WIDE;
    RowReader<DT> R{rowp, V, S.tau, greedy, &H};
    wide_route<DT, VEC>(R, S, hist, lds + a.L.cand, U, hot_bits, dg, a.diag != nullptr);
    __syncthreads();
  }
  if (tid == 0) {
    const unsigned f = S.flags;
    const bool err = (f & SIMPLE_DIAG_ERROR) != 0u;
    a.out[row] = err ? -1 : S.out_id;
    dg.flags |= f | (greedy ? SIMPLE_DIAG_GREEDY : 0u);
    dg.p_chosen = err ? 0.0f : S.out_p;
    if (a.diag) a.diag[row] = dg;
    if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
    write_decision(a, row, err ? -1 : S.out_id, dg.p_chosen, greedy);
  }
}

template <typename DT, bool VEC>
__global__ __launch_bounds__(NT, 4) void sample_rows_kernel(const SampleArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ Shared S;
  sample_row_body<DT, VEC>(a, (int)blockIdx.x, lds, S);
}

// Completes the rows the single-pass kernel queued: workgroup i takes queue entries i, i + grid, ...
// The next launch's single-pass kernel clears the count.  The queue is empty in the common case, so
// the count is looked at first.  The row body takes the arguments by reference; handing it the
// by-value parameter would make every lane of every launch copy the whole record to scratch memory
// at the kernel's entry (220 bytes a lane, 28 MB a launch), so it gets the record where the launch
// placed it, in the kernel-argument segment (the record is the kernel's only parameter).
template <typename DT, bool VEC>
__device__ __noinline__ void pending_rows_body(const SampleArgs& a, unsigned n, unsigned char* lds, Shared& S) {
  for (unsigned i = blockIdx.x; i < n; i += gridDim.x) {
    const int row = (int)a.pend[2 + i];
    if (row >= 0 && row < a.B) sample_row_body<DT, VEC>(a, row, lds, S);
    __syncthreads();
  }
}
template <typename DT, bool VEC>
__global__ __launch_bounds__(NT, 4) void pending_rows_kernel(const SampleArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ Shared S;
  const unsigned n = min(__hip_atomic_load(&a.pend[a.parity], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), (unsigned)a.B);
  if (blockIdx.x >= n) return;
  const SampleArgs* in_place = (const SampleArgs*)__builtin_amdgcn_kernarg_segment_ptr();
  pending_rows_body<DT, VEC>(*in_place, n, lds, S);
}

// Hot-set membership bitmap (section 5.3): V bits, built from the id list.
__global__ void hot_clear_kernel(uint32_t* bits, int n_words, uint32_t* flags) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) bits[i] = 0u;
  if (i == 0) *flags = 0u;
}
__global__ void hot_scatter_kernel(const int32_t* __restrict__ ids, int H, int V, uint32_t* bits, uint32_t* flags) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= H) return;
  const int id = ids[i];
  if ((unsigned)id >= (unsigned)V) { atomicOr(flags, 1u); return; }
  const uint32_t bit = 1u << (id & 31);
  if (atomicOr(&bits[id >> 5], bit) & bit) atomicOr(flags, 2u);
}

}  // namespace simple


// ------------------------------------------------------------------ launchers ------------------
namespace simple {

template <typename DT, bool VEC>
static hipError_t launch_one(const SampleArgs& a, hipStream_t st) {
  auto k = sample_rows_kernel<DT, VEC>;
  hipLaunchKernelGGL(k, dim3((unsigned)a.B), dim3(NT), a.L.total, st, a);
  return hipGetLastError();
}

template <typename DT, bool VEC>
static hipError_t launch_pending(const SampleArgs& a, hipStream_t st) {
  auto k = pending_rows_kernel<DT, VEC>;
  // One workgroup per compute unit.  Two would fit (registers, LDS) and finish a batch in which every
  // row is queued 1.4 times sooner, but the launch costs 3.5 us more on every call, and the queue
  // is empty or short in the common case; the host does not know its length.
  const unsigned resident = (unsigned)(a.n_cu > 0 ? a.n_cu : 256);
  const unsigned grid = (unsigned)a.B < resident ? (unsigned)a.B : resident;
  hipLaunchKernelGGL(k, dim3(grid), dim3(NT), a.L.total, st, a);
  return hipGetLastError();
}

hipError_t launch_pending_rows(const SampleArgs& a, int dtype, bool vec, hipStream_t st) {
  if (dtype == SIMPLE_F32) return vec ? launch_pending<float, true>(a, st) : launch_pending<float, false>(a, st);
  return vec ? launch_pending<uint16_t, true>(a, st) : launch_pending<uint16_t, false>(a, st);
}

// ev0 / ev1 (may be null): recorded right before and after the dominant kernel of the call.
hipError_t launch_sample(const SampleArgs& a, int dtype, bool vec, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (a.gated && a.order && !a.pattern_on) {  // (with no more rows than compute units every row has one to itself: nothing to balance;
                                               //  ahead of a bfloat16 call's single-pass kernel the pattern-count kernel writes the order)
    const hipError_t e = launch_order(a, st);
    if (e != hipSuccess) return e;
  }
  if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return hipErrorUnknown;
  if (a.gated) {  // single-pass kernel first; the general kernel then completes the rows it queued
    hipError_t e = a.pattern_on ? launch_pattern(a, st) : hipSuccess;
    if (e != hipSuccess) return e;
    e = launch_fast(a, dtype, st);
    if (e != hipSuccess) return e;
    if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return hipErrorUnknown;
    e = launch_wide(a, dtype, st);  // rows whose nucleus spans more of the vocabulary than the list holds
    if (e != hipSuccess) return e;
    if (dtype == SIMPLE_F32) return vec ? launch_pending<float, true>(a, st) : launch_pending<float, false>(a, st);
    return vec ? launch_pending<uint16_t, true>(a, st) : launch_pending<uint16_t, false>(a, st);
  }
  hipError_t e;
  if (dtype == SIMPLE_F32) e = vec ? launch_one<float, true>(a, st) : launch_one<float, false>(a, st);
  else e = vec ? launch_one<uint16_t, true>(a, st) : launch_one<uint16_t, false>(a, st);
  if (e == hipSuccess && ev1 && hipEventRecord(ev1, st) != hipSuccess) return hipErrorUnknown;
  return e;
}

hipError_t set_max_lds(unsigned bytes) {
  const void* fns[8] = {
    reinterpret_cast<const void*>(sample_rows_kernel<float, true>), reinterpret_cast<const void*>(sample_rows_kernel<float, false>),
    reinterpret_cast<const void*>(sample_rows_kernel<uint16_t, true>), reinterpret_cast<const void*>(sample_rows_kernel<uint16_t, false>),
    reinterpret_cast<const void*>(pending_rows_kernel<float, true>), reinterpret_cast<const void*>(pending_rows_kernel<float, false>),
    reinterpret_cast<const void*>(pending_rows_kernel<uint16_t, true>), reinterpret_cast<const void*>(pending_rows_kernel<uint16_t, false>)};
  for (int i = 0; i < 8; ++i) {
    const hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_hot_build(const int32_t* ids, int H, int V, uint32_t* bits, uint32_t* flags, hipStream_t st) {
  const int n_words = (V + 31) >> 5;
  hipLaunchKernelGGL(hot_clear_kernel, dim3((n_words + 255) / 256), dim3(256), 0, st, bits, n_words, flags);
  if (H > 0) hipLaunchKernelGGL(hot_scatter_kernel, dim3((H + 255) / 256), dim3(256), 0, st, ids, H, V, bits, flags);
  return hipGetLastError();
}

}  // namespace simple
