// Single-pass row kernel for gfx950: one workgroup per logits row, every logit read from HBM once.
//
//   history   the row's token history becomes, in LDS, a presence bit per column, a 16-bit count
//             of set bits before each mask word and 16-bit generated-token counts indexed by the
//             rank of the id among the set bits.  The V-wide histograms of section 2.2 are never
//             materialised; a column's penalty is looked up only where its bit is set, so
//             unpenalised columns are never touched (column-wise penalties, section 5.2).
//   sample    every wave's first tile (penalised) gives, by wave-ballot radix selection, a value g
//             that is expected to admit a small multiple of the requested prefix length.
//   stream    one coalesced pass of 16-byte loads per lane.  Penalised values z' are formed in
//             registers; columns with z' >= g go to an LDS candidate list; rows whose nucleus is
//             taken over the whole vocabulary also accumulate exp((z' - g) / tau) below g and a
//             histogram of that mass over bins that are linear in the tempered logit.
//   epilogue  the list certifies itself: every column whose tempered value exceeds fl(g / tau) is
//             in it, so any prefix of the total order (value descending, id ascending) that ends
//             above that value is known exactly (truncation first, section 5.2).  Top-k, top-p and
//             min-p cuts, the survivors' mass and the inverse-CDF draw (Eq. (2), step (3)) are
//             found with bucket tables of integer (fixed-point) masses, so no result depends on
//             the order in which waves appended candidates.  SHVS (section 5.3): acceptance test
//             on the hot mass, then the draw walks the hot or the tail survivors only.
//   nucleus   rows whose nucleus is wider than the list find the bin that contains the cut from
//             the mass histogram and read the row a second time: masses of the columns surely
//             inside are summed per tile, the columns of the boundary bins are resolved exactly,
//             and one tile is read a third time to locate the drawn id.
// Rows the kernel cannot certify (threshold missed, list overflow, ties wider than a bucket table,
// parameter errors, no truncation at all) are queued for the general kernel, which runs next on
// the same stream.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "simple_device.hpp"
#include "simple_kernels.hpp"

namespace simple {
namespace fast {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

constexpr int UNR = 4;      // 16-byte loads per lane and tile
constexpr int SPW = 32;     // sample entries a wave hands to the merge
constexpr int NBF = 512;    // buckets of the epilogue tables
constexpr int MEMB = 512;   // members of one bucket that can be resolved exactly
constexpr double WSCALE = 17592186044416.0;  // 2^44: fixed-point scale of probability mass

template <typename DT> struct Io;
template <> struct Io<float> {
  static constexpr int EPL = 4;
  typedef f32x4 Raw;
  __device__ static __forceinline__ Raw load(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
  __device__ static __forceinline__ void unpack(const Raw& r, float (&z)[4]) { z[0] = r.x; z[1] = r.y; z[2] = r.z; z[3] = r.w; }
  __device__ static __forceinline__ float one(const float* p) { return *p; }
};
template <> struct Io<uint16_t> {  // bfloat16 bit patterns; the upcast to float32 is exact
  static constexpr int EPL = 8;
  typedef u32x4 Raw;
  __device__ static __forceinline__ Raw load(const uint16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
  __device__ static __forceinline__ void unpack(const Raw& r, float (&z)[8]) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { z[2 * i] = __uint_as_float(w[i] << 16); z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
  }
  __device__ static __forceinline__ float one(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
};

__device__ __forceinline__ u64 composite(uint32_t key, uint32_t id) { return ((u64)key << 32) | (u64)(0xFFFFFFFFu - id); }
__device__ __forceinline__ unsigned lanes_before(u64 m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Row-wide state in static LDS.
struct FS {
  unsigned cand_count, flags, kmax, memb;
  int bk, bp, bd;
  unsigned need_k, cab_k, cab_p, n_p;
  u64 mab_k, mab_p, mab_d, cut_k, cut_p, out_w;
  int out_id;
  unsigned hist_flag;
  float wmax[16];
  unsigned wcnt[16];
  unsigned r32a[16], r32b[16];
  u64 r64a[16], r64b[16];
  double rd[16];
};

// Per-row constants, identical in every thread.
struct RowCfg {
  float tau, top_p, min_p;
  int top_k, V;
  bool greedy, k_on, p_on, p_le0, minp_on, need_sum;
  double u_draw, u_acc, u_tail;
};

// ---------------------------------------------------------------- block collectives -----------
template <int NWV>
__device__ inline void blk_reduce(FS& S, unsigned& a, unsigned& b, u64& cmax, u64& d) {
  a = wave_sum(a); b = wave_sum(b); d = wave_sum(d);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { const u64 t = __shfl_xor(cmax, o, 64); cmax = (t > cmax) ? t : cmax; }
  __syncthreads();
  if (lane_id() == 0) { const int w = wave_id(); S.r32a[w] = a; S.r32b[w] = b; S.r64a[w] = cmax; S.r64b[w] = d; }
  __syncthreads();
  unsigned ta = 0, tb = 0; u64 tc = 0, td = 0;
#pragma unroll
  for (int w = 0; w < NWV; ++w) { ta += S.r32a[w]; tb += S.r32b[w]; const u64 x = S.r64a[w]; tc = (x > tc) ? x : tc; td += S.r64b[w]; }
  a = ta; b = tb; cmax = tc; d = td;
}
template <int NWV>
__device__ inline u64 blk_sum_u64(FS& S, u64 v) {
  unsigned a = 0, b = 0; u64 c = 0;
  blk_reduce<NWV>(S, a, b, c, v);
  return v;
}
template <int NWV>
__device__ inline double blk_sum_f64(FS& S, double v) {  // fixed tree: bit-reproducible
  v = wave_sum(v);
  __syncthreads();
  if (lane_id() == 0) S.rd[wave_id()] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NWV; ++w) t += S.rd[w];
  return t;
}
// Exclusive scans of one (count, mass) pair per thread, with totals.
template <int NWV>
__device__ inline void blk_excl_scan2(FS& S, unsigned c, u64 m, unsigned& ce, u64& me, unsigned& ct, u64& mt) {
  const unsigned ci = wave_incl_scan(c);
  const u64 mi = wave_incl_scan(m);
  __syncthreads();
  if (lane_id() == 63) { S.r32a[wave_id()] = ci; S.r64a[wave_id()] = mi; }
  __syncthreads();
  unsigned cb = 0, ctt = 0; u64 mb = 0, mtt = 0;
#pragma unroll
  for (int w = 0; w < NWV; ++w) {
    const unsigned x = S.r32a[w]; const u64 y = S.r64a[w];
    if (w < wave_id()) { cb += x; mb += y; }
    ctt += x; mtt += y;
  }
  ce = cb + ci - c; me = mb + mi - m; ct = ctt; mt = mtt;
}

// q-th largest of the 64 x N keys held by a wave (N per lane): bitwise radix descent with wave
// ballots; no LDS, no barrier.  need >= 1; if the wave holds fewer keys the result is 0.
template <int N>
__device__ __forceinline__ uint32_t wave_select_key(const uint32_t (&k)[N], unsigned need) {
  uint32_t prefix = 0u;
#pragma unroll 1
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t want = (prefix >> bit) | 1u;
    unsigned c = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) c += (unsigned)__popcll(__ballot((k[j] >> bit) == want));
    if (c >= need) prefix |= (1u << bit); else need -= c;
  }
  return prefix;
}

// Fixed-point weight exp(y - y_max) * 2^44 of an orderable key (section 2.1 Eq. (2), stable softmax).
__device__ __forceinline__ u64 wfix(uint32_t key, double y_max) {
  return (u64)__double2ull_rn(exp((double)keyf(key) - y_max) * WSCALE);
}

// ---------------------------------------------------------------- history ---------------------
struct Hist {
  const uint32_t* bm;
  const uint16_t* dir;
  const uint16_t* cnt;
  float rep, freq, pres;
  double inv_rep;
  bool active;
  // Z' of a column that is in the history (section 2.2): repetition (sign-aware), then frequency,
  // then presence on generated tokens; one float32 rounding per operation.  z / rep is formed as
  // fl32(double(z) * fl64(1 / rep)), which equals the IEEE float32 quotient: the product is within
  // 2^-52 of the exact quotient, and the quotient of two 24-bit significands is never that close
  // to a float32 rounding boundary.
  __device__ __forceinline__ float apply(float z, uint32_t c) const {
    z = (z > 0.0f) ? (float)((double)z * inv_rep) : z * rep;
    if (c > 0u) { const float t = freq * (float)c; z = z - t; z = z - pres; }
    return z;
  }
};

// Builds bitmap, rank directory and counts of one row.  Out-of-range ids are ignored and flagged.
template <int NTHR>
__device__ inline void build_history(FS& S, uint32_t* bm, uint16_t* dir, uint32_t* cnt32, const int32_t* __restrict__ hist,
                                     int nnz, int n_prompt, int V) {
  constexpr int NWV = NTHR / 64;
  const int tid = threadIdx.x;
  const int n_words = (V + 31) >> 5;
  for (int i = tid; i < n_words; i += NTHR) bm[i] = 0u;
  for (int i = tid; i < (nnz + 1) / 2; i += NTHR) cnt32[i] = 0u;
  __syncthreads();
  bool bad = false;
  for (int i = tid; i < nnz; i += NTHR) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) atomicOr(&bm[id >> 5], 1u << (id & 31)); else bad = true;
  }
  if (bad) atomicOr(&S.flags, SIMPLE_DIAG_BAD_HISTORY_ID);
  __syncthreads();
  // directory: exclusive scan of the words' popcounts, NTHR * 8 words per round
  unsigned carry = 0;
  for (int w0 = 0; w0 < n_words; w0 += NTHR * 8) {
    const int wb = w0 + tid * 8;
    unsigned pc[8], tot = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) { pc[j] = (wb + j < n_words) ? (unsigned)__popc(bm[wb + j]) : 0u; tot += pc[j]; }
    unsigned ce, ct; u64 me, mt;
    blk_excl_scan2<NWV>(S, tot, 0ull, ce, me, ct, mt);
    unsigned run = carry + ce;
#pragma unroll
    for (int j = 0; j < 8; ++j) { if (wb + j < n_words) dir[wb + j] = (uint16_t)run; run += pc[j]; }
    carry += ct;
  }
  __syncthreads();
  n_prompt = min(max(n_prompt, 0), nnz);
  for (int i = n_prompt + tid; i < nnz; i += NTHR) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) {
      const uint32_t word = bm[id >> 5];
      const unsigned r = (unsigned)dir[id >> 5] + (unsigned)__popc(word & ((1u << (id & 31)) - 1u));
      atomicAdd(&cnt32[r >> 1], 1u << ((r & 1u) * 16u));
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------- stream ----------------------
struct StreamCtx {
  float g, c_hi, c_lo;
  bool need_sum;
  u64* hist;  // NBW bins of (count << 46 | mass * 2^28)
};
constexpr int NBW = 2048;
constexpr float BINS_PER_LOG2 = 64.0f;

// Unpacks one tile and applies the penalties to the columns whose history bit is set.
template <typename DT>
__device__ __forceinline__ void prep_tile(const typename Io<DT>::Raw (&A)[UNR], int tb, const Hist& H,
                                          float (&z)[UNR][Io<DT>::EPL]) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr unsigned EMASK = (1u << EPL) - 1u;
  const int lane = lane_id();
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
    Io<DT>::unpack(A[u], z[u]);
    if (H.active) {
      const int idx0 = tb + u * 64 * EPL + lane * EPL;
      const uint32_t word = H.bm[idx0 >> 5];
      const unsigned sh = (unsigned)idx0 & 31u;
      const uint32_t nib = (word >> sh) & EMASK;
      if (nib) {
        const unsigned base = (unsigned)H.dir[idx0 >> 5] + (unsigned)__popc(word & ((1u << sh) - 1u));
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          if (nib & (1u << e)) {
            const unsigned r = base + (unsigned)__popc(nib & ((1u << e) - 1u));
            z[u][e] = H.apply(z[u][e], (uint32_t)H.cnt[r]);
          }
        }
      }
    }
  }
}

__device__ __forceinline__ void append_lanes(FS& S, uint32_t* cz, uint32_t* ci, u64 m, float z, int idx) {
  const int lane = lane_id();
  unsigned base = 0;
  if (lane == 0) base = atomicAdd(&S.cand_count, (unsigned)__popcll(m));
  base = __shfl(base, 0, 64);
  if ((m >> lane) & 1ull) {
    const unsigned slot = base + lanes_before(m);
    if (slot < (unsigned)CAPF) { cz[slot] = __float_as_uint(z); ci[slot] = (uint32_t)idx; }
  }
}

// Mass of one column below g, relative to g: exp2((z - g) * log2(e) / tau), and its histogram bin.
__device__ __forceinline__ float below_term(float z, const StreamCtx& C, bool do_hist) {
  const float d = z - C.g;
  const float t = fmaf(d, C.c_hi, d * C.c_lo);
  const float w = (z < C.g) ? __builtin_amdgcn_exp2f(t) : 0.0f;
  if (do_hist && z < C.g) {
    const int b = min((int)(-t * BINS_PER_LOG2), NBW - 1);
    atomicAdd(&C.hist[b], (1ull << 46) | (u64)(w * 268435456.0f + 0.5f));
  }
  return w;
}

// Candidate test and mass accumulation of one prepared tile.
template <typename DT>
__device__ __forceinline__ void consume_tile(const float (&z)[UNR][Io<DT>::EPL], int tb, const StreamCtx& C, double& acc,
                                             FS& S, uint32_t* cz, uint32_t* ci) {
  constexpr int EPL = Io<DT>::EPL;
  const int lane = lane_id();
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
    if (C.need_sum) {
      float ps = 0.0f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) ps += below_term(z[u][e], C, C.hist != nullptr);
      acc += (double)ps;
    }
    bool any = false;
#pragma unroll
    for (int e = 0; e < EPL; ++e) any = any || !(z[u][e] < C.g);
    if (__ballot(any)) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const u64 m = __ballot(!(z[u][e] < C.g));
        if (m) append_lanes(S, cz, ci, m, z[u][e], tb + u * 64 * EPL + lane * EPL + e);
      }
    }
  }
}

// ---------------------------------------------------------------- epilogue on the list --------
enum { FIN_DONE = 0, FIN_PENDING = 1, FIN_WIDE = 2 };

// Exact selection, softmax and draw on the candidate list (see the file comment).  On FIN_DONE the
// result is in S.out_id / S.out_w (or the error flag is set); FIN_WIDE: the nucleus reaches below
// the list; FIN_PENDING: the list cannot certify the row.
template <int NTHR>
__device__ __noinline__ int finalize_list(FS& S, const RowCfg& R, uint32_t* cz, uint32_t* ci, unsigned char* scratch,
                                          float g, double S_below, const uint32_t* __restrict__ hot_bits,
                                          simple_row_diag& dg) {
  constexpr int NWV = NTHR / 64;
  constexpr int PER = CAPF / NTHR;
  const int tid = threadIdx.x;
  uint32_t* fcnt = reinterpret_cast<uint32_t*>(scratch);
  u64* fmass = reinterpret_cast<u64*>(scratch + 2048);
  u64* mc = reinterpret_cast<u64*>(scratch + 6144);
  u64* mw = reinterpret_cast<u64*>(scratch + 10240);
  const unsigned n = S.cand_count;
  uint32_t key[PER], id[PER];
  bool err = false;
  uint32_t kloc = 0u;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const unsigned i = (unsigned)tid + (unsigned)j * NTHR;
    key[j] = 0u; id[j] = 0u;
    if (i < n) {
      const float z = __uint_as_float(cz[i]);
      id[j] = ci[i];
      if (z != z || z == INFINITY) err = true;
      else {
        const float y = R.greedy ? z : z / R.tau;
        if (y == INFINITY) err = true; else key[j] = fkey(y);
      }
    }
    kloc = max(kloc, key[j]);
  }
  if (kloc) atomicMax(&S.kmax, kloc);
  if (err) atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
  __syncthreads();
  if (S.flags & SIMPLE_DIAG_ERROR) return FIN_DONE;
  const uint32_t kmax = S.kmax;
  const uint32_t key_g = fkey(R.greedy ? g : g / R.tau);
  if (kmax <= key_g || kmax <= KEY_NEG_INF) return FIN_PENDING;
  // certified entries: tempered value strictly above fl(g / tau)
  unsigned ncl = 0, nul = 0;
  u64 cl = 0ull, dummy = 0ull;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (!key[j]) continue;
    if (key[j] > key_g) { ++ncl; const u64 c = composite(key[j], id[j]); cl = (c > cl) ? c : cl; }
    else { ++nul; key[j] = 0u; }
  }
  unsigned n_cert = ncl, n_unc = nul;
  u64 cmax = cl;
  blk_reduce<NWV>(S, n_cert, n_unc, cmax, dummy);
  if (R.greedy) {
    if (tid == 0) { S.out_id = (int)(0xFFFFFFFFu - (uint32_t)cmax); S.out_w = 0ull; }
    dg.n_survivors = 1;
    dg.p_chosen = 1.0f;
    __syncthreads();
    return FIN_DONE;
  }
  const unsigned n_k = R.k_on ? (unsigned)R.top_k : (unsigned)R.V;
  if (R.k_on && n_cert < n_k) return FIN_PENDING;  // the sampled threshold admitted too few
  const double y_max = (double)keyf(kmax);
  u64 wf[PER];
  unsigned bkt[PER];
  const unsigned span = kmax - key_g;
  const int bshift = max(0, 32 - (int)__clz(span) - 9);
  for (int i = tid; i < NBF; i += NTHR) { fcnt[i] = 0u; fmass[i] = 0ull; }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    wf[j] = 0ull; bkt[j] = 0u;
    if (key[j]) {
      wf[j] = wfix(key[j], y_max);
      bkt[j] = (kmax - key[j]) >> bshift;
      atomicAdd(&fcnt[bkt[j]], 1u);
      atomicAdd(&fmass[bkt[j]], wf[j]);
    }
  }
  __syncthreads();
  const unsigned c = (tid < NBF) ? fcnt[tid] : 0u;
  const u64 m = (tid < NBF) ? fmass[tid] : 0ull;
  unsigned ce, total_c; u64 me, total_m;
  blk_excl_scan2<NWV>(S, c, m, ce, me, total_c, total_m);
  // ---- top-k cut: the bucket that holds the n_k-th entry, then its members exactly ----
  const bool kcut = R.k_on && n_cert > n_k;
  if (kcut && tid < NBF && c > 0u && ce < n_k && n_k <= ce + c) { S.bk = tid; S.need_k = n_k - ce; S.cab_k = ce; S.mab_k = me; }
  __syncthreads();
  u64 cut_k = 0ull, S_klist = total_m;
  int bk = -1;
  if (kcut) {
    bk = S.bk;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (key[j] && (int)bkt[j] == bk) {
        const unsigned slot = atomicAdd(&S.memb, 1u);
        if (slot < (unsigned)MEMB) { mc[slot] = composite(key[j], id[j]); mw[slot] = wf[j]; }
      }
    }
    __syncthreads();
    const unsigned nm = S.memb;
    if (nm > (unsigned)MEMB) return FIN_PENDING;  // ties wider than the member table
    const unsigned need = S.need_k;
    for (unsigned mi = tid; mi < nm; mi += NTHR) {
      const u64 cm = mc[mi];
      unsigned r = 0;
      for (unsigned q = 0; q < nm; ++q) r += (mc[q] > cm) ? 1u : 0u;
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
  u64 S_k_fix = S_klist;
  if (!R.k_on) {
    const double f0 = exp((double)g / (double)R.tau - y_max);
    S_k_fix = total_m + (u64)n_unc * wfix(key_g, y_max) + (u64)__double2ull_rn(S_below * f0 * WSCALE);
  }
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
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        if (key[j] && (int)bkt[j] == bp && composite(key[j], id[j]) >= cut_k) {
          const unsigned slot = atomicAdd(&S.memb, 1u);
          if (slot < (unsigned)MEMB) { mc[slot] = composite(key[j], id[j]); mw[slot] = wf[j]; }
        }
      }
      __syncthreads();
      const unsigned nm = S.memb;
      if (nm > (unsigned)MEMB) return FIN_PENDING;
      const u64 mab = S.mab_p;
      for (unsigned mi = tid; mi < nm; mi += NTHR) {
        const u64 cm = mc[mi], wm = mw[mi];
        u64 G = mab; unsigned r = 0;
        for (unsigned q = 0; q < nm; ++q) { const u64 cq = mc[q]; if (cq >= cm) G += mw[q]; if (cq > cm) ++r; }
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
    const float thr = keyf(kmax) + (float)log((double)R.min_p);
    const uint32_t key_thr = fkey(thr);
    if (key_thr > key_g) { cut_m = (u64)key_thr << 32; m_cert = true; }
  }
  const bool known = R.k_on || p_found || m_cert;
  if (!known) return (R.need_sum && !R.minp_on) ? FIN_WIDE : FIN_PENDING;
  if (R.k_on && R.p_on && !p_found) return FIN_PENDING;  // cannot happen: the top-k prefix holds its own mass
  u64 cut = cut_k;
  if (p_found && cut_p > cut) cut = cut_p;
  if (m_cert && cut_m > cut) cut = cut_m;
  if (cut > cmax) cut = cmax;  // never empty
  // ---- survivors K_b, their mass, the hot split (Eq. (7)) ----
  const bool use_hot = hot_bits != nullptr;
  bool surv[PER], hot[PER];
  unsigned ns = 0, nh = 0; u64 sk = 0ull, sh = 0ull, cdum = 0ull;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    surv[j] = key[j] && composite(key[j], id[j]) >= cut;
    hot[j] = false;
    if (surv[j]) {
      ++ns; sk += wf[j];
      if (use_hot) { hot[j] = (hot_bits[id[j] >> 5] >> (id[j] & 31)) & 1u; if (hot[j]) { ++nh; sh += wf[j]; } }
    }
  }
  // two reductions share the barriers: (ns, nh, -, sk) then sh
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
  if (S_cls == 0ull) return FIN_PENDING;  // the chosen class holds no mass here: general kernel
  // ---- inverse CDF in ascending token id: first id whose running mass exceeds u * S ----
  u64 tfix = (u64)__double2ull_rd(u * (double)S_cls);
  if (tfix >= S_cls) tfix = S_cls - 1ull;
  const int ishift = max(0, 32 - (int)__clz((unsigned)(R.V - 1) | 1u) - 9);
  for (int i = tid; i < NBF; i += NTHR) fmass[i] = 0ull;
  __syncthreads();
  bool incls[PER];
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    incls[j] = surv[j] && (!use_hot || hot[j] == pick_hot);
    if (incls[j]) atomicAdd(&fmass[id[j] >> ishift], wf[j]);
  }
  __syncthreads();
  {
    const u64 m2 = (tid < NBF) ? fmass[tid] : 0ull;
    unsigned ce2, ct2; u64 me2, mt2;
    blk_excl_scan2<NWV>(S, 0u, m2, ce2, me2, ct2, mt2);
    if (tid < NBF && m2 > 0ull && me2 <= tfix && me2 + m2 > tfix) { S.bd = tid; S.mab_d = me2; }
  }
  __syncthreads();
  const int bd = S.bd;
  if (bd < 0) return FIN_PENDING;  // cannot happen: tfix < S_cls
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (incls[j] && (int)(id[j] >> ishift) == bd) {
      const unsigned slot = atomicAdd(&S.memb, 1u);
      if (slot < (unsigned)MEMB) { mc[slot] = (u64)id[j]; mw[slot] = wf[j]; }
    }
  }
  __syncthreads();
  {
    const unsigned nm = S.memb;  // a bucket spans at most 512 ids
    const u64 mab = S.mab_d;
    for (unsigned mi = tid; mi < nm; mi += NTHR) {
      const u64 im = mc[mi], wm = mw[mi];
      u64 C = mab;
      for (unsigned q = 0; q < nm; ++q) if (mc[q] <= im) C += mw[q];
      if (C > tfix && C - wm <= tfix) { S.out_id = (int)im; S.out_w = wm; }
    }
  }
  __syncthreads();
  dg.p_chosen = (float)((double)S.out_w / (double)S_K);
  return (S.out_id >= 0) ? FIN_DONE : FIN_PENDING;
}

__device__ inline void queue_pending(const SampleArgs& a, int row) {
  const unsigned slot = atomicAdd(&a.pend[0], 1u);
  a.pend[2 + slot] = (uint32_t)row;
  a.out[row] = PENDING;
}

// ---------------------------------------------------------------- the kernel ------------------
template <typename DT, int NTHR>
__global__ __launch_bounds__(NTHR, 4) void fast_rows_kernel(const SampleArgs a) {
  constexpr int NWV = NTHR / 64;
  constexpr int EPL = Io<DT>::EPL;
  constexpr int T = 64 * EPL * UNR;
  typedef typename Io<DT>::Raw Raw;
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int V = a.V;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)row * (size_t)a.stride;
  const simple_row_params par = a.params[row];
  uint32_t* bm = reinterpret_cast<uint32_t*>(lds + a.F.bitmap);
  uint16_t* dir = reinterpret_cast<uint16_t*>(lds + a.F.dir);
  uint32_t* cnt32 = reinterpret_cast<uint32_t*>(lds + a.F.cnt);
  uint32_t* cz = reinterpret_cast<uint32_t*>(lds + a.F.cand);
  uint32_t* ci = cz + CAPF;
  unsigned char* scratch = lds + a.F.scratch;
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
  long long h0 = 0; int nnz = 0;
  if (a.hist_ptr) { h0 = a.hist_ptr[row]; const long long h1 = a.hist_ptr[row + 1]; nnz = (int)min(max(h1 - h0, 0ll), (long long)a.max_nnz + 1); }
  const bool too_long = nnz > a.max_nnz;
  const bool pen_on = par.rep_penalty != 1.0f || par.freq_penalty != 0.0f || par.pres_penalty != 0.0f;
  const bool no_trunc = !R.greedy && !R.k_on && !R.p_on && !R.minp_on;
  const bool eligible = !bad_par && !too_long && !no_trunc && (R.greedy || !R.k_on || par.top_k <= KMAXF);
  if (!eligible) {  // the general kernel takes the row (it also reports parameter errors)
    if (tid == 0) queue_pending(a, row);
    return;
  }
  const int k_sel = R.greedy ? 1 : (R.k_on ? par.top_k : (R.p_le0 ? 1 : KMAXF));
  {
    double u[3];
    row_uniforms(a.seed, a.row_offset + (uint64_t)row, a.step, u);
    R.u_draw = u[0]; R.u_acc = u[1]; R.u_tail = u[2];
  }
  if (tid == 0) {
    S.cand_count = 0u; S.flags = 0u; S.kmax = 0u; S.memb = 0u; S.bk = -1; S.bp = -1; S.bd = -1;
    S.need_k = 0u; S.cut_k = 0ull; S.cut_p = 0ull; S.n_p = 0u; S.out_id = -1; S.out_w = 0ull;
  }
  // ---- this wave's tiles; the first one is its sample ----
  const int nfull = V / T;  // the host guarantees nfull >= 2 * NWV
  const int t0 = (int)(((long long)wave * nfull) / NWV), t1 = (int)(((long long)(wave + 1) * nfull) / NWV);
  Raw A[UNR], Bf[UNR];
#pragma unroll
  for (int u = 0; u < UNR; ++u) A[u] = Io<DT>::load(rowp + (size_t)t0 * T + u * 64 * EPL + lane * EPL);
#pragma unroll
  for (int u = 0; u < UNR; ++u) Bf[u] = Io<DT>::load(rowp + (size_t)(t0 + 1) * T + u * 64 * EPL + lane * EPL);
  __syncthreads();

  // ---- history state ----
  Hist H;
  H.bm = bm; H.dir = dir; H.cnt = reinterpret_cast<const uint16_t*>(cnt32);
  H.rep = par.rep_penalty; H.freq = par.freq_penalty; H.pres = par.pres_penalty;
  H.inv_rep = 1.0 / (double)par.rep_penalty;
  H.active = (nnz > 0) && pen_on;
  if (H.active) build_history<NTHR>(S, bm, dir, cnt32, a.hist_ids + h0, nnz, par.n_prompt, V);
  const uint32_t* hot_bits = R.greedy ? nullptr : a.hot_bits;

  // ---- threshold from the sample: two largest penalised values per lane, wave select, merge ----
  float z[UNR][EPL];
  prep_tile<DT>(A, t0 * T, H, z);
  float a1 = -INFINITY, a2 = -INFINITY;
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float v = z[u][e];
      if (v > a1) { a2 = a1; a1 = v; } else if (v > a2) a2 = v;
    }
  }
  // rank in the sample whose value leaves, with high probability, >= k_sel columns above it in the row
  const float m_exp = (float)k_sel * (float)(NWV * T) / (float)V;
  const unsigned r_samp = (unsigned)ceilf(1.3f * m_exp + 3.0f * sqrtf(m_exp) + 3.0f);
  {
    const float r_w = (float)r_samp / (float)NWV;
    const unsigned q = min((unsigned)SPW, (unsigned)ceilf(r_w + 3.0f * sqrtf(r_w) + 2.0f));
    const uint32_t k2[2] = {fkey(a1), fkey(a2)};
    const uint32_t Kw = wave_select_key<2>(k2, q);
    if (lane < SPW) samp[wave * SPW + lane] = 0u;
    const u64 m1 = __ballot(k2[0] >= Kw);
    const unsigned p1 = lanes_before(m1);
    if (((m1 >> lane) & 1ull) && p1 < (unsigned)SPW) samp[wave * SPW + p1] = k2[0];
    const unsigned n1 = min((unsigned)__popcll(m1), (unsigned)SPW);
    const u64 m2 = __ballot(k2[1] >= Kw);
    const unsigned p2 = n1 + lanes_before(m2);
    if (((m2 >> lane) & 1ull) && p2 < (unsigned)SPW) samp[wave * SPW + p2] = k2[1];
    const unsigned n2 = min(n1 + (unsigned)__popcll(m2), (unsigned)SPW);
    const float wp = wave_max(a1);
    if (lane == 0) { S.wmax[wave] = wp; S.wcnt[wave] = n2; }
  }
  __syncthreads();
  StreamCtx C;
  {
    constexpr int NS = (NWV * SPW) / 64;
    uint32_t k4[NS];
    unsigned total = 0;
    float Mp = S.wmax[0];
#pragma unroll
    for (int w = 0; w < NWV; ++w) { total += S.wcnt[w]; Mp = fmaxf(Mp, S.wmax[w]); }
#pragma unroll
    for (int j = 0; j < NS; ++j) k4[j] = samp[j * 64 + lane];
    const uint32_t Kg = wave_select_key<NS>(k4, max(1u, min(r_samp, total)));
    float g = keyf(Kg);
    if (!R.greedy && !R.k_on && R.minp_on) {
      // min-p survivors lie within ln(min_p) of the row maximum, which is at least the sample's
      const float thr_lb = Mp / R.tau + (float)log((double)R.min_p);
      float gm = thr_lb * R.tau;
      gm = gm - fabsf(gm) * 1e-6f - 1e-30f;
      g = fmaxf(g, gm);
    }
    const double cd = 1.4426950408889634 / (double)R.tau;
    float c_hi = (float)cd;
    if ((double)c_hi > cd) c_hi = __uint_as_float(__float_as_uint(c_hi) - 1u);  // round down (cd > 0)
    C.g = g; C.c_hi = c_hi; C.c_lo = (float)(cd - (double)c_hi);
    C.need_sum = R.need_sum;
    C.hist = nullptr;
  }

  // ---- the stream ----
  double acc = 0.0;
  consume_tile<DT>(z, t0 * T, C, acc, S, cz, ci);
  for (int cur = t0 + 1; cur < t1; ++cur) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) A[u] = Bf[u];
    if (cur + 1 < t1) {
#pragma unroll
      for (int u = 0; u < UNR; ++u) Bf[u] = Io<DT>::load(rowp + (size_t)(cur + 1) * T + u * 64 * EPL + lane * EPL);
    }
    prep_tile<DT>(A, cur * T, H, z);
    consume_tile<DT>(z, cur * T, C, acc, S, cz, ci);
  }
  // ragged tail, element by element
  for (int idx = nfull * T + tid; idx < V; idx += NTHR) {
    float zz = Io<DT>::one(rowp + idx);
    if (H.active) {
      const uint32_t word = bm[idx >> 5];
      if ((word >> (idx & 31)) & 1u) {
        const unsigned r = (unsigned)dir[idx >> 5] + (unsigned)__popc(word & ((1u << (idx & 31)) - 1u));
        zz = H.apply(zz, (uint32_t)H.cnt[r]);
      }
    }
    if (C.need_sum) acc += (double)below_term(zz, C, false);
    if (!(zz < C.g)) {
      const unsigned slot = atomicAdd(&S.cand_count, 1u);
      if (slot < (unsigned)CAPF) { cz[slot] = __float_as_uint(zz); ci[slot] = (uint32_t)idx; }
    }
  }
  __syncthreads();

  // ---- epilogue ----
  simple_row_diag dg;
  dg.alpha = __longlong_as_double(0x7FF8000000000000ll);
  dg.s_k = 0.0; dg.p_chosen = 0.0f; dg.n_survivors = 0; dg.flags = 0u; dg.reserved = 0u;
  if (a.hot_bits && a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
  int rc = FIN_PENDING;
  if (S.cand_count <= (unsigned)CAPF) {
    const double S_below = R.need_sum ? blk_sum_f64<NWV>(S, acc) : 0.0;
    rc = finalize_list<NTHR>(S, R, cz, ci, scratch, C.g, S_below, hot_bits, dg);
  }
  if (rc == FIN_WIDE) rc = FIN_PENDING;
  if (tid == 0) {
    if (rc != FIN_DONE) {
      queue_pending(a, row);
    } else {
      const unsigned f = S.flags;
      const bool err = (f & SIMPLE_DIAG_ERROR) != 0u;
      a.out[row] = err ? -1 : S.out_id;
      if (a.diag) {
        dg.flags |= f | (R.greedy ? SIMPLE_DIAG_GREEDY : 0u);
        if (err) dg.p_chosen = 0.0f;
        a.diag[row] = dg;
      }
    }
  }
}

}  // namespace fast

hipError_t launch_fast(const SampleArgs& a, int dtype, hipStream_t st) {
  const dim3 grid((unsigned)a.B);
  if (a.F.threads == 512) {
    if (dtype == SIMPLE_F32) hipLaunchKernelGGL((fast::fast_rows_kernel<float, 512>), grid, dim3(512), a.F.total, st, a);
    else hipLaunchKernelGGL((fast::fast_rows_kernel<uint16_t, 512>), grid, dim3(512), a.F.total, st, a);
  } else {
    if (dtype == SIMPLE_F32) hipLaunchKernelGGL((fast::fast_rows_kernel<float, 1024>), grid, dim3(1024), a.F.total, st, a);
    else hipLaunchKernelGGL((fast::fast_rows_kernel<uint16_t, 1024>), grid, dim3(1024), a.F.total, st, a);
  }
  return hipGetLastError();
}

hipError_t set_max_lds_fast(unsigned bytes) {
  hipError_t e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 512>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes); if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 512>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes); if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fast::fast_rows_kernel<float, 1024>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes); if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fast::fast_rows_kernel<uint16_t, 1024>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  return e;
}

}  // namespace simple
