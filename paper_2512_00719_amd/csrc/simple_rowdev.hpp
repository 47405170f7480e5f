// Device-side pieces shared by the single-pass row kernel and the kernels of the whole-vocabulary
// nucleus: 16-byte row loads, row-wide LDS state, block collectives and the fixed-point mass of a
// column relative to the candidate threshold.  gfx950 only (wave64).
#pragma once

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

constexpr int UNR = 4;       // 16-byte loads per lane and tile
constexpr int SPW = SAMPLE_PER_WAVE;  // sample entries a wave hands to the merge
constexpr int NBF = 256;     // buckets of the long-list tables
constexpr int MEMB = 512;    // entries the sorted epilogue handles
constexpr int MEMB2 = 256;   // members of one bucket the long-list path resolves exactly
constexpr int IDR = 16;      // history ids a thread keeps in registers
constexpr double WSCALE = 17592186044416.0;  // 2^44: fixed-point scale of probability mass
constexpr int NBW = 2048;               // bins of the mass histogram (whole-vocabulary nucleus)
constexpr float BINS_PER_LOG2 = 64.0f;  // bin width: 1/64 of a factor two in probability
constexpr float MSCALE = 268435456.0f;  // 2^28: fixed-point scale of masses relative to the one at g
constexpr int RCAP = 4096;              // columns of the boundary bin that can be resolved exactly
constexpr float L2E_HI = 1.44269502162933349609375f, L2E_LO = 1.925963033500011e-8f;  // log2(e), split

// Global-memory view of a pointer.  Inside out-of-line device functions the compiler cannot tell that
// a pointer parameter is global; generic (flat) loads would also count against the LDS wait counter and
// so serialise the tile prefetch behind every LDS access.
template <typename T>
__device__ __forceinline__ const __attribute__((address_space(1))) T* as_global(const T* p) {
  return (const __attribute__((address_space(1))) T*)p;
}
__device__ __forceinline__ unsigned hot_bit(const uint32_t* __restrict__ hot_bits, uint32_t id) {
  return (as_global(hot_bits)[id >> 5] >> (id & 31u)) & 1u;
}

template <typename DT> struct Io;
template <> struct Io<float> {
  static constexpr int EPL = 4;
  typedef f32x4 Raw;
  __device__ static __forceinline__ Raw load(const float* p) { return __builtin_nontemporal_load(as_global(reinterpret_cast<const f32x4*>(p))); }
  __device__ static __forceinline__ void unpack(const Raw& r, float (&z)[4]) { z[0] = r.x; z[1] = r.y; z[2] = r.z; z[3] = r.w; }
  __device__ static __forceinline__ float one(const float* p) { return *as_global(p); }
  typedef float Elem;  // one element as loaded, converted where it is used (the load stays in flight until then)
  __device__ static __forceinline__ Elem raw(const float* p) { return *as_global(p); }
  __device__ static __forceinline__ float cvt(Elem v) { return v; }
};
template <> struct Io<uint16_t> {  // bfloat16 bit patterns; the upcast to float32 is exact
  static constexpr int EPL = 8;
  typedef u32x4 Raw;
  __device__ static __forceinline__ Raw load(const uint16_t* p) { return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4*>(p))); }
  __device__ static __forceinline__ void unpack(const Raw& r, float (&z)[8]) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { z[2 * i] = __uint_as_float(w[i] << 16); z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
  }
  __device__ static __forceinline__ float one(const uint16_t* p) { return __uint_as_float((uint32_t)(*as_global(p)) << 16); }
  typedef uint32_t Elem;
  __device__ static __forceinline__ Elem raw(const uint16_t* p) { return (uint32_t)(*as_global(p)); }
  __device__ static __forceinline__ float cvt(Elem v) { return __uint_as_float(v << 16); }
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
  unsigned n2, nunc;           // certified / uncertified entries of the list
  unsigned e_n; int e_rc, e_acc;
  unsigned distinct;           // distinct history columns of the row
  unsigned tile_ctr;           // next tile of the stream that no wave has taken yet
  u64 e_SK, e_SH, e_tfix, e_skfix;
  float wmax[16];
  unsigned wcnt[16];
  unsigned r32a[16], r32b[16];
  u64 r64a[16], r64b[16];
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
  cmax = wave_all(cmax, [](u64 x, u64 y) { return x > y ? x : y; });
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

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) { return wave_all(v, [](uint32_t x, uint32_t y) { return max(x, y); }); }
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return wave_all(v, [](uint32_t x, uint32_t y) { return min(x, y); }); }

// All-pairs helpers over small LDS tables: eight entries are loaded before they are used, so the
// reads overlap instead of each waiting out the LDS latency.
// #{q < n : a[q] > c}
__device__ __forceinline__ unsigned count_greater(const u64* a, unsigned n, u64 c) {
  unsigned r = 0, q = 0;
  for (; q + 8 <= n; q += 8) {
    u64 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = a[q + j];
#pragma unroll
    for (int j = 0; j < 8; ++j) r += (v[j] > c) ? 1u : 0u;
  }
  for (; q < n; ++q) r += (a[q] > c) ? 1u : 0u;
  return r;
}
// sum of w[q] over q < n with a[q] >= c (ge) or a[q] <= c (!ge); cnt_gt gets #{a[q] > c}
template <bool GE, typename K>
__device__ __forceinline__ u64 sum_where(const K* a, const u64* w, unsigned n, K c, unsigned& cnt_gt) {
  u64 s = 0ull; unsigned r = 0, q = 0;
  for (; q + 8 <= n; q += 8) {
    K v[8]; u64 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { v[j] = a[q + j]; x[j] = w[q + j]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) { s += (GE ? v[j] >= c : v[j] <= c) ? x[j] : 0ull; r += (v[j] > c) ? 1u : 0u; }
  }
  for (; q < n; ++q) { const K v = a[q]; s += (GE ? v >= c : v <= c) ? w[q] : 0ull; r += (v > c) ? 1u : 0u; }
  cnt_gt = r;
  return s;
}

// Z' of a column that is in the history (section 2.2): repetition (sign-aware), then frequency,
// then presence on generated tokens (count > 0); one float32 rounding per operation.  z / rep is
// formed as fl32(double(z) * fl64(1 / rep)), which equals the IEEE float32 quotient: the product is
// within 2^-52 of the exact quotient, and the quotient of two 24-bit significands is never that
// close to a float32 rounding boundary.
__device__ __forceinline__ float apply_penalties(float z, uint32_t count, float rep, double inv_rep, float freq, float pres) {
  z = (z > 0.0f) ? (float)((double)z * inv_rep) : z * rep;
  if (count > 0u) { const float t = freq * (float)count; z = z - t; z = z - pres; }
  return z;
}

// ---------------------------------------------------------------- history ---------------------
struct Hist {
  uint32_t* bm;     // V bits
  uint16_t* dir;    // set bits before each pair of mask words
  uint32_t* cnt32;  // 16-bit counts by rank, two per word
  int n_words;
  float rep, freq, pres;
  double inv_rep;
  bool active;
  __device__ __forceinline__ const uint16_t* cnt() const { return reinterpret_cast<const uint16_t*>(cnt32); }
  // Rank of column idx among the set bits (`word` is its mask word).
  __device__ __forceinline__ unsigned rank(int idx, uint32_t word) const {
    const int w = idx >> 5;
    unsigned r = (unsigned)dir[w >> 1];
    if (w & 1) r += (unsigned)__popc(bm[w - 1]);
    return r + (unsigned)__popc(word & ((1u << (idx & 31)) - 1u));
  }
  __device__ __forceinline__ float apply(float z, uint32_t c) const { return apply_penalties(z, c, rep, inv_rep, freq, pres); }
  __device__ __forceinline__ float penalised_at(float z, int idx) const {
    const uint32_t word = bm[idx >> 5];
    if ((word >> (idx & 31)) & 1u) z = apply(z, (uint32_t)cnt()[rank(idx, word)]);
    return z;
  }
};

// Clears `bytes` (rounded up to 16; the regions are 16-byte aligned and padded) with 16-byte stores.
__device__ __forceinline__ void zero16(void* p, int bytes, int tid, int nthr) {
  u32x4* q = reinterpret_cast<u32x4*>(p);
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (int i = tid; i < (bytes + 15) / 16; i += nthr) q[i] = z;
}

// The presence mask alone (enough for the threshold sample): ids[j] is history entry tid + j * NTHR.
template <int NTHR>
__device__ inline void build_bitmap(FS& S, const Hist& H, const int (&ids)[IDR], const int32_t* __restrict__ hist, int nnz, int V) {
  const int tid = threadIdx.x;
  const int n_pairs = (H.n_words + 1) >> 1;
  zero16(H.bm, n_pairs * 8, tid, NTHR);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < IDR; ++j) {
    const int i = tid + j * NTHR;
    if (i < nnz && (unsigned)ids[j] < (unsigned)V) atomicOr(&H.bm[ids[j] >> 5], 1u << (ids[j] & 31));
  }
  for (int i = tid + IDR * NTHR; i < nnz; i += NTHR) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) atomicOr(&H.bm[id >> 5], 1u << (id & 31));
  }
  __syncthreads();
}

// Builds bitmap, rank directory and counts of one row from the ids a thread holds in registers
// (ids[j] is history entry tid + j * NTHR) and, beyond those, from global memory.  own gets bit j
// set when this thread was the first to mark ids[j] (one owner per distinct id).  Out-of-range ids
// are ignored and flagged.
template <int NTHR>
__device__ inline void build_history(FS& S, const Hist& H, const int (&ids)[IDR], const int32_t* __restrict__ hist,
                                     int nnz, int n_prompt, int V, unsigned& own) {
  constexpr int NWV = NTHR / 64;
  const int tid = threadIdx.x;
  const int n_pairs = (H.n_words + 1) >> 1;
  zero16(H.bm, n_pairs * 8, tid, NTHR);
  zero16(H.cnt32, ((nnz + 2) / 2) * 4, tid, NTHR);
  __syncthreads();
  bool bad = false;
  own = 0u;
#pragma unroll
  for (int j = 0; j < IDR; ++j) {
    const int i = tid + j * NTHR;
    if (i < nnz) {
      if ((unsigned)ids[j] < (unsigned)V) {
        const uint32_t bit = 1u << (ids[j] & 31);
        if (!(atomicOr(&H.bm[ids[j] >> 5], bit) & bit)) own |= 1u << j;
      } else bad = true;
    }
  }
  for (int i = tid + IDR * NTHR; i < nnz; i += NTHR) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) atomicOr(&H.bm[id >> 5], 1u << (id & 31)); else bad = true;
  }
  if (bad) atomicOr(&S.flags, SIMPLE_DIAG_BAD_HISTORY_ID);
  __syncthreads();
  // directory: exclusive scan of the word pairs' popcounts, NTHR * 8 pairs per round
  unsigned carry = 0;
  for (int p0 = 0; p0 < n_pairs; p0 += NTHR * 8) {
    const int pb = p0 + tid * 8;
    unsigned pc[8], tot = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      pc[j] = (pb + j < n_pairs) ? (unsigned)(__popc(H.bm[2 * (pb + j)]) + __popc(H.bm[2 * (pb + j) + 1])) : 0u;
      tot += pc[j];
    }
    const unsigned incl = wave_incl_scan(tot);
    __syncthreads();
    if (lane_id() == 63) S.r32a[wave_id()] = incl;
    __syncthreads();
    unsigned base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NWV; ++w) { const unsigned x = S.r32a[w]; if (w < wave_id()) base += x; all += x; }
    unsigned run = carry + base + incl - tot;
#pragma unroll
    for (int j = 0; j < 8; ++j) { if (pb + j < n_pairs) H.dir[pb + j] = (uint16_t)run; run += pc[j]; }
    carry += all;
  }
  if (tid == 0) S.distinct = carry;
  __syncthreads();
  n_prompt = min(max(n_prompt, 0), nnz);
  auto count_one = [&](int id) {
    if ((unsigned)id < (unsigned)V) {
      const unsigned r = H.rank(id, H.bm[id >> 5]);
      atomicAdd(&H.cnt32[r >> 1], 1u << ((r & 1u) * 16u));
    }
  };
#pragma unroll
  for (int j = 0; j < IDR; ++j) { const int i = tid + j * NTHR; if (i >= n_prompt && i < nnz) count_one(ids[j]); }
  for (int i = tid + IDR * NTHR; i < nnz; i += NTHR) if (i >= n_prompt) count_one(hist[i]);
  __syncthreads();
}


// ---------------------------------------------------------------- stream ----------------------
struct StreamCtx {
  float g, y_g;    // candidate threshold on the logit, and its tempered value fl32(g / tau)
  double inv_tau;
  float l2e_tau;   // log2(e) / tau
  bool need_sum;   // the row needs the mass of the columns below g
};

// Whole-vocabulary nucleus (top-p over all of V, section 2.1 Eq. (2)): rows whose nucleus is wider
// than the candidate list are handed to three further kernels through a queue of records and one
// workspace slot per queued row.
struct WideRec {  // 64 bytes: everything the later kernels need to know about the row
  uint32_t row; float g; uint32_t mode, flags;
  float tau, top_p, rep, freq;
  float pres; int nnz, n_prompt, h_active;
  float min_p; int32_t top_k; uint32_t distinct, reserved1;
};
// What delimits the survivors of a queued row (each is a prefix of the total order, section 5.2):
enum { WIDE_TOP_P = 0,   // the shortest prefix whose mass reaches top_p of the row's mass
       WIDE_ALL = 1,     // no truncation: every column
       WIDE_MIN_P = 2,   // tempered value >= fl(y_max + fl(ln min_p))
       WIDE_TOP_K = 3 }; // the first top_k columns of the order (top-k alone, beyond the candidate list's reach)
constexpr int CNT_SHIFT = 46;  // top-k route: a bin's column count rides above its mass (< 2^18 columns of <= 2^28 each)
constexpr int WQ_HEAD = 16;             // words before the records
constexpr uint32_t WS_HIST = 0u;        // u64[NBW]: mass of the columns below g, by bin
constexpr uint32_t WS_TILES = 16384u;   // u64[2][256]: survivors' mass per tile, tail class then hot class
constexpr uint32_t WS_SCAL = 20480u;    // u64 mass at or above g; u32 sure survivors; u32 boundary columns; u64 exact mass
                                        // of the row; u32 largest key of a tempered value; u32 columns at or above g
constexpr uint32_t WS_RL = 20544u;      // u64[RCAP]: columns of the boundary bin (value bits << 32 | id)
constexpr uint32_t WS_HT = 53312u;      // the row's history tables as the single-pass kernel laid them out in LDS
// [0, WS_RL) must be zero when a row is queued

// Mass of one column relative to the mass at y_g, w = exp(y - y_g) with y = fl32(z / tau), and the
// bin of y (linear in y, so columns of equal y share a bin).  y is formed as fl32(double(z) * fl64(1 /
// tau)): the IEEE float32 quotient (see apply_penalties).  float32 exponential, split log2(e).
__device__ __forceinline__ float tempered(float z, const StreamCtx& C) { return (float)((double)z * C.inv_tau); }
// UNIT_TAU: the caller knows that tau == 1, where y is z itself (the same float as the product).
template <bool UNIT_TAU = false>
__device__ __forceinline__ float mass_term(float z, const StreamCtx& C, int& bin, float& y) {
  y = UNIT_TAU ? z : (float)((double)z * C.inv_tau);
  const float d = y - C.y_g;
  const float t = fmaf(d, L2E_HI, d * L2E_LO);
  bin = (int)fminf(fmaxf(-t * BINS_PER_LOG2, 0.0f), (float)(NBW - 1));
  return __builtin_amdgcn_exp2f(t);
}
template <bool UNIT_TAU = false>
__device__ __forceinline__ float mass_term(float z, const StreamCtx& C, int& bin) { float y; return mass_term<UNIT_TAU>(z, C, bin, y); }
constexpr float W_LIMIT = 2097152.0f;  // 2^21: largest mass relative to the one at g that the 2^28 fixed point carries
// Nearest integer of a float in [0, 2^52) as 64 bits, in two 32-bit conversions (the split is exact:
// a float has 24 significant bits): hi counts units of 2^24.  The two parts of several values can
// be summed separately in 32 bits and combined once.
__device__ __forceinline__ void float_to_parts(float v, uint32_t& hi, uint32_t& lo) {
  const float h = floorf(v * 0x1p-24f);
  hi = (uint32_t)h;
  lo = (uint32_t)(fmaf(-h, 0x1p24f, v) + 0.5f);  // v - h * 2^24 is exact either way
}
__device__ __forceinline__ u64 parts_to_u64(uint32_t hi, uint32_t lo) { return ((u64)hi << 24) + (u64)lo; }
__device__ __forceinline__ u64 float_to_u64(float v) {
  uint32_t hi, lo;
  float_to_parts(v, hi, lo);
  return parts_to_u64(hi, lo);
}
__device__ __forceinline__ u64 mass_fix(float w) { return float_to_u64(w * MSCALE); }
// same integer for w <= 1 (every column below g), one conversion instruction (the product with the
// scale is exact, so the fused form rounds once, as the sum does)
__device__ __forceinline__ u64 mass_fix_below(float w) { return (u64)(uint32_t)fmaf(w, MSCALE, 0.5f); }
// Mass of a column below g for the single-pass kernel's running total: exp((z - g) / tau) * 2^28
// without the exactly rounded tempered value; the scale rides in the exponent and the conversion
// rounds to nearest (truncating would lose half a unit per column, all in one direction: with V
// columns below a g that a min-p bound holds close to the row maximum that is V * 2^-29 of the mass
// at g, up to 4e-5 of the row's mass).  Relative error of the total below 1e-6 (rounding of the
// exponent at magnitude 28 and of the integer, independent from column to column), inside the 1e-5
// tolerance on probabilities; the total only decides whether the nucleus fits the list, and the
// list's target.
__device__ __forceinline__ uint32_t below_term(float z, const StreamCtx& C) {
  return (uint32_t)(__builtin_amdgcn_exp2f(fmaf(z - C.g, C.l2e_tau, 28.0f)) + 0.5f);
}
// The same for any column, without a test: a column at or above g (or a NaN) yields exactly 2^28, so
// a sum over all columns exceeds the mass below g by 2^28 times the number of columns at or above g.
__device__ __forceinline__ uint32_t below_term_clamped(float z, const StreamCtx& C) {
  return (uint32_t)(__builtin_amdgcn_exp2f(fminf(fmaf(z - C.g, C.l2e_tau, 28.0f), 28.0f)) + 0.5f);  // 2^28 + 0.5 is 2^28 in float32
}

}  // namespace fast

// The order in which the single-pass kernel's workgroups take the rows of a launch: rows with long
// epilogues first (a stable partition of 0 .. B-1 by long_epilogue), written to a.order by one
// workgroup of NT_ threads; `wsum` is LDS scratch of NT_ / 64 words.
template <int NT_>
__device__ __forceinline__ void order_rows_body(const SampleArgs& a, unsigned* wsum) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int PER = (WIDE_SLOTS + NT_ - 1) / NT_;  // rows per thread, contiguous (a launch has at most WIDE_SLOTS rows)
  const int r0 = tid * PER;
  unsigned flags = 0u, n_long = 0u;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int r = r0 + j;
    if (r < a.B && long_epilogue(a.params[r], a.V)) { flags |= 1u << j; ++n_long; }
  }
  const unsigned incl = wave_incl_scan(n_long);
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  unsigned before = 0u, total = 0u;
#pragma unroll
  for (int w = 0; w < NT_ / 64; ++w) { const unsigned x = wsum[w]; if (w < wave) before += x; total += x; }
  unsigned pos_long = before + incl - n_long;            // long rows before this thread's
  unsigned pos_short = total + (unsigned)min(r0, a.B) - pos_long;  // behind all long rows: short rows before this thread's
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int r = r0 + j;
    if (r < a.B) a.order[((flags >> j) & 1u) ? pos_long++ : pos_short++] = r;
  }
}

}  // namespace simple
