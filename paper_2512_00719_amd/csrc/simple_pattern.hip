// bfloat16 rows whose survivors are a long prefix of the vocabulary (top-p and / or min-p without
// top-k, no truncation, or a top-k beyond what the single-pass kernel's candidate list certifies:
// section 2.1 Eq. (2)) and that carry no penalties: the row is reduced to a count per distinct value.
//
// A bfloat16 logit has 16 bits, and under one temperature everything the filter and the softmax
// need of a column (its tempered value, its place in the order "value descending", its mass) is a
// function of that bit pattern.  One read of the row therefore only counts columns per pattern (an
// LDS integer atomic each); every order statistic then comes from the counts, exactly as it would
// from the sorted row:
//
//   counts    one pass over the row: hist[pattern] += 1;
//   cut       per occupied pattern one exponential gives the exact (2^44 fixed-point) mass of one of
//             its columns; exclusive sums over the patterns in descending value give, exactly as a
//             sorted row would, the row's mass, the min-p prefix, the shortest prefix that reaches
//             top_p of the mass, and the survivor count |K_b|.  Columns of one pattern tie: the cut
//             takes the first j of the cut pattern's columns in ascending id;
//   masses    one more read of the row, patterns looked up in a table (mass of a surviving column;
//             the cut pattern's entry counts instead), gives per tile of 2048 columns the mass of the
//             sure survivors, the hot part of it (section 5.3), and the cut pattern's columns, hot
//             and all.  The tile counts place the j-th column of the cut pattern; one tile is read
//             again for its id;
//   draw      the SHVS acceptance test on the class masses (Eq. (7)-(8)), the tile that holds u * S
//             from the tile masses of the drawn class, and a last read of that tile to locate the
//             id (inverse CDF in ascending id, step (3) of section 2.1).
//
// Patterns are kept for magnitudes from 2^-14 to 2^8 (2814 per sign).  Smaller magnitudes share one
// bin per sign, valued zero: the kernel checks that what this costs in mass stays five orders below
// the decision tolerance and that no cut falls into such a bin.  The last bin holds -inf (masked
// columns) and anything else at or below -256: columns without mass.  A row with a value of 256 or
// more, +inf or a NaN, or one that fails one of these checks, is left to the single-pass kernel, which
// runs after this one: this kernel leaves NOT_TAKEN as the id of every row it does not complete (the
// rows that are not of its route among them), and the single-pass kernel skips the others.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_rowdev.hpp"

namespace simple {
namespace pattern {

using namespace fast;

constexpr int PT = 512;        // threads per row
constexpr int PNW = PT / 64;
constexpr int PLO = 0x3882;    // smallest magnitude pattern with a bin of its own (just above 2^-14)
constexpr int PHI = 0x4380;    // 256.0: magnitudes from here on are not handled
constexpr int QMAX = PHI - PLO + 1;  // magnitude index: 0 merged, 1 .. QMAX - 1 one pattern each, QMAX too large
constexpr int NMAG = QMAX + 1;
constexpr int NB = 2 * NMAG;   // bins in descending value: positive patterns from the largest down, then negative ones
constexpr int BPT = NB / PT;   // bins per thread in the cut phase
static_assert(NB % PT == 0, "bins divide among the threads");
constexpr int TG = 4;          // 16-byte groups per lane and tile
constexpr int TILE = 64 * 8 * TG;  // columns per tile of the second pass, one wave each
constexpr int NTILE = (1 << 18) / TILE;  // V < 2^18
static_assert(NTILE <= PT, "one tile per thread in the scans over tiles");
constexpr int UN = 4;          // 16-byte loads in flight per lane, twice (two register sets take turns)
constexpr uint32_t FILL = 0xFF80FF80u;  // two patterns (-inf) of the last bin, whose columns have no mass
constexpr int CBIT = 58;       // a table entry counts a column of the cut pattern from this bit up
constexpr u64 MASS_PART = (1ull << CBIT) - 1ull;
static_assert(TILE / 64 < (1 << (64 - CBIT)), "a lane's columns of one tile fit the count");

typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// bin of a bit pattern (its 16 low bits)
__device__ __forceinline__ int bin_of(uint32_t raw) {
  const int p = (int)(raw & 0x7FFFu);
  const int s = -(int)((raw >> 15) & 1u);
  const int q = min(max(p - (PLO - 1), 0), QMAX);
  return (NMAG - 1) - (q ^ s);
}
// The same for the two patterns of a 32-bit word at once (packed 16-bit arithmetic), as byte offsets
// into a table of (1 << SHIFT)-byte entries, low pattern in the low half.  TRACK: smax gathers the
// largest patterns read as signed numbers (the largest positive value), umax read as unsigned
// numbers (the negative value of the largest magnitude, if there is a negative one).
template <bool TRACK, int SHIFT>
__device__ __forceinline__ uint32_t bin_offsets2(uint32_t x, s16x2& smax, u16x2& umax) {
  const s16x2 xs = __builtin_bit_cast(s16x2, x);
  if (TRACK) {
    smax = __builtin_elementwise_max(smax, xs);
    umax = __builtin_elementwise_max(umax, __builtin_bit_cast(u16x2, x));
  }
  const s16x2 s = xs >> (short)15;
  const s16x2 p = xs & (short)0x7FFF;
  s16x2 q = __builtin_elementwise_max((s16x2)(p - (short)(PLO - 1)), (s16x2)((short)0));
  q = __builtin_elementwise_min(q, (s16x2)((short)QMAX));
  const s16x2 d = (short)(NMAG - 1) - (q ^ s);
  return __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, d) << (unsigned short)SHIFT));
}
// bit pattern of a bin (zero for the merged bins)
__device__ __forceinline__ uint32_t raw_of(int d) {
  const int s = d >= NMAG ? 1 : 0;
  const int q = s ? d - NMAG : NMAG - 1 - d;
  const uint32_t p = q == 0 ? 0u : (uint32_t)(q + PLO - 1);
  return ((uint32_t)s << 15) | p;
}
__device__ __forceinline__ bool merged_bin(int d) { return d == NMAG - 1 || d == NMAG; }
__device__ __forceinline__ float value_of(uint32_t raw) { return __uint_as_float(raw << 16); }
// Nearest integer to exp(y - y_max) * 2^44: 2^n * 2^f with n = rint(x log2 e) and the Taylor
// polynomial of degree 10 for 2^f on [-1/2, 1/2] (relative error below 1e-12).
__device__ __forceinline__ u64 mass_fix44(float y, float y_max) {
  const double x = (double)y - (double)y_max;
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
  return (u64)__double2ull_rn(ldexp(p, (int)n + 44));
}

// Sum over the wave, the same in every lane (data-parallel primitives: no LDS, no waiting).
template <typename T>
__device__ __forceinline__ T wave_total(T v) { return wave_sum(v); }

struct PS {  // row-wide state
  int dtop, dcut, bad, tdraw, id_cut, partial, pos_max;
  unsigned neg_max, pos_m, pos_p, jcut, ccut, tcut, rcut, hot_before, hot_in, merged_n;
  u64 mcut, sure_all, mab, m_merged, s_k;
};

// The 16-byte groups of a tile that a lane holds (group g < n_groups), and the hot bits of their columns.
struct TileRegs { u32x4 r[TG]; uint32_t hq[TG]; };
template <bool USE_HOT>
__device__ __forceinline__ void tile_load(TileRegs& R, const uint16_t* rowp, const uint32_t* hot_bits, int tile, int lane, int n_groups) {
#pragma unroll
  for (int h = 0; h < TG; ++h) {
    const int g = tile * (TILE / 8) + h * 64 + lane;
    R.r[h] = u32x4{FILL, FILL, FILL, FILL};
    R.hq[h] = 0u;
    if (g < n_groups) {
      R.r[h] = *as_global(reinterpret_cast<const u32x4*>(rowp) + g);
      if (USE_HOT) R.hq[h] = (as_global(hot_bits)[g >> 2] >> ((g & 3) * 8)) & 0xFFu;
    }
  }
}
__device__ __forceinline__ uint32_t raw_at(const u32x4& r, int e) {
  const uint32_t w = (e >> 1) == 0 ? r.x : (e >> 1) == 1 ? r.y : (e >> 1) == 2 ? r.z : r.w;
  return (e & 1) ? (w >> 16) : (w & 0xFFFFu);
}

template <bool USE_HOT>
__global__ __launch_bounds__(PT, 4) void pattern_rows_kernel(const SampleArgs a) {
  __shared__ __align__(16) u64 tab[NB];   // 32-bit counts (in its first half) in the first pass, then per bin the mass of a surviving column
  __shared__ u64 tall[NTILE], thot[NTILE];  // per tile: mass of the sure survivors, and of the hot ones among them
  __shared__ uint32_t tcc[NTILE];           // per tile: columns of the cut pattern, the hot ones among them from bit 16
  __shared__ PS P;
  __shared__ FS S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int V = a.V;
  if (row == a.B) {  // the workgroup behind the rows: the order in which the kernel after this one takes them
    order_rows_body<PT>(a, reinterpret_cast<unsigned*>(tcc));
    return;
  }
  const simple_row_params par = a.params[row];
  {
    const RowHist rh = row_history(a, row, par.n_prompt);
    // (ahead of the hot-first kernel: not the rows that kernel decides from the hot columns alone)
    if (!pattern_route(par, V, rh.nnz, a.max_nnz) || (a.pattern_on == 2 && hot_first_plain(par, V))) {  // the kernel behind this one takes the row
      if (threadIdx.x == 0) a.out[row] = NOT_TAKEN;
      return;
    }
  }
  const uint16_t* rowp = reinterpret_cast<const uint16_t*>(a.logits) + (size_t)row * (size_t)a.stride;
  const uint32_t* hot_bits = a.hot_bits;
  const int n_groups = V >> 3;          // whole 16-byte groups; the columns behind them are read one by one
  const int n_tiles = (V + TILE - 1) / TILE;
  const float tau = par.temperature;
  unsigned char* tabb = reinterpret_cast<unsigned char*>(tab);
  const u32x4* rp = reinterpret_cast<const u32x4*>(rowp);
  auto hand_back = [&]() { if (tid == 0) a.out[row] = NOT_TAKEN; };

  // ---- first pass: columns per pattern ----
  u32x4 A[UN], Bq[UN];
  auto fetch = [&](u32x4 (&R)[UN], int g0) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int g = g0 + u * PT + tid;
      R[u] = u32x4{0u, 0u, 0u, 0u};
      if (g < n_groups) R[u] = *as_global(rp + g);
    }
  };
  fetch(A, 0);
  for (int i = tid; i < NB / 2; i += PT) tab[i] = 0ull;
  if (tid == 0) {
    P.dtop = NB; P.dcut = -1; P.bad = 0; P.tdraw = -1; P.id_cut = -1; P.partial = 0;
    P.pos_max = 0; P.neg_max = 0u; P.pos_m = 0u; P.pos_p = 0u; P.jcut = 0u; P.ccut = 0u; P.tcut = 0u; P.rcut = 0u; P.hot_before = 0u; P.hot_in = 0u; P.merged_n = 0u;
    P.mcut = 0ull; P.sure_all = 0ull; P.mab = 0ull; P.m_merged = 0ull; P.s_k = 0ull;
  }
  __syncthreads();
  s16x2 smax = {0, 0};  // largest positive patterns seen by this thread
  u16x2 umax = {0, 0};  // negative patterns of the largest magnitude (any negative one is above every positive one)
  auto count2 = [&](uint32_t x) {
    const uint32_t off = bin_offsets2<true, 2>(x, smax, umax);
    __hip_atomic_fetch_add(reinterpret_cast<uint32_t*>(tabb + (off & 0xFFFFu)), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_add(reinterpret_cast<uint32_t*>(tabb + (off >> 16)), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  };
  auto consume = [&](const u32x4 (&R)[UN], int g0) {
#pragma unroll
    for (int u = 0; u < UN; ++u)
      if (g0 + u * PT + tid < n_groups) { count2(R[u].x); count2(R[u].y); count2(R[u].z); count2(R[u].w); }
  };
  for (int g0 = 0; g0 < n_groups; g0 += 2 * UN * PT) {
    fetch(Bq, g0 + UN * PT);
    consume(A, g0);
    fetch(A, g0 + 2 * UN * PT);
    consume(Bq, g0 + UN * PT);
  }
  int pos_max = max((int)smax.x, (int)smax.y);
  uint32_t neg_max = max((uint32_t)umax.x, (uint32_t)umax.y);
  if (tid < V - n_groups * 8) {  // the ragged end of the row
    const uint32_t raw = (uint32_t)*as_global(rowp + n_groups * 8 + tid);
    __hip_atomic_fetch_add(reinterpret_cast<uint32_t*>(tabb + 4 * bin_of(raw)), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    pos_max = max(pos_max, (int)(short)raw);
    neg_max = max(neg_max, raw);
  }
  pos_max = (int)wave_max_u32((uint32_t)max(pos_max, 0));
  neg_max = wave_max_u32(neg_max);
  if (lane == 0) { atomicMax(&P.pos_max, pos_max); atomicMax(&P.neg_max, neg_max); }
  __syncthreads();

  // ---- the cut, from the counts ----
  const int d_first = tid * BPT;
  uint32_t ca[BPT];
  unsigned csum = 0u;
  {
    int dfirst = NB;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      ca[j] = reinterpret_cast<const uint32_t*>(tab)[d_first + j];
      csum += ca[j];
      if (ca[j] && dfirst == NB) dfirst = d_first + j;
    }
    if (dfirst < NB) atomicMin(&P.dtop, dfirst);
  }
  __syncthreads();
  const int dtop = P.dtop;
  // a positive magnitude outside the bins (also: +inf, NaN), a negative NaN, or a row maximum inside a
  // merged bin or in the last bin (every column at or below -256)
  if (P.pos_max >= PHI || P.neg_max > 0xFF80u || dtop >= NB - 1 || merged_bin(dtop)) { hand_back(); return; }
  const float y_max = value_of(raw_of(dtop)) / tau;
  if (!(fabsf(y_max) < INFINITY)) { hand_back(); return; }  // the division overflowed: an error row, reported by the other kernels
  const bool p_on = par.top_p < 1.0f, minp_on = par.min_p > 0.0f;
  // The last bin holds -inf (masked columns) and whatever else lies at or below -256: its columns
  // count as survivors where nothing is truncated, with no mass.  That is exact for -inf; for a
  // finite value it requires that the value's mass rounds to nothing (31 below the maximum in the
  // exponent) and, with min-p, that no threshold reaches that far down (ln of the smallest float32 is -103.3).
  if (P.neg_max >= (0x8000u | (uint32_t)PHI) && !((value_of(raw_of(dtop)) + 256.0f) / tau >= (minp_on ? 104.0f : 32.0f))) { hand_back(); return; }
  const float thr_y = minp_on ? y_max + (float)log((double)par.min_p) : -INFINITY;
  u64 mb[BPT];
  u64 msum = 0ull;
  uint32_t ge_thr = 0u;  // bins at or above the min-p threshold
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    mb[j] = 0ull;
    if (ca[j] && d_first + j < NB - 1) {
      const float y = value_of(raw_of(d_first + j)) / tau;
      mb[j] = mass_fix44(y, y_max);
      ge_thr |= (y >= thr_y) ? (1u << j) : 0u;
      if (merged_bin(d_first + j)) { atomicAdd(&P.merged_n, ca[j]); P.m_merged = mb[j]; }
    }
    msum += (u64)ca[j] * mb[j];
  }
  unsigned ce, ct; u64 me, s_tot;
  blk_excl_scan2<PNW>(S, csum, msum, ce, me, ct, s_tot);  // barriers inside
  // top-k (only above what the single-pass kernel's list certifies): exactly k columns, and S_k, the mass of that prefix
  const bool k_on = par.top_k >= 1 && par.top_k < V;
  u64 s_k = s_tot;
  if (k_on) {
    unsigned cb = ce; u64 mbef = me;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      if (ca[j] && cb < (unsigned)par.top_k && (unsigned)par.top_k <= cb + ca[j]) P.s_k = mbef + (u64)((unsigned)par.top_k - cb) * mb[j];
      cb += ca[j]; mbef += (u64)ca[j] * mb[j];
    }
    __syncthreads();
    s_k = P.s_k;
  }
  const u64 target = p_on ? (u64)__double2ull_ru((double)par.top_p * (double)s_k) : 0ull;
  {
    unsigned cb = ce; u64 mbef = me;
    unsigned pos_m = 0u;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      const u64 bm = (u64)ca[j] * mb[j];
      if (minp_on && ((ge_thr >> j) & 1u)) pos_m = cb + ca[j];
      if (p_on && bm > 0ull && mbef < target && mbef + bm >= target) P.pos_p = cb + (unsigned)((target - mbef + mb[j] - 1ull) / mb[j]);
      cb += ca[j]; mbef += bm;
    }
    if (pos_m) atomicMax(&P.pos_m, pos_m);
  }
  __syncthreads();
  // what the merged bins cost: their columns are valued zero, off by up to 6.2e-5 / tau in the exponent
  if (P.merged_n) {
    const double err = (double)P.merged_n * (double)P.m_merged * (6.2e-5 / (double)tau);
    const bool near_thr = minp_on && fabsf(thr_y) * tau <= 1.3e-4f;
    if (err > (double)s_k * 0x1p-24 || near_thr) { hand_back(); return; }
  }
  unsigned n = k_on ? (unsigned)par.top_k : (unsigned)V;
  if (minp_on) n = min(n, P.pos_m);
  if (p_on && P.pos_p) n = min(n, P.pos_p);
  n = max(n, 1u);
  {
    unsigned cb = ce; u64 mbef = me;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      if (ca[j] && cb < n && n <= cb + ca[j]) {
        P.dcut = d_first + j; P.jcut = n - cb; P.ccut = ca[j]; P.mcut = mb[j]; P.sure_all = mbef;
        P.partial = (n - cb < ca[j]) ? 1 : 0;
      }
      cb += ca[j]; mbef += (u64)ca[j] * mb[j];
    }
  }
  __syncthreads();
  const int dcut = P.dcut;
  const bool partial = P.partial != 0;
  if (dcut < 0 || (partial && (merged_bin(dcut) || dcut == NB - 1))) { hand_back(); return; }
  const u64 mcut = P.mcut;
  const uint32_t cut_raw = raw_of(dcut);
  // from here on the table holds, per bin, the mass of a surviving column; a cut pattern of which
  // only a part survives counts its columns instead
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    const int d = d_first + j;
    tab[d] = d < dcut ? mb[j] : (d == dcut ? (partial ? 1ull << CBIT : mb[j]) : 0ull);
  }
  __syncthreads();

  // ---- second pass: per tile, mass of the sure survivors (all, hot) and columns of the cut pattern ----
  auto ragged_each = [&](auto&& f) {  // the columns behind the last whole group, in ascending id (one thread calls)
    for (int idx = n_groups * 8; idx < V; ++idx) f((uint32_t)*as_global(rowp + idx), idx);
  };
  {
    TileRegs R{}, N{};
    if (wave < n_tiles) tile_load<USE_HOT>(R, rowp, hot_bits, wave, lane, n_groups);
    for (int t = wave; t < n_tiles; t += PNW) {
      if (t + PNW < n_tiles) tile_load<USE_HOT>(N, rowp, hot_bits, t + PNW, lane, n_groups);
      u64 acc = 0ull, acc_h = 0ull;
#pragma unroll
      for (int h = 0; h < TG; ++h) {  // (groups behind the row's end hold FILL: -inf, no mass)
        const uint32_t w4[4] = {R.r[h].x, R.r[h].y, R.r[h].z, R.r[h].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          s16x2 unused_s = {0, 0};
          u16x2 unused_u = {0, 0};
          const uint32_t off = bin_offsets2<false, 3>(w4[k], unused_s, unused_u);
          const u64 m0 = *reinterpret_cast<const u64*>(tabb + (off & 0xFFFFu));
          const u64 m1 = *reinterpret_cast<const u64*>(tabb + (off >> 16));
          acc += m0 + m1;
          if (USE_HOT) {
            const u64 h0 = 0ull - (u64)((R.hq[h] >> (2 * k)) & 1u), h1 = 0ull - (u64)((R.hq[h] >> (2 * k + 1)) & 1u);
            acc_h += (m0 & h0) + (m1 & h1);
          }
        }
      }
      const uint32_t cc = (uint32_t)(acc >> CBIT) | ((uint32_t)(acc_h >> CBIT) << 16);
      const u64 s_all = wave_total(acc & MASS_PART);
      const u64 s_hot = USE_HOT ? wave_total(acc_h & MASS_PART) : 0ull;
      const uint32_t s_cc = partial ? wave_total(cc) : 0u;
      if (lane == 0) { tall[t] = s_all; thot[t] = s_hot; tcc[t] = s_cc; }
      R = N;
    }
  }
  __syncthreads();
  if (tid == 0 && V > n_groups * 8) {  // the ragged end of the row belongs to the last tile
    u64 s_all = 0ull, s_hot = 0ull; uint32_t cc = 0u;
    ragged_each([&](uint32_t raw, int idx) {
      const u64 m = tab[bin_of(raw)];
      const bool hot = USE_HOT && hot_bit(hot_bits, (uint32_t)idx);
      s_all += m & MASS_PART; cc += (uint32_t)(m >> CBIT);
      if (hot) { s_hot += m & MASS_PART; cc += (uint32_t)(m >> CBIT) << 16; }
    });
    tall[n_tiles - 1] += s_all; thot[n_tiles - 1] += s_hot; tcc[n_tiles - 1] += cc;
  }
  __syncthreads();
  const u64 my_all = tid < n_tiles ? tall[tid] : 0ull, my_hot = tid < n_tiles ? thot[tid] : 0ull;
  const uint32_t my_cc = tid < n_tiles ? tcc[tid] : 0u;

  // ---- a cut inside a pattern: the id of its j-th column in ascending id ----
  if (partial) {
    {
      const unsigned c = my_cc & 0xFFFFu;
      unsigned ce2, ct2; u64 he2, ht2;
      blk_excl_scan2<PNW>(S, c, (u64)(my_cc >> 16), ce2, he2, ct2, ht2);
      if (c && ce2 < P.jcut && P.jcut <= ce2 + c) { P.tcut = (unsigned)tid; P.rcut = P.jcut - ce2; P.hot_before = (unsigned)he2; }
      if (tid == 0 && ct2 != P.ccut) P.bad = 1;  // the passes disagree
    }
    __syncthreads();
    if (P.bad || P.rcut == 0u) { hand_back(); return; }
    if (wave == 0) {  // the r-th match inside the tile, and the hot ones among the matches up to it
      const int t = (int)P.tcut;
      const unsigned r = P.rcut;
      TileRegs R;
      tile_load<USE_HOT>(R, rowp, hot_bits, t, lane, n_groups);
      // matches per 16-byte group of each lane; the group row (64 groups) that holds the r-th match
      uint32_t mm[TG];
      unsigned tot[TG];
#pragma unroll
      for (int h = 0; h < TG; ++h) {
        const bool in = t * (TILE / 8) + h * 64 + lane < n_groups;
        mm[h] = 0u;
#pragma unroll
        for (int e = 0; e < 8; ++e) mm[h] |= (in && raw_at(R.r[h], e) == cut_raw) ? (1u << e) : 0u;
        tot[h] = wave_total((uint32_t)__popc(mm[h]));
      }
      unsigned before = 0u, hot_in = 0u;
      int id = -1;
      bool found = false;
#pragma unroll
      for (int h = 0; h < TG; ++h) {
        if (found) continue;
        if (before + tot[h] < r) {  // all of this group row's matches come before the r-th
          hot_in += (unsigned)__popc(mm[h] & R.hq[h]);
          before += tot[h];
          continue;
        }
        found = true;
        const unsigned c = (unsigned)__popc(mm[h]);
        const unsigned lo = before + wave_incl_scan(c) - c;  // matches before this lane's
        uint32_t keep = 0u;                                   // this lane's matches that are among the first r
        if (lo + c <= r) keep = mm[h];
        else if (lo < r) {
          uint32_t m = mm[h];
          for (unsigned k = lo; k < r; ++k) { keep |= m & (0u - m); m &= m - 1u; }
        }
        hot_in += (unsigned)__popc(keep & R.hq[h]);
        const u64 bal = __ballot(c > 0u && lo < r && r <= lo + c);
        if (bal) {
          const int src = (int)__ffsll((long long)bal) - 1;
          const int e_last = 31 - __clz((int)(keep | 1u));  // only meaningful in the lane `src`
          id = __shfl((t * (TILE / 8) + h * 64 + lane) * 8 + e_last, src, 64);
        }
        before += tot[h];
      }
      hot_in = wave_total(hot_in);
      if (lane == 0) {
        if (id < 0 && t == n_tiles - 1) {  // among the columns behind the last whole group
          unsigned k = before;
          ragged_each([&](uint32_t raw, int idx) {
            if (raw == cut_raw && id < 0) {
              ++k;
              if (USE_HOT && hot_bit(hot_bits, (uint32_t)idx)) ++hot_in;
              if (k == r) id = idx;
            }
          });
        }
        P.id_cut = id;
        P.hot_in = hot_in;
      }
    }
    __syncthreads();
    if (P.id_cut < 0) { hand_back(); return; }
  }
  const int id_cut = P.id_cut;
  const int tcut = partial ? (int)P.tcut : -1;

  // ---- class masses, acceptance (section 5.3), the draw's target ----
  double u3[3];
  row_uniforms(a.seed, a.row_offset + (uint64_t)row, a.step, u3);
  const u64 sum_all = blk_sum_u64<PNW>(S, my_all);  // barriers inside
  const u64 sum_hot = USE_HOT ? blk_sum_u64<PNW>(S, my_hot) : 0ull;
  const u64 sure = partial ? P.sure_all : P.sure_all + (u64)P.jcut * mcut;
  if (sum_all != sure) { hand_back(); return; }  // the passes disagree
  const u64 S_K = P.sure_all + (u64)P.jcut * mcut;
  const u64 S_H = USE_HOT ? sum_hot + (partial ? (u64)(P.hot_before + P.hot_in) * mcut : 0ull) : 0ull;
  bool pick_hot = false;
  if (USE_HOT) pick_hot = (S_H > 0ull) && (u3[1] * (double)S_K <= (double)S_H);
  const uint32_t cls = pick_hot ? 1u : 0u;
  const u64 S_cls = USE_HOT ? (pick_hot ? S_H : S_K - S_H) : S_K;
  const double u = USE_HOT ? (pick_hot ? u3[0] : u3[2]) : u3[0];
  if (S_cls == 0ull) { hand_back(); return; }
  u64 tfix = (u64)__double2ull_rd(u * (double)S_cls);
  if (tfix >= S_cls) tfix = S_cls - 1ull;
  {  // the tile that holds the draw, from the tile masses of the drawn class
    u64 m = USE_HOT ? (pick_hot ? my_hot : my_all - my_hot) : my_all;
    if (partial && tid < n_tiles) {
      const unsigned c_all = my_cc & 0xFFFFu, c_hot = my_cc >> 16;
      unsigned c = USE_HOT ? (pick_hot ? c_hot : c_all - c_hot) : c_all;
      if (tid == tcut) c = USE_HOT ? (pick_hot ? P.hot_in : P.rcut - P.hot_in) : P.rcut;
      if (tid <= tcut) m += (u64)c * mcut;
    }
    unsigned ce3, ct3; u64 me3, mt3;
    blk_excl_scan2<PNW>(S, 0u, m, ce3, me3, ct3, mt3);
    if (m > 0ull && me3 <= tfix && tfix < me3 + m) { P.tdraw = tid; P.mab = me3; }
    if (tid == 0 && mt3 != S_cls) P.bad = 1;  // the passes disagree
  }
  __syncthreads();
  if (P.bad || P.tdraw < 0) { hand_back(); return; }
  // ---- the drawn id inside its tile ----
  if (wave == 0) {
    // mass of one column in the drawn class (zero outside it and outside K_b)
    auto col_mass = [&](uint32_t raw, uint32_t hot, int idx) -> u64 {
      if (USE_HOT && hot != cls) return 0ull;
      const u64 m = tab[bin_of(raw)];
      if (m >> CBIT) return idx <= id_cut ? mcut : 0ull;
      return m;
    };
    const int t = P.tdraw;
    TileRegs R;
    tile_load<USE_HOT>(R, rowp, hot_bits, t, lane, n_groups);
    u64 base = P.mab;
    int id = -1; u64 w_id = 0ull; uint32_t raw_id = 0u;
    u64 ls[TG], tot[TG];  // mass of each lane's 16-byte groups, and of each group row (64 groups)
#pragma unroll
    for (int h = 0; h < TG; ++h) {
      const int idx0 = (t * (TILE / 8) + h * 64 + lane) * 8;
      ls[h] = 0ull;
      if (idx0 < n_groups * 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ls[h] += col_mass(raw_at(R.r[h], e), (R.hq[h] >> e) & 1u, idx0 + e);
      }
      tot[h] = wave_total(ls[h]);
    }
    bool found = false;
#pragma unroll
    for (int h = 0; h < TG; ++h) {
      if (found) continue;
      if (base + tot[h] <= tfix) { base += tot[h]; continue; }
      found = true;  // the draw lies in this group row
      const int idx0 = (t * (TILE / 8) + h * 64 + lane) * 8;
      u64 run = base + wave_incl_scan(ls[h]) - ls[h];
      if (ls[h] > 0ull && run <= tfix && tfix < run + ls[h]) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const u64 m = col_mass(raw_at(R.r[h], e), (R.hq[h] >> e) & 1u, idx0 + e);
          if (m > 0ull && run <= tfix && tfix < run + m) { id = idx0 + e; w_id = m; raw_id = raw_at(R.r[h], e); }
          run += m;
        }
      }
      base += tot[h];
    }
    const u64 bal = __ballot(id >= 0);
    if (bal) {
      const int src = (int)__ffsll((long long)bal) - 1;
      id = __shfl(id, src, 64); w_id = __shfl(w_id, src, 64); raw_id = (uint32_t)__shfl((int)raw_id, src, 64);
    } else if (lane == 0 && t == n_tiles - 1) {
      u64 run = base;
      ragged_each([&](uint32_t raw, int idx) {
        const u64 m = col_mass(raw, USE_HOT ? hot_bit(hot_bits, (uint32_t)idx) : 0u, idx);
        if (m > 0ull && run <= tfix && tfix < run + m) { id = idx; w_id = m; raw_id = raw; }
        run += m;
      });
    }
    if (lane == 0) {
      if (id < 0) a.out[row] = NOT_TAKEN;
      else {
        // a column of a merged bin was walked with the bin's mass; its own is reported
        if (merged_bin(bin_of(raw_id))) w_id = mass_fix44(value_of(raw_id) / tau, y_max);
        simple_row_diag dg;
        dg.alpha = USE_HOT ? (double)S_H / (double)S_K : __longlong_as_double(0x7FF8000000000000ll);
        dg.s_k = (double)s_k / WSCALE;
        dg.p_chosen = (float)((double)w_id / (double)S_K);
        dg.n_survivors = (int)n;
        dg.reserved = 0u;
        dg.flags = SIMPLE_DIAG_WIDE | SIMPLE_DIAG_PATTERN | (USE_HOT ? (SIMPLE_DIAG_SHVS | (pick_hot ? SIMPLE_DIAG_ACCEPTED : 0u)) : 0u);
        if (USE_HOT && a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
        a.out[row] = id;
        if (a.diag) a.diag[row] = dg;
        if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
        write_decision(a, row, id, dg.p_chosen, false);
      }
    }
  }
}

}  // namespace pattern

hipError_t launch_pattern(const SampleArgs& a, hipStream_t st) {
  if (a.B <= 0) return hipSuccess;
  // (one more workgroup when the single-pass kernel behind this one takes its rows in a written order:
  // it writes that order, which saves the launch of a kernel for it)
  const dim3 grid((unsigned)a.B + (a.order && a.pattern_on == 1 ? 1u : 0u));
  if (a.hot_bits) hipLaunchKernelGGL((pattern::pattern_rows_kernel<true>), grid, dim3(pattern::PT), 0, st, a);
  else hipLaunchKernelGGL((pattern::pattern_rows_kernel<false>), grid, dim3(pattern::PT), 0, st, a);
  return hipGetLastError();
}

}  // namespace simple
