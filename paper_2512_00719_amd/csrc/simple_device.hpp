// Device-side building blocks shared by the sampling kernels: orderable float keys, wave/block
// scans and reductions, the counter-based random numbers, and the per-row history state that
// drives the penalties.  gfx950 only (wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_sample.h"

namespace simple {

constexpr int NT = 512;        // threads per row workgroup
constexpr int NW = NT / 64;    // waves per workgroup
constexpr int CAP = 4096;      // candidate-list capacity (entries)
constexpr int KMAX = 1024;     // largest prefix the candidate list certifies
constexpr int NBINS = 2048;    // radix histogram bins (11 bits)
constexpr int UNROLL = 4;      // 16-byte loads in flight per lane
constexpr int QBITS = 43;      // fixed-point scale of probability mass on the multi-pass route

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Order-preserving map float -> uint32 (larger float, larger key); -0 and +0 share a key.
// Keys of non-NaN values lie in [key(-inf), key(+inf)] = [0x007FFFFF, 0xFF800000]; 0 is free and
// serves as the "dropped entry" mark.
__device__ __forceinline__ uint32_t fkey(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float keyf(uint32_t k) {
  uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __uint_as_float(b);
}
constexpr uint32_t KEY_NEG_INF = 0x007FFFFFu;
constexpr uint32_t KEY_POS_INF = 0xFF800000u;

// ---------------------------------------------------------------- wave / block collectives ----
// Built on the data-parallel primitives (a lane reads another lane's register inside the vector
// unit: no trip through the LDS pipe, which a shuffle would take and wait for).  All 64 lanes of the
// wave must be active.
// A value moved between lanes: CTRL selects the pattern; lanes of rows outside ROW_MASK, and lanes
// whose source lies outside the row, keep `old`.
template <int CTRL, int ROW_MASK, typename T>
__device__ __forceinline__ T dpp_move(T old, T v) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit values");
  if constexpr (sizeof(T) == 4) {
    const int r = __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false);
    return __builtin_bit_cast(T, r);
  } else {
    const unsigned long long o = __builtin_bit_cast(unsigned long long, old), x = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp((int)(unsigned)o, (int)(unsigned)x, CTRL, ROW_MASK, 0xF, false);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp((int)(unsigned)(o >> 32), (int)(unsigned)(x >> 32), CTRL, ROW_MASK, 0xF, false);
    return __builtin_bit_cast(T, ((unsigned long long)hi << 32) | (unsigned long long)lo);
  }
}
template <typename T>
__device__ __forceinline__ T read_lane(T v, int lane) {  // `lane` must be the same in every lane
  if constexpr (sizeof(T) == 4) return __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
  else {
    const unsigned long long x = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)x, lane), hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(x >> 32), lane);
    return __builtin_bit_cast(T, ((unsigned long long)hi << 32) | (unsigned long long)lo);
  }
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;  // partners inside a row of 16 lanes
constexpr int DPP_BCAST15 = 0x142, DPP_BCAST31 = 0x143;  // last lane of a row (of the first two rows) to the next row (the last two)
template <int N> constexpr int dpp_row_shr() { return 0x110 + N; }
// f over all 64 lanes, the same in every lane: a butterfly inside each row of 16, then the four rows.
template <typename T, typename F>
__device__ __forceinline__ T wave_all(T v, F&& f) {
  v = f(v, dpp_move<DPP_XOR1, 0xF>(v, v));
  v = f(v, dpp_move<DPP_XOR2, 0xF>(v, v));
  v = f(v, dpp_move<DPP_HALF_MIRROR, 0xF>(v, v));
  v = f(v, dpp_move<DPP_MIRROR, 0xF>(v, v));
  return f(f(read_lane(v, 0), read_lane(v, 16)), f(read_lane(v, 32), read_lane(v, 48)));
}
template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {  // sums of lanes 0 .. l
  const T zero = T(0);
  v += dpp_move<dpp_row_shr<1>(), 0xF>(zero, v);
  v += dpp_move<dpp_row_shr<2>(), 0xF>(zero, v);
  v += dpp_move<dpp_row_shr<4>(), 0xF>(zero, v);
  v += dpp_move<dpp_row_shr<8>(), 0xF>(zero, v);
  v += dpp_move<DPP_BCAST15, 0xA>(zero, v);
  v += dpp_move<DPP_BCAST31, 0xC>(zero, v);
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
  return wave_all(v, [](T a, T b) { return a + b; });
}
__device__ __forceinline__ float wave_max(float v) {
  return wave_all(v, [](float a, float b) { return fmaxf(a, b); });
}

// Block-wide inclusive scan; `ws` is LDS scratch of NW+1 elements.  All threads must call.
template <typename T>
__device__ inline T block_incl_scan(T v, T* ws, T& total) {
  T incl = wave_incl_scan(v);
  __syncthreads();
  if (lane_id() == 63) ws[wave_id()] = incl;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    T x = ws[w];
    if (w < wave_id()) base += x;
    tot += x;
  }
  total = tot;
  return incl + base;
}
// Block-wide sum with a fixed reduction tree (bit-reproducible).
template <typename T>
__device__ inline T block_sum(T v, T* ws) {
  T s = wave_sum(v);
  __syncthreads();
  if (lane_id() == 0) ws[wave_id()] = s;
  __syncthreads();
  T tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) tot += ws[w];
  return tot;
}
__device__ inline float block_max(float v, float* ws) {
  float s = wave_max(v);
  __syncthreads();
  if (lane_id() == 0) ws[wave_id()] = s;
  __syncthreads();
  float m = ws[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) m = fmaxf(m, ws[w]);
  return m;
}

// ---------------------------------------------------------------- random numbers --------------
// Philox4x32 with 10 rounds (Salmon et al., SC'11), one block per (row, step); see the header
// for the key/counter convention (deterministic random numbers, paper section 5.1).
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                     uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    if (r < 9) { k0 += W0; k1 += W1; }
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
__device__ inline void row_uniforms(uint64_t seed, uint64_t row, uint64_t step, double (&u)[3]) {
  uint32_t x[4];
  philox4x32_10((uint32_t)row, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t)(row >> 32), (uint32_t)seed,
                (uint32_t)(seed >> 32), x);
#pragma unroll
  for (int i = 0; i < 3; ++i) u[i] = (double)(x[i] >> 8) * 0x1p-24;
}

// ---------------------------------------------------------------- aggregate over rows ---------
// One completed row's share of the optional aggregate (called by one thread per row).  Integer
// atomics only: the sums do not depend on the order in which rows finish.
constexpr uint32_t DIAG_ERROR_BITS = SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_PARAM | SIMPLE_DIAG_BAD_LOGIT | SIMPLE_DIAG_BAD_HISTORY_ID |
                                     SIMPLE_DIAG_HISTORY_TOO_LONG | SIMPLE_DIAG_BAD_HOT_SET;
__device__ __forceinline__ void stats_add(simple_stats* st, uint32_t flags, double alpha) {
  typedef unsigned long long ull;
  atomicAdd(reinterpret_cast<ull*>(&st->rows), 1ull);
  if (flags & SIMPLE_DIAG_GREEDY) atomicAdd(reinterpret_cast<ull*>(&st->greedy_rows), 1ull);
  if ((flags & SIMPLE_DIAG_SHVS) && !(flags & SIMPLE_DIAG_ERROR)) {
    atomicAdd(reinterpret_cast<ull*>((flags & SIMPLE_DIAG_ACCEPTED) ? &st->shvs_accepted : &st->shvs_rejected), 1ull);
    atomicAdd(reinterpret_cast<ull*>(&st->sum_alpha_q32), (ull)__double2ull_rn(alpha * 4294967296.0));
  }
  if (flags & SIMPLE_DIAG_WIDE) atomicAdd(reinterpret_cast<ull*>(&st->second_pass_rows), 1ull);
  if (flags & SIMPLE_DIAG_GENERAL) atomicAdd(reinterpret_cast<ull*>(&st->general_rows), 1ull);
  if (flags & DIAG_ERROR_BITS) atomicOr(&st->error_flags, flags & DIAG_ERROR_BITS);
}

// ---------------------------------------------------------------- per-row history state -------
// The histograms of section 2.2 are never materialised over V.  A row keeps, in LDS:
//   bits  : V-bit presence mask  M_p or M_o            (which columns are penalised at all)
//   grp   : number of set bits before each group of 8 mask words (rank directory)
//   cnt   : 16-bit generated-token counts C_o, indexed by the rank of the id among the set bits
// so a column's penalty is found in O(1) from its id, and columns outside the history are never
// touched (column-wise penalties, section 5.2).
struct History {
  uint32_t* bits;
  uint32_t* grp;
  uint32_t* cnt;  // two 16-bit counters per word
  int n_words;
  int distinct;
  float rep, freq, pres;
  bool active;

  __device__ __forceinline__ bool test(int id) const { return (bits[id >> 5] >> (id & 31)) & 1u; }
  __device__ inline int rank(int id) const {
    const int w = id >> 5, g = w >> 3;
    int r = grp[g];
    for (int j = g << 3; j < w; ++j) r += __popc(bits[j]);
    return r + __popc(bits[w] & ((1u << (id & 31)) - 1u));
  }
  __device__ __forceinline__ uint32_t count_at(int r) const { return (cnt[r >> 1] >> ((r & 1) * 16)) & 0xFFFFu; }
  // Z' for a column that is in the history: repetition (sign-aware), frequency, presence; each
  // operation rounded to float32 on its own (the file is built with FP contraction off).
  __device__ __forceinline__ float penalise_inline(float z, int id) const {
    const uint32_t c = count_at(rank(id));
    z = (z > 0.0f) ? z / rep : z * rep;
    if (c > 0u) {
      const float t = freq * (float)c;
      z = z - t;
      z = z - pres;
    }
    return z;
  }
  // The same as a call: for loops that keep no loads in flight across it.
  __device__ __noinline__ float penalise(float z, int id) const { return penalise_inline(z, id); }
};

// Builds the history state of one row.  hist points at the row's ids (nnz of them, the first
// n_prompt are prompt tokens).  Returns false (all threads) if some id is outside [0, V).
__device__ __noinline__ bool build_history(History& H, const int32_t* __restrict__ hist, int nnz,
                                     int n_prompt, int V, uint32_t* scan_ws, uint32_t* flag_ws) {
  const int tid = threadIdx.x;
  const int n_grp = (H.n_words + 7) >> 3;
  for (int i = tid; i < n_grp * 8; i += NT) H.bits[i] = 0u;
  for (int i = tid; i < (nnz + 1) / 2; i += NT) H.cnt[i] = 0u;
  if (tid == 0) *flag_ws = 0u;
  __syncthreads();
  for (int i = tid; i < nnz; i += NT) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) atomicOr(&H.bits[id >> 5], 1u << (id & 31));
    else atomicOr(flag_ws, 1u);
  }
  __syncthreads();
  // rank directory: exclusive scan of per-group popcounts, NT groups at a time
  uint32_t carry = 0;
  for (int g0 = 0; g0 < n_grp; g0 += NT) {
    const int g = g0 + tid;
    uint32_t pc = 0;
    if (g < n_grp) {
#pragma unroll
      for (int j = 0; j < 8; ++j) pc += __popc(H.bits[g * 8 + j]);
    }
    uint32_t total;
    const uint32_t incl = block_incl_scan(pc, scan_ws, total);
    if (g < n_grp) H.grp[g] = carry + incl - pc;
    carry += total;
  }
  H.distinct = (int)carry;
  __syncthreads();
  n_prompt = min(max(n_prompt, 0), nnz);
  for (int i = n_prompt + tid; i < nnz; i += NT) {
    const int id = hist[i];
    if ((unsigned)id < (unsigned)V) {
      const int r = H.rank(id);
      atomicAdd(&H.cnt[r >> 1], 1u << ((r & 1) * 16));
    }
  }
  __syncthreads();
  return *flag_ws == 0u;
}

}  // namespace simple
