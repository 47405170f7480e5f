// Speculative hot-vocab sampling that reads only the hot columns on acceptance (paper section 5.3).
//
// The paper's samplers draw on a small hot set and fall back to the tail only on rejection, with the
// weights w = exp(z' - max) "pre-computed on GPUs when writing logits".  On a GPU the row mass is the
// obstacle: alpha_b = S_H / (S_H + S_T) needs the tail's mass S_T, and summing the tail means
// reading it.  This kernel takes S_T from the producer of the logits instead: the vocabulary is laid
// out hot-first (the hot set is the columns [0, H)), and every row comes with the maximum of its
// tail logits and the sum of exp((z - tail_max) / tau) over the tail.  A row whose draw is accepted
// then costs H columns; only a rejected row streams its V - H tail columns (the cost model of
// section 5.4: c H + c0 on acceptance, the rest of the vocabulary on rejection).
//
// Rows the kernel takes itself: temperature > 0 and no truncation (no top-k, top-p, min-p) — with a
// survivor set that is all of V, Eq. (7) needs nothing of the tail but its mass.  (A truncated
// row's survivor set may reach into the tail, and which tail columns survive cannot be told from a
// maximum and a sum.)  Every other row is served with the hot set [0, H) as a membership mask: in
// a bfloat16 call the pattern-count kernel, which runs ahead of this one, completes the truncated
// rows without penalties; the rest is queued for the general kernel.  So each row of the call gets
// the ids of the speculative sampler as the definition over the whole row gives them.
//
// One workgroup per row.  Masses are 2^44 fixed-point integers relative to the row maximum (the
// stable softmax numerator of Eq. (2)), so sums do not depend on the order of the additions; the
// inverse CDF runs in ascending token id: per tile of 256 x 16 bytes a sum, the tile that holds the
// target, the thread in it, the column in the thread's group.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "simple_rowdev.hpp"

namespace simple {
namespace hotfirst {

using fast::FS;
using fast::Io;
using fast::u64;

constexpr int HT = 256;
constexpr int HWV = HT / 64;
constexpr int MAX_TILES = 1024;  // tiles of a row's tail (V below 2^20 with float32, 2^21 with bfloat16)

__device__ __forceinline__ u64 wfix_y(float y, float y_max) {  // exp(y - y_max) * 2^44, float32 exponential with a split log2(e)
  const float d = y - y_max;
  const float t = fmaf(d, fast::L2E_HI, d * fast::L2E_LO);
  return fast::float_to_u64(__builtin_amdgcn_exp2f(t) * 0x1p44f);
}

// Sums of the masses of columns [c0, c1) by tile (tile i covers columns c0 + i * TILE ...), into
// tsum[]; returns (all threads) their total.  bad is raised for a NaN or +inf tempered value.
template <typename DT>
__device__ inline u64 tile_masses(const DT* rowp, int c0, int c1, double inv_tau, float y_max, u64* tsum, FS& S, bool& bad) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int TILE = HT * EPL;
  const int tid = threadIdx.x, lane = tid & 63;
  const int n_tiles = (c1 - c0 + TILE - 1) / TILE;
  for (int i = tid; i < n_tiles; i += HT) tsum[i] = 0ull;
  __syncthreads();
  u64 total = 0ull;
  for (int i = 0; i < n_tiles; ++i) {
    const int idx0 = c0 + i * TILE + tid * EPL;
    u64 m = 0ull;
    if (idx0 + EPL <= c1) {
      float z[EPL];
      Io<DT>::unpack(Io<DT>::load(rowp + idx0), z);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float y = (float)((double)z[e] * inv_tau);
        bad = bad || (y != y) || y == INFINITY;
        m += wfix_y(y, y_max);
      }
    } else {
      for (int idx = idx0; idx < c1; ++idx) {
        const float y = (float)((double)Io<DT>::one(rowp + idx) * inv_tau);
        bad = bad || (y != y) || y == INFINITY;
        m += wfix_y(y, y_max);
      }
    }
    const u64 w = wave_sum(m);
    if (lane == 0 && w) atomicAdd(&tsum[i], w);
    total += m;
  }
  return fast::blk_sum_u64<HWV>(S, total);  // barriers inside: the tile sums are complete after it
}

// The column of [c0, c1) at which the running mass (ascending id) first exceeds tfix; its mass in w_out.
template <typename DT>
__device__ inline int locate(const DT* rowp, int c0, int c1, double inv_tau, float y_max, const u64* tsum, u64 tfix, FS& S, u64& w_out) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int TILE = HT * EPL;
  const int tid = threadIdx.x;
  const int n_tiles = (c1 - c0 + TILE - 1) / TILE;
  if (tid == 0) { S.bd = -1; S.out_id = -1; S.out_w = 0ull; }
  __syncthreads();
  // the tile: an exclusive scan over the tile sums, HT tiles per round
  u64 carry = 0ull;
  for (int t0 = 0; t0 < n_tiles; t0 += HT) {
    const u64 m = (t0 + tid < n_tiles) ? tsum[t0 + tid] : 0ull;
    unsigned ce, ct; u64 me, mt;
    fast::blk_excl_scan2<HWV>(S, 0u, m, ce, me, ct, mt);
    if (m > 0ull && carry + me <= tfix && carry + me + m > tfix) { S.bd = t0 + tid; S.mab_d = carry + me; }
    carry += mt;
    __syncthreads();
  }
  const int tile = S.bd;
  if (tile < 0) return -1;
  const int idx0 = c0 + tile * TILE + tid * EPL;
  u64 w[EPL], sum = 0ull;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    w[e] = 0ull;
    if (idx0 + e < c1) w[e] = wfix_y((float)((double)Io<DT>::one(rowp + idx0 + e) * inv_tau), y_max);
    sum += w[e];
  }
  unsigned ce, ct; u64 me, mt;
  fast::blk_excl_scan2<HWV>(S, 0u, sum, ce, me, ct, mt);
  u64 run = S.mab_d + me;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    if (w[e] > 0ull && run <= tfix && run + w[e] > tfix) { S.out_id = idx0 + e; S.out_w = w[e]; }
    run += w[e];
  }
  __syncthreads();
  w_out = S.out_w;
  return S.out_id;
}

template <typename DT>
__global__ __launch_bounds__(HT) void hot_first_rows_kernel(const SampleArgs a, int H, const simple_tail_stats* __restrict__ tail) {
  constexpr int EPL = Io<DT>::EPL;
  constexpr int TILE = HT * EPL;
  __shared__ FS S;
  __shared__ u64 tsum[MAX_TILES];
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const int V = a.V;
  const DT* rowp = reinterpret_cast<const DT*>(a.logits) + (size_t)row * (size_t)a.stride;
  const simple_row_params par = a.params[row];
  const simple_tail_stats ts = tail[row];
  if (row == 0 && tid == 0) { a.pend[a.parity ^ 1] = 0u; a.wq[a.parity ^ 1] = 0u; }  // the previous launch's counts
  // the pattern-count kernel, when it ran before this one, has left NOT_TAKEN on every row that is still to do
  if (a.pattern_on && a.out[row] != NOT_TAKEN) return;
  const bool plain = hot_first_plain(par, V);
  if (!plain) {  // truncated, penalised, greedy or invalid rows: the general kernel, with [0, H) as the hot set
    if (tid == 0) { const unsigned slot = atomicAdd(&a.pend[a.parity], 1u); a.pend[2 + slot] = (uint32_t)row; a.out[row] = PENDING; }
    return;
  }
  const double inv_tau = 1.0 / (double)par.temperature;
  double u[3];
  row_uniforms(a.seed, a.row_offset + (uint64_t)row, a.step, u);
  // ---- maximum of the hot columns, then of the row ----
  uint32_t kmax = KEY_NEG_INF;
  bool bad = false;
  for (int idx0 = tid * EPL; idx0 < H; idx0 += TILE) {  // H is a whole number of tiles
    float z[EPL];
    Io<DT>::unpack(Io<DT>::load(rowp + idx0), z);
#pragma unroll
    for (int e = 0; e < EPL; ++e) { bad = bad || (z[e] != z[e]); kmax = max(kmax, fkey(z[e])); }
  }
  kmax = fast::wave_max_u32(kmax);
  if (tid == 0) { S.kmax = KEY_NEG_INF; S.flags = 0u; }
  __syncthreads();
  if ((tid & 63) == 0) atomicMax(&S.kmax, kmax);
  __syncthreads();
  const bool has_tail = H < V;
  const float z_hot = keyf(S.kmax);
  const float z_top = has_tail ? fmaxf(z_hot, ts.tail_max) : z_hot;      // tempering is monotone: the maximum is taken on z
  const float y_max = (float)((double)z_top * inv_tau);
  const float y_tmax = (float)((double)ts.tail_max * inv_tau);
  if (has_tail && (ts.tail_max != ts.tail_max || ts.tail_max == INFINITY || !(ts.tail_sum >= 0.0) || ts.tail_sum == (double)INFINITY)) bad = true;
  if (y_max == INFINITY || z_top == -INFINITY) bad = true;               // overflow of z / tau, or nothing to draw
  // ---- hot mass by tile, tail mass from the caller's statistics (Eq. (7)) ----
  const u64 S_H = tile_masses<DT>(rowp, 0, H, inv_tau, y_max, tsum, S, bad);
  if (bad) atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
  __syncthreads();
  simple_row_diag dg;
  dg.alpha = __longlong_as_double(0x7FF8000000000000ll);
  dg.s_k = 0.0; dg.p_chosen = 0.0f; dg.n_survivors = V; dg.flags = SIMPLE_DIAG_SHVS; dg.reserved = 0u;
  int id = -1;
  u64 w_id = 0ull, S_K = 0ull;
  if (!(S.flags & SIMPLE_DIAG_ERROR)) {
    u64 S_T = 0ull;
    if (has_tail && ts.tail_sum > 0.0) S_T = (u64)__double2ull_rn(ts.tail_sum * exp((double)y_tmax - (double)y_max) * fast::WSCALE);
    S_K = S_H + S_T;
    const bool pick_hot = (S_H > 0ull) && (u[1] * (double)S_K <= (double)S_H);   // accept iff u <= alpha_b (Eq. (8))
    dg.alpha = S_K ? (double)S_H / (double)S_K : 0.0;
    if (pick_hot) {
      dg.flags |= SIMPLE_DIAG_ACCEPTED;
      u64 tfix = (u64)__double2ull_rd(u[0] * (double)S_H);
      if (tfix >= S_H) tfix = S_H - 1ull;
      id = locate<DT>(rowp, 0, H, inv_tau, y_max, tsum, tfix, S, w_id);
    } else {
      // rejected: the tail proposal r of Eq. (8), over the columns the kernel has not read yet
      bool bad_t = false;
      const u64 S_T_exact = tile_masses<DT>(rowp, H, V, inv_tau, y_max, tsum, S, bad_t);
      if (bad_t) atomicOr(&S.flags, SIMPLE_DIAG_ERROR | SIMPLE_DIAG_BAD_LOGIT);
      __syncthreads();
      if (!(S.flags & SIMPLE_DIAG_ERROR) && S_T_exact > 0ull) {
        u64 tfix = (u64)__double2ull_rd(u[2] * (double)S_T_exact);
        if (tfix >= S_T_exact) tfix = S_T_exact - 1ull;
        id = locate<DT>(rowp, H, V, inv_tau, y_max, tsum, tfix, S, w_id);
        S_K = S_H + S_T_exact;  // p~ of the drawn id over the masses as summed here
      }
    }
  }
  const bool err = (S.flags & SIMPLE_DIAG_ERROR) != 0u;
  if (!err && id < 0) {  // nothing could be located (a class without mass): the general kernel decides
    if (tid == 0) { const unsigned slot = atomicAdd(&a.pend[a.parity], 1u); a.pend[2 + slot] = (uint32_t)row; a.out[row] = PENDING; }
    return;
  }
  if (tid == 0) {
    dg.flags |= S.flags;
    if (a.hot_flags && *a.hot_flags) dg.flags |= SIMPLE_DIAG_BAD_HOT_SET;
    dg.p_chosen = err ? 0.0f : (float)((double)w_id / (double)S_K);
    if (err) dg.n_survivors = 0;
    a.out[row] = err ? -1 : id;
    if (a.diag) a.diag[row] = dg;
    if (a.stats) stats_add(a.stats, dg.flags, dg.alpha);
    write_decision(a, row, err ? -1 : id, dg.p_chosen, false);
  }
}

// The membership mask of the hot set [0, H): V bits.
__global__ void hot_range_kernel(uint32_t* bits, int n_words, int H, uint32_t* flags) {
  const int w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w < n_words) {
    const int lo = w << 5;
    bits[w] = lo + 32 <= H ? 0xFFFFFFFFu : (lo >= H ? 0u : ((1u << (H - lo)) - 1u));
  }
  if (w == 0) *flags = 0u;
}

}  // namespace hotfirst

hipError_t launch_hot_range(uint32_t* bits, uint32_t* flags, int V, int H, hipStream_t st) {
  const int n_words = (V + 31) >> 5;
  hipLaunchKernelGGL(hotfirst::hot_range_kernel, dim3((n_words + 255) / 256), dim3(256), 0, st, bits, n_words, H, flags);
  return hipGetLastError();
}

hipError_t launch_hot_first(const SampleArgs& a, int dtype, int H, const simple_tail_stats* tail, hipStream_t st) {
  const dim3 grid((unsigned)a.B);
  if (dtype == SIMPLE_F32) hipLaunchKernelGGL((hotfirst::hot_first_rows_kernel<float>), grid, dim3(hotfirst::HT), 0, st, a, H, tail);
  else hipLaunchKernelGGL((hotfirst::hot_first_rows_kernel<uint16_t>), grid, dim3(hotfirst::HT), 0, st, a, H, tail);
  return hipGetLastError();
}

int hot_first_tile(int dtype) { return hotfirst::HT * (dtype == SIMPLE_F32 ? 4 : 8); }
int hot_first_max_tiles() { return hotfirst::MAX_TILES; }

}  // namespace simple
