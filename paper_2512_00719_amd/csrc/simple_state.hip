// Incremental penalty state (paper section 5.2: row-append token buffer, C_o^{s+1} = C_o^s + Hist(Y_s)).
//
// A state holds, per sequence slot, in device memory:
//   tokens   the sequence's ids, prompt first, then one generated id per step (the paper's token
//            buffer, stored sequence-major so that one row's history is contiguous);
//   tables   what the single-pass sampling kernel otherwise builds in LDS from that list on every
//            call: the presence mask M_p or M_o (one bit per column), the 16-bit count of set bits
//            before each pair of mask words, and the 16-bit generated-token counts C_o indexed by
//            the rank of the id among the set bits, at the offsets the kernel uses in LDS;
//   record   length, prompt length, number of distinct ids, flags.
// The sampling call copies a row's tables into LDS instead of rebuilding them.  A step costs one
// update per sequence from its newest token alone: a count goes up, or, for an id not seen before, one
// bit is set, the directory entries behind it go up by one and the counts behind its rank move up one
// place.  The prompt's share (C_p, M_p) is set once, when the slot is (re)started.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_rowdev.hpp"

namespace simple {
namespace state {

using fast::FS;
using fast::Hist;
using fast::IDR;
using fast::u32x4;

constexpr int ST = 256;  // threads per sequence

struct StateArgs {
  StateRec* rec;
  int32_t* tokens;
  unsigned char* tables;
  int n_slots, lmax, V;
  uint32_t stride, off_dir, off_cnt;
};

// (Re)start of n slots: slot slots[i] gets the token list prompt_ids[prompt_ptr[i] .. prompt_ptr[i + 1])
// (none if prompt_ptr is null).  One workgroup per entry; the tables are built in LDS from the list
// (a prompt token sets its mask bit only: it counts towards repetition, not frequency or presence)
// and copied to the slot.
__global__ __launch_bounds__(ST) void state_reset_kernel(const StateArgs st, const int32_t* __restrict__ slots, int n,
                                                         const int64_t* __restrict__ prompt_ptr, const int32_t* __restrict__ prompt_ids,
                                                         const int32_t* __restrict__ n_prompt) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ FS S;
  const int tid = threadIdx.x;
  const int i = blockIdx.x;
  if (i >= n) return;
  const int slot = slots ? slots[i] : i;
  if ((unsigned)slot >= (unsigned)st.n_slots) return;
  long long p0 = 0, p1 = 0;
  if (prompt_ptr) { p0 = prompt_ptr[i]; p1 = prompt_ptr[i + 1]; }
  const long long want = p1 > p0 ? p1 - p0 : 0;
  const int len = (int)(want < (long long)st.lmax ? want : (long long)st.lmax);  // what the slot can hold
  const int32_t* src = prompt_ids + p0;
  int32_t* tok = st.tokens + (size_t)slot * (size_t)st.lmax;
  for (int j = tid; j < len; j += ST) tok[j] = src[j];
  Hist H;
  H.bm = reinterpret_cast<uint32_t*>(lds);
  H.dir = reinterpret_cast<uint16_t*>(lds + st.off_dir);
  H.cnt32 = reinterpret_cast<uint32_t*>(lds + st.off_cnt);
  H.n_words = (st.V + 31) >> 5;
  H.rep = 1.0f; H.freq = 0.0f; H.pres = 0.0f; H.inv_rep = 1.0; H.active = true;
  if (tid == 0) { S.flags = 0u; S.distinct = 0u; }
  int ids[IDR];
#pragma unroll
  for (int j = 0; j < IDR; ++j) { const int k = tid + j * ST; ids[j] = (k < len) ? src[k] : -1; }
  __syncthreads();
  unsigned own;
  // without n_prompt the whole list is the prompt (no generated token yet); with it, the ids behind
  // the first n_prompt[i] are tokens the sequence has generated elsewhere (a sequence that moves in)
  const int np = n_prompt ? min(max(n_prompt[i], 0), len) : len;
  fast::build_history<ST>(S, H, ids, src, len, np, st.V, own);
  // the whole table area of the slot (what lies behind the prompt's part must read as zero counts)
  const u32x4* from = reinterpret_cast<const u32x4*>(lds);
  u32x4* to = reinterpret_cast<u32x4*>(st.tables + (size_t)slot * st.stride);
  const unsigned used = (st.off_cnt + (unsigned)((len + 3) / 2) * 4u + 15u) / 16u;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (unsigned k = tid; k < st.stride / 16u; k += ST) to[k] = k < used ? from[k] : zero;
  if (tid == 0) {
    StateRec r;
    r.len = (int32_t)(want > 0x7FFFFFFFll ? 0x7FFFFFFFll : want);  // above the capacity: rows of the slot report a history that is too long
    r.n_prompt = np;
    r.distinct = (int32_t)S.distinct;
    r.flags = S.flags & SIMPLE_DIAG_BAD_HISTORY_ID;
    st.rec[slot] = r;
  }
}

// One step: new_ids[b] is the token generated for the sequence in slot slots[b] (or b); a negative
// id means none.  One workgroup per row; no two rows of a call may name the same slot.
__global__ __launch_bounds__(ST) void state_append_kernel(const StateArgs st, const int32_t* __restrict__ slots,
                                                          const int32_t* __restrict__ new_ids, int B) {
  extern __shared__ __align__(16) unsigned char lds[];  // staging of the counts that move up: 2 bytes per token of capacity
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  if (b >= B) return;
  const int slot = slots ? slots[b] : b;
  if ((unsigned)slot >= (unsigned)st.n_slots) return;
  const int t = new_ids[b];
  if (t < 0) return;
  StateRec r = st.rec[slot];
  if (r.len >= st.lmax) {  // full: the sequence is too long from here on
    if (tid == 0) { r.len = r.len < 0x7FFFFFFF ? r.len + 1 : r.len; st.rec[slot] = r; }
    return;
  }
  int32_t* tok = st.tokens + (size_t)slot * (size_t)st.lmax;
  unsigned char* tb = st.tables + (size_t)slot * st.stride;
  uint32_t* bm = reinterpret_cast<uint32_t*>(tb);
  uint16_t* dir = reinterpret_cast<uint16_t*>(tb + st.off_dir);
  uint16_t* cnt = reinterpret_cast<uint16_t*>(tb + st.off_cnt);
  if ((unsigned)t >= (unsigned)st.V) {  // kept in the list (the general kernel flags it too), ignored by the tables
    if (tid == 0) { tok[r.len] = t; r.len += 1; r.flags |= SIMPLE_DIAG_BAD_HISTORY_ID; st.rec[slot] = r; }
    return;
  }
  const int w = t >> 5;
  const uint32_t bit = 1u << (t & 31);
  const uint32_t word = bm[w];
  unsigned rank = (unsigned)dir[w >> 1];
  if (w & 1) rank += (unsigned)__popc(bm[w - 1]);
  rank += (unsigned)__popc(word & (bit - 1u));
  if (word & bit) {  // seen before: C_o goes up by one
    if (tid == 0) { cnt[rank] = (uint16_t)(cnt[rank] + 1u); tok[r.len] = t; r.len += 1; st.rec[slot] = r; }
    return;
  }
  // a new distinct id: the counts from its rank on move up one place, the directory entries of the
  // pairs behind its own go up by one, its bit is set and its count starts at one
  const unsigned D = (unsigned)r.distinct;
  uint16_t* stage = reinterpret_cast<uint16_t*>(lds);
  for (unsigned k = rank + tid; k < D; k += ST) stage[k - rank] = cnt[k];
  __syncthreads();
  for (unsigned k = rank + tid; k < D; k += ST) cnt[k + 1] = stage[k - rank];
  const int n_pairs = (((st.V + 31) >> 5) + 1) >> 1;
  for (int p = (w >> 1) + 1 + tid; p < n_pairs; p += ST) dir[p] = (uint16_t)(dir[p] + 1u);
  if (tid == 0) {
    cnt[rank] = 1u;
    bm[w] = word | bit;
    tok[r.len] = t;
    r.len += 1; r.distinct += 1;
    st.rec[slot] = r;
  }
}

}  // namespace state

// ------------------------------------------------------------------ launchers ------------------
hipError_t launch_state_reset(StateRec* rec, int32_t* tokens, unsigned char* tables, int n_slots, int lmax, int V, uint32_t stride,
                              uint32_t off_dir, uint32_t off_cnt, const int32_t* slots, int n, const int64_t* prompt_ptr,
                              const int32_t* prompt_ids, const int32_t* n_prompt, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const state::StateArgs a = {rec, tokens, tables, n_slots, lmax, V, stride, off_dir, off_cnt};
  hipLaunchKernelGGL(state::state_reset_kernel, dim3((unsigned)n), dim3(state::ST), stride, st, a, slots, n, prompt_ptr, prompt_ids, n_prompt);
  return hipGetLastError();
}

hipError_t launch_state_append(StateRec* rec, int32_t* tokens, unsigned char* tables, int n_slots, int lmax, int V, uint32_t stride,
                               uint32_t off_dir, uint32_t off_cnt, const int32_t* slots, const int32_t* new_ids, int B, hipStream_t st) {
  if (B <= 0) return hipSuccess;
  const state::StateArgs a = {rec, tokens, tables, n_slots, lmax, V, stride, off_dir, off_cnt};
  hipLaunchKernelGGL(state::state_append_kernel, dim3((unsigned)B), dim3(state::ST), (size_t)lmax * 2u + 16u, st, a, slots, new_ids, B);
  return hipGetLastError();
}

hipError_t set_max_lds_state(unsigned bytes) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(state::state_reset_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(state::state_append_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace simple
