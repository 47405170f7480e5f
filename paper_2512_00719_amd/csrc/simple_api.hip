// C boundary of the sampling library: argument checks, context, stream-ordered launches.
// No torch types; every pointer marked *_dev is a device pointer owned by the caller.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <new>

#include "simple_device.hpp"
#include "simple_kernels.hpp"
#include "simple_sample.h"

struct simple_ctx {
  int device;
  int64_t max_V, max_nnz;
  uint32_t* hot_bits;   // device, max_V bits
  uint32_t* hot_flags;  // device, one word
  int64_t hot_V;        // V the installed hot set was built for, 0 if none
  int32_t hot_H;
  bool hot_is_range;    // the installed hot set is the column range [0, hot_H) (built for the hot-first call)
  int lds_limit;
  int n_cu;
  uint32_t* pend;       // device: queue of rows the single-pass kernel leaves to the general kernel
  int32_t* order;       // device: row of each workgroup of the single-pass kernel (rows with long epilogues first)
  uint32_t* wq;         // device: queue of rows for the whole-vocabulary-nucleus kernels
  unsigned char* wws;   // device: their workspace, `slots` slots
  uint32_t ws_stride;   // bytes per slot
  int slots;            // rows per launch: every row of a launch can be queued, with a slot
  int parity;           // which queue counters the next launch uses
  hipEvent_t* prof_ev;  // 2 * PROF_MAX events while profiling is enabled, else null
  int prof_n;           // launches recorded so far
  void* base;           // device allocation that holds all of the above (null: not owned)
  simple_stats* stats;  // caller's aggregate (device), or null
  float* logprobs;      // caller's per-row outputs (device), or null
  uint8_t* eos_out;
  int32_t eos_ids[8];
  int n_eos;
};
constexpr int PROF_MAX = 1024;

struct simple_state {
  int device;
  int64_t n_slots, V, lmax;
  uint32_t stride, off_dir, off_cnt;  // bytes of tables per slot; offsets of the rank directory and the counts in them
  simple::StateRec* rec;
  int32_t* tokens;
  unsigned char* tables;
  void* base;
};

namespace simple {

// Device memory of a context, carved from one block: hot-set bitmap (max_V bits), one flag word, the
// pending-row queue (two counters, then one entry per row of a launch), the wide-row queue (a head,
// then one 64-byte record per slot) and the slots.  Every part starts on a 256-byte boundary.
struct CtxLayout { size_t hot_bits, hot_flags, pend, order, wq, wws, total; uint32_t ws_stride; };
// Maxima of simple_sample_static, whose context lives in a static device array.
constexpr int64_t STATIC_MAX_V = ((int64_t)1 << 18) - 1;
constexpr int64_t STATIC_MAX_NNZ = 8192;
constexpr int STATIC_SLOTS = 64;
constexpr size_t STATIC_BYTES = (size_t)8 << 20;

uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }

LdsLayout make_layout(int64_t V, int64_t max_nnz, bool with_history) {
  LdsLayout L{};
  uint32_t off = 0;
  const uint32_t n_words = (uint32_t)((V + 31) / 32);
  const uint32_t n_grp = (n_words + 7u) / 8u;
  L.bitmap = off; if (with_history) off = align16(off + n_grp * 8u * 4u);
  L.grp = off;    if (with_history) off = align16(off + n_grp * 4u);
  L.counts = off; if (with_history) off = align16(off + (uint32_t)((max_nnz + 2) / 2) * 4u);
  L.cand = off;   off = align16(off + (uint32_t)CAP * 8u);
  L.hist = off;   off = align16(off + (uint32_t)NBINS * 4u);
  L.total = off;
  return L;
}

// The single-pass kernel needs 16-byte aligned rows, a vocabulary whose columns fit 18 bits, 16-bit
// token counts and at least two tiles per wave.  Its row state is sized so that four workgroups of
// 256 threads share a compute unit when the history tables allow it, else 512 threads are used.  A
// batch with fewer rows than that many workgroups gets more threads per row (up to 1024: sixteen
// waves, what a compute unit holds of this kernel), so that the compute units it reaches are full.
FastLayout make_fast_layout(int64_t V, int dtype, int64_t max_nnz, bool with_history, bool vec, int lds_limit,
                            int64_t B, int n_cu) {
  FastLayout F{};
  if (!vec || V >= ((int64_t)1 << 18) || max_nnz > 65535) return F;
  const int64_t tile = 64 * 4 * ((dtype == SIMPLE_F32) ? 4 : 8);
  const uint32_t n_words = (uint32_t)((V + 31) / 32), n_pairs = (n_words + 1u) / 2u;
  uint32_t off = 0;
  F.bitmap = 0;
  if (with_history) {
    off = align16(n_pairs * 8u);
    F.dir = off; off = align16(off + n_pairs * 2u);
    F.cnt = off; off = align16(off + (uint32_t)((max_nnz + 3) / 2) * 4u);
    F.claim = off; off = align16(off + (uint32_t)((max_nnz + 31) / 32) * 4u);
  }
  const uint32_t tables = 256u * 12u + 256u * 16u;           // bucket tables of the long-list epilogue
  uint32_t body = off < 28672u ? 28672u : off;               // >= 14 KB of sorted-epilogue arrays, >= 3072-entry list
  F.long_cap = (body - tables) / 8u;
  F.samp = body;
  // the sample merge area holds SPW keys per wave
  F.threads = ((int64_t)body + 2048 <= (int64_t)lds_limit / 4) ? 256 : 512;  // four workgroups per compute unit, static LDS included
  if (B <= (int64_t)n_cu) F.threads = 1024;
  else if (B <= 2 * (int64_t)n_cu) F.threads = 512;
  while (F.threads > 256 && V / tile < 2 * (F.threads / 64)) F.threads /= 2;  // two tiles per wave
  const uint32_t total = body + align16((uint32_t)(F.threads / 64) * (uint32_t)SAMPLE_PER_WAVE * 4u);
  const uint32_t reg_cap = (uint32_t)(CAPF_PER_THREAD * F.threads);  // the epilogue moves the list to registers
  F.list_cap = body / 8u < reg_cap ? body / 8u : reg_cap;
  if ((int64_t)total + 1024 > (int64_t)lds_limit) return F;  // total stays 0
  if (V / tile < 2 * (F.threads / 64)) return F;
  F.total = total;
  return F;
}

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

CtxLayout ctx_layout(int64_t max_V, int64_t max_nnz, int slots, int lds_limit, int n_cu) {
  CtxLayout L{};
  size_t off = 0;
  L.hot_bits = off;  off = align256(off + ((size_t)((max_V + 31) / 32) + 1) * 4u);
  L.hot_flags = off; off = align256(off + 4u);
  L.pend = off;      off = align256(off + (2u + (size_t)slots) * 4u);
  L.order = off;     off = align256(off + (size_t)slots * 4u);  // the order in which the single-pass kernel takes a launch's rows
  L.wq = off;        off = align256(off + 64u + 64u * (size_t)slots);  // head, then one 64-byte record per slot
  // a slot holds the fixed part and the largest history tables the single-pass kernel can have
  const FastLayout Fm = make_fast_layout(max_V < ((int64_t)1 << 18) ? max_V : ((int64_t)1 << 18) - 1, SIMPLE_F32,
                                         max_nnz, max_nnz > 0, true, lds_limit, (int64_t)1 << 30, n_cu);
  const uint32_t tables = (max_nnz > 0 && Fm.total) ? Fm.cnt + (uint32_t)((max_nnz + 3) / 2) * 4u + 16u : 0u;
  L.ws_stride = (WIDE_SLOT_FIXED + tables + 255u) & ~255u;
  L.wws = off;       off = align256(off + (size_t)L.ws_stride * (size_t)slots);
  L.total = off;
  return L;
}

struct DeviceGuard {
  int prev = -1; bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
    if (prev == dev) prev = -1;
  }
  ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

}  // namespace simple

extern "C" {

int simple_version(void) { return 100; }

const char* simple_strerror(int code) {
  switch (code) {
    case SIMPLE_OK: return "ok";
    case SIMPLE_EINVAL: return "invalid argument";
    case SIMPLE_ENOMEM: return "device allocation failed";
    case SIMPLE_EDEVICE: return "HIP runtime call failed";
    case SIMPLE_ECAPACITY: return "size exceeds the context's capacity or the LDS of a compute unit";
    default: return "unknown error code";
  }
}

int simple_create(simple_ctx** out, int device, int64_t max_B, int64_t max_V, int64_t max_nnz_per_row) {
  if (!out) return SIMPLE_EINVAL;
  *out = nullptr;
  if (max_B <= 0 || max_V <= 0 || max_V >= (int64_t)1 << 30 || max_nnz_per_row < 0 || device < 0) return SIMPLE_EINVAL;
  if (max_nnz_per_row > 65535) return SIMPLE_ECAPACITY;  // 16-bit per-token counts
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device >= n_dev) return SIMPLE_EDEVICE;
  simple::DeviceGuard guard(device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  int lds = 0;
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) return SIMPLE_EDEVICE;
  int n_cu = 0;
  if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n_cu <= 0) return SIMPLE_EDEVICE;
  const simple::LdsLayout L = simple::make_layout(max_V, max_nnz_per_row, max_nnz_per_row > 0);
  if ((int64_t)L.total + 1024 > (int64_t)lds) return SIMPLE_ECAPACITY;
  if (simple::set_max_lds((unsigned)lds - 1024u) != hipSuccess) return SIMPLE_EDEVICE;
  if (simple::set_max_lds_fast((unsigned)lds - 1024u) != hipSuccess) return SIMPLE_EDEVICE;
  simple_ctx* c = new (std::nothrow) simple_ctx();
  if (!c) return SIMPLE_ENOMEM;
  c->device = device; c->max_V = max_V; c->max_nnz = max_nnz_per_row; c->lds_limit = lds; c->n_cu = n_cu;
  c->hot_V = 0; c->hot_H = 0; c->hot_is_range = false; c->hot_bits = nullptr; c->hot_flags = nullptr; c->pend = nullptr; c->order = nullptr; c->wq = nullptr; c->wws = nullptr; c->ws_stride = 0; c->parity = 0;
  c->prof_ev = nullptr; c->prof_n = 0; c->base = nullptr; c->slots = 0; c->stats = nullptr;
  c->logprobs = nullptr; c->eos_out = nullptr; c->n_eos = 0;
  c->slots = (int)(max_B < (int64_t)simple::WIDE_SLOTS ? max_B : (int64_t)simple::WIDE_SLOTS);
  const simple::CtxLayout CL = simple::ctx_layout(max_V, max_nnz_per_row, c->slots, lds, n_cu);
  unsigned char* base = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&base), CL.total) != hipSuccess) {
    delete c;
    return SIMPLE_ENOMEM;
  }
  c->base = base;
  c->hot_bits = reinterpret_cast<uint32_t*>(base + CL.hot_bits);
  c->hot_flags = reinterpret_cast<uint32_t*>(base + CL.hot_flags);
  c->pend = reinterpret_cast<uint32_t*>(base + CL.pend);
  c->order = reinterpret_cast<int32_t*>(base + CL.order);
  c->wq = reinterpret_cast<uint32_t*>(base + CL.wq);
  c->wws = base + CL.wws;
  c->ws_stride = CL.ws_stride;
  if (hipMemset(base, 0, CL.wws) != hipSuccess) {  // everything before the slots (a slot is cleared when a row takes it)
    (void)hipFree(base);
    delete c;
    return SIMPLE_EDEVICE;
  }
  *out = c;
  return SIMPLE_OK;
}

void simple_destroy(simple_ctx* ctx) {
  if (!ctx) return;
  {
    simple::DeviceGuard guard(ctx->device);
    if (guard.ok) {
      (void)hipDeviceSynchronize();
      if (ctx->prof_ev) (void)simple_profile_enable(ctx, 0);
      if (ctx->base) (void)hipFree(ctx->base);
    }
  }
  delete ctx;
}

int simple_set_stats(simple_ctx* ctx, simple_stats* stats_dev) {
  if (!ctx || (reinterpret_cast<uintptr_t>(stats_dev) & 7u) != 0) return SIMPLE_EINVAL;
  ctx->stats = stats_dev;
  return SIMPLE_OK;
}

int simple_set_decision_outputs(simple_ctx* ctx, float* logprobs_dev, uint8_t* eos_dev, const int32_t* eos_ids_host, int n_eos) {
  if (!ctx || n_eos < 0 || n_eos > 8 || (n_eos > 0 && !eos_ids_host)) return SIMPLE_EINVAL;
  ctx->logprobs = logprobs_dev; ctx->eos_out = eos_dev; ctx->n_eos = n_eos;
  for (int i = 0; i < 8; ++i) ctx->eos_ids[i] = i < n_eos ? eos_ids_host[i] : -1;
  return SIMPLE_OK;
}

int simple_profile_enable(simple_ctx* ctx, int on) {
  if (!ctx) return SIMPLE_EINVAL;
  simple::DeviceGuard guard(ctx->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  if (ctx->prof_ev) {
    for (int i = 0; i < 2 * PROF_MAX; ++i) if (ctx->prof_ev[i]) (void)hipEventDestroy(ctx->prof_ev[i]);
    delete[] ctx->prof_ev;
    ctx->prof_ev = nullptr;
  }
  ctx->prof_n = 0;
  if (!on) return SIMPLE_OK;
  ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * PROF_MAX]();
  if (!ctx->prof_ev) return SIMPLE_ENOMEM;
  for (int i = 0; i < 2 * PROF_MAX; ++i) {
    if (hipEventCreate(&ctx->prof_ev[i]) != hipSuccess) { (void)simple_profile_enable(ctx, 0); return SIMPLE_EDEVICE; }
  }
  return SIMPLE_OK;
}

int simple_profile_read_launches(simple_ctx* ctx, float* ms_host, int cap, double* total_ms_host) {
  if (!ctx || !total_ms_host || cap < 0 || (cap > 0 && !ms_host)) return SIMPLE_EINVAL;
  *total_ms_host = 0.0;
  if (!ctx->prof_ev) return 0;
  simple::DeviceGuard guard(ctx->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  double total = 0.0;
  for (int i = 0; i < ctx->prof_n; ++i) {
    if (hipEventSynchronize(ctx->prof_ev[2 * i + 1]) != hipSuccess) return SIMPLE_EDEVICE;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]) != hipSuccess) return SIMPLE_EDEVICE;
    if (i < cap) ms_host[i] = ms;
    total += (double)ms;
  }
  *total_ms_host = total;
  return ctx->prof_n;
}

int simple_profile_read(simple_ctx* ctx, double* total_ms_host) {
  return simple_profile_read_launches(ctx, nullptr, 0, total_ms_host);
}

int64_t simple_lds_bytes(const simple_ctx* ctx) {
  if (!ctx) return SIMPLE_EINVAL;
  return (int64_t)simple::make_layout(ctx->max_V, ctx->max_nnz, ctx->max_nnz > 0).total;
}

int simple_set_hot_set(simple_ctx* ctx, const int32_t* hot_ids_dev, int32_t H, int64_t V, void* hip_stream) {
  if (!ctx || !hot_ids_dev || H <= 0 || V <= 0 || H > V) return SIMPLE_EINVAL;
  if (V > ctx->max_V) return SIMPLE_ECAPACITY;
  simple::DeviceGuard guard(ctx->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  if (simple::launch_hot_build(hot_ids_dev, H, (int)V, ctx->hot_bits, ctx->hot_flags,
                               static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SIMPLE_EDEVICE;
  ctx->hot_V = V; ctx->hot_H = H; ctx->hot_is_range = false;
  return SIMPLE_OK;
}

}  // extern "C"

// The sampling call; the rows' histories come from the CSR arrays or, with `state`, from its slots.
static int sample_impl(simple_ctx* ctx, const simple_state* state, const int32_t* slots_dev, const simple_tail_stats* tail,
                       const void* logits_dev, int64_t B, int64_t V,
                       int dtype, int64_t row_stride_elems, const simple_row_params* params_dev,
                       const int64_t* hist_ptr_dev, const int32_t* hist_ids_dev,
                       const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step,
                       uint64_t row_offset, int32_t* out_ids_dev, simple_row_diag* diag_dev,
                       void* hip_stream) {
  if (!ctx || B < 0 || V <= 0) return SIMPLE_EINVAL;
  if (state && (state->V != V || state->device != ctx->device || hist_ptr_dev || hist_ids_dev)) return SIMPLE_EINVAL;
  if (state && (state->lmax > ctx->max_nnz || (!slots_dev && B > state->n_slots))) return SIMPLE_ECAPACITY;
  if (dtype != SIMPLE_F32 && dtype != SIMPLE_BF16) return SIMPLE_EINVAL;
  if (row_stride_elems < V) return SIMPLE_EINVAL;
  if (H < -1 || (int64_t)H > V) return SIMPLE_EINVAL;
  if (hot_ids_dev && H <= 0) return SIMPLE_EINVAL;
  if (!hot_ids_dev && H > 0 && !tail) return SIMPLE_EINVAL;
  if (H == -1 && ctx->hot_V != V) return SIMPLE_EINVAL;
  if (hist_ptr_dev && !hist_ids_dev) return SIMPLE_EINVAL;
  if (B == 0) return SIMPLE_OK;
  if (!logits_dev || !params_dev || !out_ids_dev) return SIMPLE_EINVAL;
  if (B > (int64_t)0x7FFFFFFF) return SIMPLE_EINVAL;
  if (V > ctx->max_V) return SIMPLE_ECAPACITY;
  if (hist_ptr_dev && ctx->max_nnz == 0) return SIMPLE_ECAPACITY;
  simple::DeviceGuard guard(ctx->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const bool use_hot = (H != 0);
  const size_t esz0 = (dtype == SIMPLE_F32) ? 4 : 2;
  if (tail) {  // the hot-first call: the hot set is the column range [0, H)
    const int tile = simple::hot_first_tile(dtype);
    const bool aligned = ((reinterpret_cast<uintptr_t>(logits_dev) & 15u) == 0) && (((size_t)row_stride_elems * esz0) % 16 == 0);
    if (H <= 0 || H % tile != 0 || !aligned || hot_ids_dev || state || hist_ptr_dev) return SIMPLE_EINVAL;
    if ((int64_t)H / tile > simple::hot_first_max_tiles() || (V - H + tile - 1) / tile > simple::hot_first_max_tiles()) return SIMPLE_ECAPACITY;
    if (ctx->hot_V != V || ctx->hot_H != H || !ctx->hot_is_range) {
      if (simple::launch_hot_range(ctx->hot_bits, ctx->hot_flags, (int)V, (int)H, st) != hipSuccess) return SIMPLE_EDEVICE;
      ctx->hot_V = V; ctx->hot_H = H; ctx->hot_is_range = true;
    }
  }
  if (hot_ids_dev) {
    if (simple::launch_hot_build(hot_ids_dev, H, (int)V, ctx->hot_bits, ctx->hot_flags, st) != hipSuccess)
      return SIMPLE_EDEVICE;
    ctx->hot_V = V; ctx->hot_H = H; ctx->hot_is_range = false;
  }
  const size_t esz = (dtype == SIMPLE_F32) ? 4 : 2;
  const bool vec = ((reinterpret_cast<uintptr_t>(logits_dev) & 15u) == 0) && (((size_t)row_stride_elems * esz) % 16 == 0);
  simple::SampleArgs a{};
  a.logits = logits_dev; a.stride = row_stride_elems; a.V = (int)V;
  a.params = params_dev; a.hist_ptr = hist_ptr_dev; a.hist_ids = hist_ids_dev;
  const bool with_hist = hist_ptr_dev != nullptr || state != nullptr;
  if (state) {
    a.st_rec = state->rec; a.st_tokens = state->tokens; a.st_tables = state->tables;
    a.st_lmax = (int)state->lmax; a.st_nslots = (int)state->n_slots; a.st_stride = state->stride;
  }
  a.hot_bits = use_hot ? ctx->hot_bits : nullptr;
  a.hot_flags = use_hot ? ctx->hot_flags : nullptr;
  a.seed = seed; a.step = step;
  a.stats = ctx->stats;
  a.n_eos = ctx->n_eos;
  for (int i = 0; i < 8; ++i) a.eos_ids[i] = ctx->eos_ids[i];
  a.max_nnz = (int)ctx->max_nnz;
  a.pend = ctx->pend;
  a.order = ctx->order;
  a.n_cu = ctx->n_cu;
  a.wq = ctx->wq; a.wws = ctx->wws; a.wide_slots = ctx->slots; a.ws_stride = ctx->ws_stride;
  a.L = simple::make_layout(V, ctx->max_nnz, with_hist);
  // rows go out in launches that neither queue can overflow
  const int64_t per_launch = ctx->slots;
  a.F = simple::make_fast_layout(V, dtype, with_hist ? ctx->max_nnz : 0, with_hist, vec, ctx->lds_limit,
                                 B < per_launch ? B : per_launch, ctx->n_cu);
  a.gated = (a.F.total != 0u || tail) ? 1 : 0;
  a.pattern_on = (dtype == SIMPLE_BF16 && V < ((int64_t)1 << 18)) ? (tail ? 2 : (a.F.total != 0u ? 1 : 0)) : 0;
  for (int64_t b0 = 0; b0 < B; b0 += per_launch) {
    const int64_t nb = (B - b0 < per_launch) ? (B - b0) : per_launch;
    a.B = (int)nb;
    a.logits = static_cast<const char*>(logits_dev) + (size_t)b0 * (size_t)row_stride_elems * esz;
    a.params = params_dev + b0;
    a.hist_ptr = hist_ptr_dev ? hist_ptr_dev + b0 : nullptr;
    a.st_slots = slots_dev ? slots_dev + b0 : nullptr;
    a.st_slot0 = (int)b0;
    a.row_offset = row_offset + (uint64_t)b0;
    a.out = out_ids_dev + b0;
    a.diag = diag_dev ? diag_dev + b0 : nullptr;
    a.logprobs = ctx->logprobs ? ctx->logprobs + b0 : nullptr;
    a.eos_out = ctx->eos_out ? ctx->eos_out + b0 : nullptr;
    a.order = (a.F.total != 0u && !tail && nb > (int64_t)ctx->n_cu) ? ctx->order : nullptr;
    a.parity = ctx->parity;
    if (a.gated) ctx->parity ^= 1;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (ctx->prof_ev && ctx->prof_n < PROF_MAX) { ev0 = ctx->prof_ev[2 * ctx->prof_n]; ev1 = ctx->prof_ev[2 * ctx->prof_n + 1]; ++ctx->prof_n; }
    if (tail) {  // the hot-first kernel, then the general kernel on the rows it left
      if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return SIMPLE_EDEVICE;
      if (a.pattern_on && simple::launch_pattern(a, st) != hipSuccess) return SIMPLE_EDEVICE;  // truncated bfloat16 rows
      if (simple::launch_hot_first(a, dtype, (int)H, tail + b0, st) != hipSuccess) return SIMPLE_EDEVICE;
      if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return SIMPLE_EDEVICE;
      if (simple::launch_pending_rows(a, dtype, vec, st) != hipSuccess) return SIMPLE_EDEVICE;
      continue;
    }
    if (simple::launch_sample(a, dtype, vec, st, ev0, ev1) != hipSuccess) return SIMPLE_EDEVICE;
  }
  return SIMPLE_OK;
}

extern "C" {

int simple_sample(simple_ctx* ctx, const void* logits_dev, int64_t B, int64_t V, int dtype,
                  int64_t row_stride_elems, const simple_row_params* params_dev,
                  const int64_t* hist_ptr_dev, const int32_t* hist_ids_dev,
                  const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step,
                  uint64_t row_offset, int32_t* out_ids_dev, simple_row_diag* diag_dev,
                  void* hip_stream) {
  return sample_impl(ctx, nullptr, nullptr, nullptr, logits_dev, B, V, dtype, row_stride_elems, params_dev, hist_ptr_dev, hist_ids_dev,
                     hot_ids_dev, H, seed, step, row_offset, out_ids_dev, diag_dev, hip_stream);
}

// ---- incremental penalty state (section 5.2) ------------------------------------------------------
int simple_state_create(simple_state** out, int device, int64_t max_seqs, int64_t V, int64_t L_max) {
  if (!out) return SIMPLE_EINVAL;
  *out = nullptr;
  if (device < 0 || max_seqs <= 0 || max_seqs > (int64_t)0x7FFFFFFF || V <= 0 || V >= (int64_t)1 << 30 || L_max <= 0) return SIMPLE_EINVAL;
  if (L_max > 65535) return SIMPLE_ECAPACITY;  // 16-bit per-token counts
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device >= n_dev) return SIMPLE_EDEVICE;
  simple::DeviceGuard guard(device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  int lds = 0;
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) return SIMPLE_EDEVICE;
  simple_state* s = new (std::nothrow) simple_state();
  if (!s) return SIMPLE_ENOMEM;
  s->device = device; s->n_slots = max_seqs; s->V = V; s->lmax = L_max;
  // the tables of a slot lie as the single-pass kernel lays them out in LDS (make_fast_layout)
  const uint32_t n_words = (uint32_t)((V + 31) / 32), n_pairs = (n_words + 1u) / 2u;
  s->off_dir = simple::align16(n_pairs * 8u);
  s->off_cnt = simple::align16(s->off_dir + n_pairs * 2u);
  s->stride = (s->off_cnt + (uint32_t)((L_max + 3) / 2) * 4u + 16u + 255u) & ~255u;
  if ((int64_t)s->stride + 2048 > (int64_t)lds) { delete s; return SIMPLE_ECAPACITY; }  // the restart kernel builds a slot's tables in LDS
  if (simple::set_max_lds_state((unsigned)lds - 1024u) != hipSuccess) { delete s; return SIMPLE_EDEVICE; }
  const size_t rec_b = simple::align256(sizeof(simple::StateRec) * (size_t)max_seqs);
  const size_t tok_b = simple::align256(4u * (size_t)L_max * (size_t)max_seqs);
  const size_t tab_b = (size_t)s->stride * (size_t)max_seqs;
  unsigned char* base = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&base), rec_b + tok_b + tab_b) != hipSuccess) { delete s; return SIMPLE_ENOMEM; }
  if (hipMemset(base, 0, rec_b + tok_b + tab_b) != hipSuccess) { (void)hipFree(base); delete s; return SIMPLE_EDEVICE; }  // every slot: an empty sequence
  s->base = base;
  s->rec = reinterpret_cast<simple::StateRec*>(base);
  s->tokens = reinterpret_cast<int32_t*>(base + rec_b);
  s->tables = base + rec_b + tok_b;
  *out = s;
  return SIMPLE_OK;
}

void simple_state_destroy(simple_state* state) {
  if (!state) return;
  {
    simple::DeviceGuard guard(state->device);
    if (guard.ok) {
      (void)hipDeviceSynchronize();
      if (state->base) (void)hipFree(state->base);
    }
  }
  delete state;
}

int simple_state_restart(simple_state* state, const int32_t* slots_dev, int64_t n, const int64_t* prompt_ptr_dev,
                         const int32_t* prompt_ids_dev, const int32_t* n_prompt_dev, void* hip_stream) {
  if (!state || n < 0 || n > state->n_slots || (prompt_ptr_dev && !prompt_ids_dev)) return SIMPLE_EINVAL;
  if (n == 0) return SIMPLE_OK;
  simple::DeviceGuard guard(state->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  if (simple::launch_state_reset(state->rec, state->tokens, state->tables, (int)state->n_slots, (int)state->lmax, (int)state->V, state->stride,
                                 state->off_dir, state->off_cnt, slots_dev, (int)n, prompt_ptr_dev, prompt_ids_dev, n_prompt_dev,
                                 static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SIMPLE_EDEVICE;
  return SIMPLE_OK;
}

int simple_state_append(simple_state* state, const int32_t* slots_dev, const int32_t* new_ids_dev, int64_t B, void* hip_stream) {
  if (!state || B < 0 || (B > 0 && !new_ids_dev) || (!slots_dev && B > state->n_slots) || B > (int64_t)0x7FFFFFFF) return SIMPLE_EINVAL;
  if (B == 0) return SIMPLE_OK;
  simple::DeviceGuard guard(state->device);
  if (!guard.ok) return SIMPLE_EDEVICE;
  if (simple::launch_state_append(state->rec, state->tokens, state->tables, (int)state->n_slots, (int)state->lmax, (int)state->V, state->stride,
                                  state->off_dir, state->off_cnt, slots_dev, new_ids_dev, (int)B,
                                  static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SIMPLE_EDEVICE;
  return SIMPLE_OK;
}

int simple_sample_hot_first(simple_ctx* ctx, const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                            const simple_row_params* params_dev, int32_t H, const simple_tail_stats* tail_stats_dev,
                            uint64_t seed, uint64_t step, uint64_t row_offset, int32_t* out_ids_dev,
                            simple_row_diag* diag_dev, void* hip_stream) {
  if (!tail_stats_dev || H <= 0) return SIMPLE_EINVAL;
  return sample_impl(ctx, nullptr, nullptr, tail_stats_dev, logits_dev, B, V, dtype, row_stride_elems, params_dev, nullptr, nullptr,
                     nullptr, H, seed, step, row_offset, out_ids_dev, diag_dev, hip_stream);
}

int simple_sample_state(simple_ctx* ctx, const simple_state* state, const int32_t* slots_dev, const void* logits_dev, int64_t B, int64_t V,
                        int dtype, int64_t row_stride_elems, const simple_row_params* params_dev,
                        const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step, uint64_t row_offset,
                        int32_t* out_ids_dev, simple_row_diag* diag_dev, void* hip_stream) {
  if (!state) return SIMPLE_EINVAL;
  return sample_impl(ctx, state, slots_dev, nullptr, logits_dev, B, V, dtype, row_stride_elems, params_dev, nullptr, nullptr,
                     hot_ids_dev, H, seed, step, row_offset, out_ids_dev, diag_dev, hip_stream);
}

// ---- the entry point that allocates nothing -----------------------------------------------------
// Its context memory is a static device array.  `scratch` is a host-side stand-in for the symbol: the
// device address is taken once per device with hipGetSymbolAddress and used from then on.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[simple::STATIC_BYTES];

namespace simple {
constexpr int STATIC_MAX_DEVICES = 64;
static simple_ctx g_static_ctx[STATIC_MAX_DEVICES];
static bool g_static_ready[STATIC_MAX_DEVICES];

// The static context of the current device, set up at the first call on it; null with *err set on failure.
static simple_ctx* static_ctx(int* err) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0) { *err = SIMPLE_EDEVICE; return nullptr; }
  if (device >= STATIC_MAX_DEVICES) { *err = SIMPLE_ECAPACITY; return nullptr; }
  simple_ctx* c = &g_static_ctx[device];
  if (g_static_ready[device]) return c;
  int lds = 0, n_cu = 0;
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n_cu <= 0) { *err = SIMPLE_EDEVICE; return nullptr; }
  if (set_max_lds((unsigned)lds - 1024u) != hipSuccess || set_max_lds_fast((unsigned)lds - 1024u) != hipSuccess) { *err = SIMPLE_EDEVICE; return nullptr; }
  const CtxLayout L = ctx_layout(STATIC_MAX_V, STATIC_MAX_NNZ, STATIC_SLOTS, lds, n_cu);
  if (L.total > STATIC_BYTES) { *err = SIMPLE_ECAPACITY; return nullptr; }
  unsigned char* ptr = nullptr;  // this device's copy of the array
  if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { *err = SIMPLE_EDEVICE; return nullptr; }
  *c = simple_ctx();
  c->device = device; c->max_V = STATIC_MAX_V; c->max_nnz = STATIC_MAX_NNZ; c->lds_limit = lds; c->n_cu = n_cu;
  c->hot_bits = reinterpret_cast<uint32_t*>(ptr + L.hot_bits);
  c->hot_flags = reinterpret_cast<uint32_t*>(ptr + L.hot_flags);
  c->pend = reinterpret_cast<uint32_t*>(ptr + L.pend);
  c->order = reinterpret_cast<int32_t*>(ptr + L.order);
  c->wq = reinterpret_cast<uint32_t*>(ptr + L.wq);
  c->wws = ptr + L.wws;
  c->ws_stride = L.ws_stride;
  c->slots = STATIC_SLOTS;
  // The array is zero when the code object is loaded, which is what the queue counters need at the
  // first launch; afterwards every launch clears the pair of counters the previous one used, the
  // hot-set bitmap is rebuilt by the call that passes a hot set, and a slot is cleared by the row
  // that takes it.
  g_static_ready[device] = true;
  return c;
}
}  // namespace simple

extern "C" {

int simple_sample_static(const void* logits_dev, int64_t B, int64_t V, int dtype,
                         int64_t row_stride_elems, const simple_row_params* params_dev,
                         const int64_t* hist_ptr_dev, const int32_t* hist_ids_dev,
                         const int32_t* hot_ids_dev, int32_t H, uint64_t seed, uint64_t step,
                         uint64_t row_offset, int32_t* out_ids_dev, simple_row_diag* diag_dev,
                         void* hip_stream) {
  if (H == -1) return SIMPLE_EINVAL;  // no installed hot set here: pass the ids with the call
  if (V > simple::STATIC_MAX_V) return SIMPLE_ECAPACITY;
  int err = SIMPLE_OK;
  simple_ctx* c = simple::static_ctx(&err);
  if (!c) return err;
  return simple_sample(c, logits_dev, B, V, dtype, row_stride_elems, params_dev, hist_ptr_dev, hist_ids_dev,
                       hot_ids_dev, H, seed, step, row_offset, out_ids_dev, diag_dev, hip_stream);
}

int64_t simple_static_limit(int what) {
  switch (what) {
    case 0: return simple::STATIC_MAX_V;
    case 1: return simple::STATIC_MAX_NNZ;
    case 2: return (int64_t)simple::STATIC_SLOTS;
    case 3: return (int64_t)simple::STATIC_BYTES;
    default: return SIMPLE_EINVAL;
  }
}

}  // extern "C"
