// Host-visible launch interface of the sampling kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_sample.h"

namespace simple {

// Byte offsets of one row's LDS regions (dynamic shared memory of the row workgroup).
struct LdsLayout {
  uint32_t bitmap;  // history presence mask, V bits rounded up to groups of 8 words
  uint32_t grp;     // rank directory, one word per group
  uint32_t counts;  // 16-bit generated-token counts by rank
  uint32_t cand;    // candidate list: CAP keys then CAP ids (32 KB); reused by the multi-pass route
  uint32_t hist;    // radix histogram / staging (8 KB)
  uint32_t total;
};

struct SampleArgs {
  const void* logits;
  int64_t stride;  // elements between rows
  int V, B;
  const simple_row_params* params;
  const int64_t* hist_ptr;
  const int32_t* hist_ids;
  const uint32_t* hot_bits;   // V-bit hot-set mask or nullptr
  const uint32_t* hot_flags;  // bit 0: id out of range, bit 1: duplicate
  uint64_t seed, step, row_offset;
  int32_t* out;
  simple_row_diag* diag;
  int max_nnz;
  LdsLayout L;
};

LdsLayout make_layout(int64_t V, int64_t max_nnz, bool with_history);
hipError_t launch_sample(const SampleArgs& a, int dtype, bool vec, hipStream_t st);
hipError_t set_max_lds(unsigned bytes);
hipError_t launch_hot_build(const int32_t* ids, int H, int V, uint32_t* bits, uint32_t* flags, hipStream_t st);

}  // namespace simple
