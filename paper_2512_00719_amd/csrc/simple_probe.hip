// Measurement aid: a read-only streaming reduction (row maximum) over a logits matrix, with the
// access pattern of the sampling kernel's stream (one workgroup per row, 16-byte non-temporal
// loads, tiles interleaved over the waves, next tile in flight while the current one is reduced)
// and none of its arithmetic.  Its rate is the bandwidth a one-pass row kernel can reach on the
// device, which is what the sampling kernel's achieved rate is compared with besides the
// published HBM peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_sample.h"

namespace simple {
namespace probe {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
constexpr int PT = 512;   // threads per row
constexpr int PU = 4;     // 16-byte loads in flight per lane and buffer

template <typename T> __device__ __forceinline__ float elem_max(v4u q);
template <> __device__ __forceinline__ float elem_max<float>(v4u q) {
  return fmaxf(fmaxf(__uint_as_float(q.x), __uint_as_float(q.y)), fmaxf(__uint_as_float(q.z), __uint_as_float(q.w)));
}
template <> __device__ __forceinline__ float elem_max<uint16_t>(v4u q) {
  float m = -INFINITY;
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m = fmaxf(m, __uint_as_float(w[i] << 16));
    m = fmaxf(m, __uint_as_float(w[i] & 0xFFFF0000u));
  }
  return m;
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Row b of `logits` (row_stride elements apart, rows 16-byte aligned) -> row_max[b].
template <typename T>
__global__ __launch_bounds__(PT) void row_max_kernel(const T* __restrict__ logits, int64_t V, int64_t row_stride,
                                                     float* __restrict__ row_max) {
  __shared__ float part[PT / 64];
  constexpr int EPL = 16 / (int)sizeof(T);        // elements per 16-byte load
  constexpr int64_t TILE = 64 * EPL * PU;         // elements per wave and step
  const T* row = logits + (int64_t)blockIdx.x * row_stride;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NW = PT / 64;
  const int64_t n_full = V / TILE;
  float m = -INFINITY;
  v4u cur[PU], nxt[PU];
  int64_t t = wave;
  if (t < n_full) {
#pragma unroll
    for (int u = 0; u < PU; ++u)
      cur[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(row + t * TILE + (u * 64 + lane) * EPL));
  }
  for (; t < n_full; t += NW) {
    const bool more = t + NW < n_full;
    if (more) {
#pragma unroll
      for (int u = 0; u < PU; ++u)
        nxt[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(row + (t + NW) * TILE + (u * 64 + lane) * EPL));
    }
#pragma unroll
    for (int u = 0; u < PU; ++u) m = fmaxf(m, elem_max<T>(cur[u]));
    if (more) {
#pragma unroll
      for (int u = 0; u < PU; ++u) cur[u] = nxt[u];
    }
  }
  for (int64_t c = n_full * TILE + threadIdx.x; c < V; c += PT) m = fmaxf(m, to_f<T>(row[c]));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if (lane == 0) part[wave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = part[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmaxf(r, part[w]);
    row_max[blockIdx.x] = r;
  }
}

}  // namespace probe
}  // namespace simple

extern "C" int simple_stream_probe(const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                                   float* row_max_dev, void* hip_stream) {
  using namespace simple::probe;
  if (B == 0) return SIMPLE_OK;
  if (!logits_dev || !row_max_dev || B < 0 || V <= 0 || row_stride_elems < V) return SIMPLE_EINVAL;
  if (dtype != SIMPLE_F32 && dtype != SIMPLE_BF16) return SIMPLE_EINVAL;
  if (B > 0x7FFFFFFF) return SIMPLE_ECAPACITY;
  const int64_t esize = (dtype == SIMPLE_F32) ? 4 : 2;
  if (((uintptr_t)logits_dev & 15u) != 0 || ((row_stride_elems * esize) & 15) != 0) return SIMPLE_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dtype == SIMPLE_F32)
    hipLaunchKernelGGL(row_max_kernel<float>, dim3((unsigned)B), dim3(PT), 0, st, (const float*)logits_dev, V,
                       row_stride_elems, row_max_dev);
  else
    hipLaunchKernelGGL(row_max_kernel<uint16_t>, dim3((unsigned)B), dim3(PT), 0, st, (const uint16_t*)logits_dev, V,
                       row_stride_elems, row_max_dev);
  return hipGetLastError() == hipSuccess ? SIMPLE_OK : SIMPLE_EDEVICE;
}
