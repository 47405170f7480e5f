// Logit bias and allow-lists (paper section 5.2 lists allow-lists among the constraints that compose
// on the survivor set; its implementation section mentions optional biases).  They are applied by a
// pass of their own, ahead of the sampling call: out[b, v] = allowed(b, v) ? fl32(z[b, v] + bias(b, v))
// : -inf, written as float32 to a matrix the caller owns and then samples (dtype float32).  The
// sampling kernels are untouched by it: a call that uses no constraint pays nothing, one that does
// pays one more read and one write of its logits.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "simple_sample.h"

namespace simple {
namespace constraints {

constexpr int CT = 256;

template <typename T> __device__ __forceinline__ float up(T v);
template <> __device__ __forceinline__ float up<float>(float v) { return v; }
template <> __device__ __forceinline__ float up<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// One workgroup per row.  The allow-list, if the row has one, becomes a V-bit mask in LDS; the row is
// then streamed once (mask applied, float32 written); the bias entries follow.  Entries that name
// the same column add up in list order: the thread of a column's first entry walks the rest of
// the list for it, so the float32 additions happen in the order the list gives.
template <typename T>
__global__ __launch_bounds__(CT) void constraints_kernel(const T* __restrict__ logits, int64_t V, int64_t stride,
                                                         const int64_t* __restrict__ bias_ptr, const int32_t* __restrict__ bias_ids,
                                                         const float* __restrict__ bias_vals, const int64_t* __restrict__ allow_ptr,
                                                         const int32_t* __restrict__ allow_ids, float* out, int64_t out_stride) {
  extern __shared__ __align__(16) uint32_t mask[];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const T* src = logits + row * stride;
  float* dst = out + row * out_stride;
  int64_t a0 = 0, a1 = 0, b0 = 0, b1 = 0;
  if (allow_ptr) { a0 = allow_ptr[row]; a1 = allow_ptr[row + 1]; }
  if (bias_ptr) { b0 = bias_ptr[row]; b1 = bias_ptr[row + 1]; }
  const bool masked = a1 > a0;  // a row without entries has no allow-list: every column stays
  if (masked) {
    const int n_words = (int)((V + 31) >> 5);
    for (int w = tid; w < n_words; w += CT) mask[w] = 0u;
    __syncthreads();
    for (int64_t i = a0 + tid; i < a1; i += CT) {
      const int id = allow_ids[i];
      if ((unsigned)id < (unsigned)V) atomicOr(&mask[id >> 5], 1u << (id & 31));  // an id outside the vocabulary is ignored
    }
    __syncthreads();
  }
  for (int64_t v = tid; v < V; v += CT) {
    float z = up<T>(src[v]);
    if (masked && !((mask[v >> 5] >> (v & 31)) & 1u)) z = -INFINITY;
    dst[v] = z;
  }
  __syncthreads();  // the row is written before the bias entries read it back
  for (int64_t i = b0 + tid; i < b1; i += CT) {
    const int id = bias_ids[i];
    if ((unsigned)id >= (unsigned)V) continue;
    bool first = true;
    for (int64_t j = b0; j < i; ++j) first = first && (bias_ids[j] != id);
    if (!first) continue;
    float acc = dst[id];
    for (int64_t j = i; j < b1; ++j) if (bias_ids[j] == id) acc = acc + bias_vals[j];  // one float32 rounding per entry
    dst[id] = acc;
  }
}

}  // namespace constraints
}  // namespace simple

extern "C" int simple_apply_logit_constraints(const void* logits_dev, int64_t B, int64_t V, int dtype, int64_t row_stride_elems,
                                              const int64_t* bias_ptr_dev, const int32_t* bias_ids_dev, const float* bias_vals_dev,
                                              const int64_t* allow_ptr_dev, const int32_t* allow_ids_dev,
                                              float* out_dev, int64_t out_stride_elems, void* hip_stream) {
  using namespace simple::constraints;
  if (B < 0 || V <= 0 || row_stride_elems < V || out_stride_elems < V) return SIMPLE_EINVAL;
  if (dtype != SIMPLE_F32 && dtype != SIMPLE_BF16) return SIMPLE_EINVAL;
  if ((bias_ptr_dev && (!bias_ids_dev || !bias_vals_dev)) || (allow_ptr_dev && !allow_ids_dev)) return SIMPLE_EINVAL;
  if (B == 0) return SIMPLE_OK;
  if (!logits_dev || !out_dev) return SIMPLE_EINVAL;
  if (B > (int64_t)0x7FFFFFFF) return SIMPLE_EINVAL;
  const size_t lds = allow_ptr_dev ? (size_t)((V + 31) / 32) * 4u : 0u;  // the allow-list's mask
  if (lds > (size_t)96 * 1024) return SIMPLE_ECAPACITY;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dtype == SIMPLE_F32) {
    auto k = constraints_kernel<float>;
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SIMPLE_EDEVICE;
    hipLaunchKernelGGL(k, dim3((unsigned)B), dim3(CT), lds, st, (const float*)logits_dev, V, row_stride_elems, bias_ptr_dev, bias_ids_dev,
                       bias_vals_dev, allow_ptr_dev, allow_ids_dev, out_dev, out_stride_elems);
  } else {
    auto k = constraints_kernel<uint16_t>;
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SIMPLE_EDEVICE;
    hipLaunchKernelGGL(k, dim3((unsigned)B), dim3(CT), lds, st, (const uint16_t*)logits_dev, V, row_stride_elems, bias_ptr_dev, bias_ids_dev,
                       bias_vals_dev, allow_ptr_dev, allow_ids_dev, out_dev, out_stride_elems);
  }
  return hipGetLastError() == hipSuccess ? SIMPLE_OK : SIMPLE_EDEVICE;
}
