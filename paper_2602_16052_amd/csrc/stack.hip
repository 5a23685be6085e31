// The layer stack of the coarse-expert workload: consecutive MoE layers joined by the residual stream,
// h <- h + MoE_S(x), with x = h or x = h scaled row by row to unit root-mean-square.  The scaling is the only
// arithmetic here; every layer is the fused layer call.
#include "common.h"

namespace moespec {

// x[t] = h[t] / sqrt(mean_j h[t, j]^2) in fp32 (rms_scale_of_row: a fixed summation order).  One workgroup per row;
// x may alias h (every element is read before the barriers that precede its store).  d <= 8192.
template <typename T>
__global__ __launch_bounds__(kRmsThreads) void rms_scale_kernel(const T *__restrict__ h, int d, T *x) {
  __shared__ float part[kRmsThreads];
  const int t = blockIdx.x, tid = threadIdx.x;
  float v[kRmsChunks][4];
#pragma unroll
  for (int c = 0; c < kRmsChunks; ++c) {
    const int j = (c * kRmsThreads + tid) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[c][i] = j < d ? Elem<T>::load(h + (size_t)t * d + j + i) : 0.f;
  }
  const float scale = rms_scale_of_row(v, d, part);
#pragma unroll
  for (int c = 0; c < kRmsChunks; ++c) {
    const int j = (c * kRmsThreads + tid) * 4;
    if (j < d)
#pragma unroll
      for (int i = 0; i < 4; ++i) Elem<T>::store(x + (size_t)t * d + j + i, v[c][i] * scale);
  }
}

hipError_t launch_rms_scale(const moespec_desc &ds, const void *h, int M, void *x, hipStream_t st) {
  if (ds.dtype == MOESPEC_BF16)
    rms_scale_kernel<uint16_t><<<M, kRmsThreads, 0, st>>>(static_cast<const uint16_t *>(h), ds.d, static_cast<uint16_t *>(x));
  else
    rms_scale_kernel<float><<<M, kRmsThreads, 0, st>>>(static_cast<const float *>(h), ds.d, static_cast<float *>(x));
  return hipGetLastError();
}

}  // namespace moespec
