// The layer stack of the coarse-expert workload: consecutive MoE layers joined by the residual stream,
// h <- h + MoE_S(x), with x = h or x = h scaled row by row to unit root-mean-square.  The scaling is the only
// arithmetic here; every layer is the fused layer call.
#include "common.h"

namespace moespec {

constexpr int kRmsThreads = 256;

// x[t] = h[t] / sqrt(mean_j h[t, j]^2) in fp32: thread i adds the squares of elements i, i + 256, ... in ascending
// order, the 256 partial sums are folded pairwise through LDS (a fixed tree), so the result does not depend on
// timing.  One workgroup per row; x may alias h (every element is read before the barrier that precedes its store).
template <typename T>
__global__ __launch_bounds__(kRmsThreads) void rms_scale_kernel(const T *__restrict__ h, int d, T *x) {
  __shared__ float part[kRmsThreads];
  const int t = blockIdx.x, tid = threadIdx.x;
  const T *row = h + (size_t)t * d;
  float ss = 0.f;
  for (int j = tid; j < d; j += kRmsThreads) {
    const float v = Elem<T>::load(row + j);
    ss = fmaf(v, v, ss);
  }
  part[tid] = ss;
  __syncthreads();
  for (int s = kRmsThreads / 2; s >= 1; s >>= 1) {
    if (tid < s) part[tid] += part[tid + s];
    __syncthreads();
  }
  const float scale = 1.0f / sqrtf(part[0] / (float)d);
  for (int j = tid; j < d; j += kRmsThreads) Elem<T>::store(x + (size_t)t * d + j, Elem<T>::load(row + j) * scale);
}

hipError_t launch_rms_scale(const moespec_desc &ds, const void *h, int M, void *x, hipStream_t st) {
  if (ds.dtype == MOESPEC_BF16)
    rms_scale_kernel<uint16_t><<<M, kRmsThreads, 0, st>>>(static_cast<const uint16_t *>(h), ds.d, static_cast<uint16_t *>(x));
  else
    rms_scale_kernel<float><<<M, kRmsThreads, 0, st>>>(static_cast<const float *>(h), ds.d, static_cast<float *>(x));
  return hipGetLastError();
}

}  // namespace moespec
