// Stage 1 of Algorithm 1: router projection, softmax over all N experts (Eq. (1)), per-token
// top-k and mixing weights (Section 2.1).  One workgroup per tree token; every decision in fp64.
#include "common.h"

namespace moespec {

constexpr int kRouteThreads = 512;

template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const T *__restrict__ h, const T *__restrict__ w_r,
                                                              const float *__restrict__ b_r, int d, int N, int k,
                                                              int renorm, double *__restrict__ probs,
                                                              int32_t *__restrict__ topk_ids,
                                                              float *__restrict__ topk_w) {
  extern __shared__ __align__(16) unsigned char smem[];
  double *g = reinterpret_cast<double *>(smem);              // [N rounded up to even] logits, then probabilities
  double *red = g + ((N + 1) & ~1);                                       // [8] per-wave partials
  double *wsel = red + 8;                                    // [k]
  int32_t *sel = reinterpret_cast<int32_t *>(wsel + ((k + 1) & ~1));      // [k]
  float *hrow = reinterpret_cast<float *>(sel + ((k + 3) & ~3));  // [d], 16-byte aligned

  const int t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwave = blockDim.x >> 6;

  for (int j = tid; j < d; j += blockDim.x) hrow[j] = Elem<T>::load(h + (size_t)t * d + j);
  __syncthreads();

  // logit_i = w_i . h_t (+ b_i): one wave per expert, each lane takes 16-byte pieces of the row.
  constexpr int VEC = 16 / sizeof(T);
  for (int i = wave; i < N; i += nwave) {
    const T *wi = w_r + (size_t)i * d;
    double acc = 0.0;
#pragma unroll 4
    for (int j = lane * VEC; j < d; j += kWave * VEC) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(wi + j);
      const T *wv = reinterpret_cast<const T *>(&raw);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc = fma((double)Elem<T>::load(wv + v), (double)hrow[j + v], acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) g[i] = acc + (b_r ? (double)b_r[i] : 0.0);
  }
  __syncthreads();

  // softmax, max-subtracted
  double m = -INFINITY;
  for (int i = tid; i < N; i += blockDim.x) m = fmax(m, g[i]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = red[0];
  for (int w = 1; w < nwave; ++w) m = fmax(m, red[w]);
  __syncthreads();
  double part = 0.0;
  for (int i = tid; i < N; i += blockDim.x) {
    const double e = exp(g[i] - m);
    g[i] = e;
    part += e;
  }
  part = wave_sum(part);
  if (lane == 0) red[wave] = part;
  __syncthreads();
  double denom = red[0];
  for (int w = 1; w < nwave; ++w) denom += red[w];
  for (int i = tid; i < N; i += blockDim.x) {
    const double p = g[i] / denom;
    g[i] = p;
    probs[(size_t)t * N + i] = p;
  }
  __syncthreads();

  if (topk_ids == nullptr && topk_w == nullptr) return;
  select_topk(g, nullptr, N, k, sel);
  __syncthreads();
  mixing_weights(g, sel, k, renorm, wsel);
  __syncthreads();
  for (int s = tid; s < k; s += blockDim.x) {
    if (topk_ids) topk_ids[(size_t)t * k + s] = sel[s];
    if (topk_w) topk_w[(size_t)t * k + s] = (float)wsel[s];
  }
}

hipError_t launch_route(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, double *probs,
                        int32_t *topk_ids, float *topk_w, hipStream_t st) {
  const int N = ds.n_experts, k = ds.top_k, d = ds.d;
  const size_t smem = sizeof(double) * (((N + 1) & ~1) + 8 + ((k + 1) & ~1)) + sizeof(int32_t) * ((k + 3) & ~3) + sizeof(float) * d;
  if (ds.dtype == MOESPEC_BF16) {
    route_kernel<uint16_t><<<M, kRouteThreads, smem, st>>>(static_cast<const uint16_t *>(h),
                                                           static_cast<const uint16_t *>(wt.w_router), wt.b_router, d,
                                                           N, k, ds.renorm, probs, topk_ids, topk_w);
  } else {
    route_kernel<float><<<M, kRouteThreads, smem, st>>>(static_cast<const float *>(h),
                                                        static_cast<const float *>(wt.w_router), wt.b_router, d, N, k,
                                                        ds.renorm, probs, topk_ids, topk_w);
  }
  return hipGetLastError();
}

}  // namespace moespec
