// Stage 1 of Algorithm 1: router projection, softmax over all N experts (Eq. (1)), per-token
// top-k and mixing weights (Section 2.1).  Every decision in fp64.
//
// Two kernels.  The projection is spread over (token, group of 4 experts) workgroups so that the
// whole chip takes part: converting bf16 operands to fp64 costs several vector instructions per
// element, and one workgroup per token would leave that work on M compute units.  The softmax and
// the top-k then need one small workgroup per token.  Cross-lane fp64 shuffles are slow on this
// hardware (two 32-bit permutes per step), so all reductions go through LDS.
#include "common.h"

namespace moespec {

constexpr int kLogitThreads = 256;
constexpr int kRowsPerGroup = 4;                               // router rows per workgroup
constexpr int kSlices = kLogitThreads / kRowsPerGroup;         // threads that share one row (= 64)
constexpr int kSoftmaxThreads = 256;

// logits[t, i] = w_i . h_t (+ b_i).  Thread (el, sl) takes the 16-byte pieces sl, sl+64, ... of row
// i = 4 blockIdx.x + el and of h_t; all loads of a batch are issued together (the router weights of a
// layer are cold in every cache).
template <typename T>
__global__ __launch_bounds__(kLogitThreads) void logits_kernel(const T *__restrict__ h, const T *__restrict__ w_r,
                                                               const float *__restrict__ b_r, int d, int N,
                                                               double *__restrict__ logits) {
  __shared__ double part[kLogitThreads];
  __shared__ double part2[kRowsPerGroup * 8];
  const int t = blockIdx.y, tid = threadIdx.x;
  const int el = tid / kSlices, sl = tid % kSlices;
  const int e = blockIdx.x * kRowsPerGroup + el;
  constexpr int VEC = 16 / sizeof(T);  // elements per 16-byte piece
  constexpr int PB = 4;                // pieces in flight per operand
  const int npieces = d / VEC;         // d is a multiple of VEC
  const T *wrow = w_r + (size_t)(e < N ? e : N - 1) * d;
  const T *hrow = h + (size_t)t * d;
  double acc = 0.0;
  for (int p0 = 0; p0 < npieces; p0 += PB * kSlices) {
    uint4 wr[PB], hr[PB];
#pragma unroll
    for (int q = 0; q < PB; ++q) {
      const int pc = p0 + sl + q * kSlices;
      const bool ok = pc < npieces;
      wr[q] = ok ? *reinterpret_cast<const uint4 *>(wrow + (size_t)pc * VEC) : uint4{0u, 0u, 0u, 0u};
      hr[q] = ok ? *reinterpret_cast<const uint4 *>(hrow + (size_t)pc * VEC) : uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int q = 0; q < PB; ++q)
#pragma unroll
      for (int v = 0; v < VEC; ++v)
        acc = fma((double)Elem<T>::load(reinterpret_cast<const T *>(&wr[q]) + v),
                  (double)Elem<T>::load(reinterpret_cast<const T *>(&hr[q]) + v), acc);
  }
  part[tid] = acc;
  __syncthreads();
  if (sl < 8) {
    double a = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) a += part[el * kSlices + sl * 8 + q];
    part2[el * 8 + sl] = a;
  }
  __syncthreads();
  if (sl == 0 && e < N) {
    double a = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) a += part2[el * 8 + q];
    logits[(size_t)t * N + e] = a + (b_r ? (double)b_r[e] : 0.0);
  }
}

// probs[t, :] = softmax(logits[t, :]) in place (max-subtracted) - or, with the sigmoid gate, 1 / (1 + exp(-logit))
// per expert - then the natural top-k and its mixing weights if asked for.  One workgroup per token.
__global__ __launch_bounds__(kSoftmaxThreads) void softmax_topk_kernel(double *__restrict__ probs, int N, int k,
                                                                       int renorm, int sigmoid_gate,
                                                                       int32_t *__restrict__ topk_ids,
                                                                       float *__restrict__ topk_w,
                                                                       int32_t *__restrict__ zero_words, int n_zero) {
  extern __shared__ __align__(16) unsigned char smem[];
  double *g = reinterpret_cast<double *>(smem);               // [N, even] logits, then probabilities
  double *part = g + ((N + 1) & ~1);                          // [32] partial reductions
  double *wsel = part + 32;                                   // [k, even] + 1 denominator (+1 pad)
  int32_t *sel = reinterpret_cast<int32_t *>(wsel + ((k + 1) & ~1) + 2);  // [k, multiple of 4]
  int32_t *rank = sel + ((k + 3) & ~3);                       // [N]
  const int t = blockIdx.x, tid = threadIdx.x;
  if (zero_words && t == 0)
    for (int i = tid; i < n_zero; i += blockDim.x) zero_words[i] = 0;
  for (int i = tid; i < N; i += blockDim.x) g[i] = probs[(size_t)t * N + i];
  __syncthreads();
  if (sigmoid_gate) {  // uniform
    for (int i = tid; i < N; i += blockDim.x) {
      const double p = 1.0 / (1.0 + exp(-g[i]));
      g[i] = p;
      probs[(size_t)t * N + i] = p;
    }
    __syncthreads();
  } else {
    // 32 strided partial results, then every thread folds the 32 in index order
    if (tid < 32) {
      double m = -INFINITY;
      for (int i = tid; i < N; i += 32) m = fmax(m, g[i]);
      part[tid] = m;
    }
    __syncthreads();
    double m = part[0];
  #pragma unroll
    for (int j = 1; j < 32; ++j) m = fmax(m, part[j]);
    __syncthreads();
    for (int i = tid; i < N; i += blockDim.x) g[i] = exp(g[i] - m);
    __syncthreads();
    if (tid < 32) {
      double a = 0.0;
      for (int i = tid; i < N; i += 32) a += g[i];
      part[tid] = a;
    }
    __syncthreads();
    double denom = part[0];
  #pragma unroll
    for (int j = 1; j < 32; ++j) denom += part[j];
    for (int i = tid; i < N; i += blockDim.x) {
      const double p = g[i] / denom;
      g[i] = p;
      probs[(size_t)t * N + i] = p;
    }
    __syncthreads();
  }

  if (topk_ids == nullptr && topk_w == nullptr) return;
  select_topk(g, nullptr, N, k, sel, rank);
  __syncthreads();
  mixing_weights(g, sel, k, renorm, wsel, wsel + ((k + 1) & ~1));
  __syncthreads();
  for (int s = tid; s < k; s += blockDim.x) {
    if (topk_ids) topk_ids[(size_t)t * k + s] = sel[s];
    if (topk_w) topk_w[(size_t)t * k + s] = (float)wsel[s];
  }
}

hipError_t launch_route(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, double *probs,
                        int32_t *topk_ids, float *topk_w, int32_t *zero_words, int n_zero, hipStream_t st) {
  const int N = ds.n_experts, k = ds.top_k, d = ds.d;
  dim3 grid((N + kRowsPerGroup - 1) / kRowsPerGroup, M);
  if (ds.dtype == MOESPEC_BF16) {
    logits_kernel<uint16_t><<<grid, kLogitThreads, 0, st>>>(static_cast<const uint16_t *>(h),
                                                            static_cast<const uint16_t *>(wt.w_router), wt.b_router, d,
                                                            N, probs);
  } else {
    logits_kernel<float><<<grid, kLogitThreads, 0, st>>>(static_cast<const float *>(h),
                                                         static_cast<const float *>(wt.w_router), wt.b_router, d, N,
                                                         probs);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t smem = sizeof(double) * (((N + 1) & ~1) + 32 + ((k + 1) & ~1) + 2) +
                      sizeof(int32_t) * (((k + 3) & ~3) + N);
  softmax_topk_kernel<<<M, kSoftmaxThreads, smem, st>>>(probs, N, k, ds.renorm, ds.gate == MOESPEC_GATE_SIGMOID ? 1 : 0,
                                                        topk_ids, topk_w, zero_words,
                                                        n_zero);
  return hipGetLastError();
}

}  // namespace moespec
