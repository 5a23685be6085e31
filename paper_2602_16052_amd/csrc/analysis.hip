// Analysis steps around the hot path: the static ranking of Eq. (4) (selection frequency over
// calibration tokens and the B most frequent experts, which enter the layer as an external
// shortlist), the coverage curve of Section 4.6 (cumulative routing probability captured by the
// top-B experts) and the reconstruction error of Section 4.5 (||O_S - O*||^2 / ||O*||^2).
// Tiny, latency-bound kernels; integer work is exact, floating point is fp64 in a fixed order.
#include "common.h"

namespace moespec {

constexpr int kAnalysisThreads = 1024;

// c_i += #{(t, slot) : topk_ids[t, slot] == i}.  Integer atomics: the result does not depend on order.
__global__ __launch_bounds__(256) void calibration_count_kernel(const int32_t *__restrict__ topk_ids, int n, int N,
                                                                unsigned long long *__restrict__ counts) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const int e = topk_ids[i];
    if ((uint32_t)e < (uint32_t)N) atomicAdd(&counts[e], 1ull);
  }
}

// shortlist[r] = expert with rank r < B when ordered by (count descending, id ascending).  One workgroup.
__global__ __launch_bounds__(kAnalysisThreads) void static_shortlist_kernel(const long long *__restrict__ counts,
                                                                            int N, int B,
                                                                            int32_t *__restrict__ shortlist) {
  __shared__ long long c[1024];
  for (int i = threadIdx.x; i < N; i += blockDim.x) c[i] = counts[i];
  __syncthreads();
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    const long long ci = c[i];
    int r = 0;
    for (int j = 0; j < N; ++j) r += (c[j] > ci || (c[j] == ci && j < i)) ? 1 : 0;
    if (r < B) shortlist[r] = i;
  }
}

// curve[B-1] = (sum of the B largest scores) / (sum of all scores); the total is added in expert order,
// the partial sums in rank order (ties: lowest id first).  One workgroup.
__global__ __launch_bounds__(kAnalysisThreads) void coverage_curve_kernel(const double *__restrict__ scores, int N,
                                                                          double *__restrict__ curve) {
  __shared__ double s[1024];
  __shared__ int32_t order[1024];
  for (int i = threadIdx.x; i < N; i += blockDim.x) s[i] = scores[i];
  __syncthreads();
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    const double si = s[i];
    int r = 0;
    for (int j = 0; j < N; ++j) r += ranks_before(s[j], j, si, i) ? 1 : 0;
    order[r] = i;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (int i = 0; i < N; ++i) total += s[i];
    double acc = 0.0;
    for (int r = 0; r < N; ++r) {
      acc += s[order[r]];
      curve[r] = acc / total;
    }
  }
}

// part[2 t] = ||a_t - b_t||^2, part[2 t + 1] = ||b_t||^2 for token t (one workgroup per token; thread i
// folds the elements i, i + 256, ... in ascending order, then the 256 partial sums are folded in
// thread order).
template <typename T>
__global__ __launch_bounds__(256) void sqdiff_rows_kernel(const T *__restrict__ a, const T *__restrict__ b, int d,
                                                          double *__restrict__ part) {
  __shared__ double num[256], den[256];
  const int t = blockIdx.x, tid = threadIdx.x;
  double n = 0.0, q = 0.0;
  for (int j = tid; j < d; j += 256) {
    const double av = (double)Elem<T>::load(a + (size_t)t * d + j), bv = (double)Elem<T>::load(b + (size_t)t * d + j);
    const double df = av - bv;
    n += df * df;
    q += bv * bv;
  }
  num[tid] = n;
  den[tid] = q;
  __syncthreads();
  if (tid == 0) {
    double sn = 0.0, sd = 0.0;
    for (int i = 0; i < 256; ++i) {
      sn += num[i];
      sd += den[i];
    }
    part[2 * t] = sn;
    part[2 * t + 1] = sd;
  }
}

// err[0] = num / den, err[1] = num, err[2] = den, tokens added in ascending order.
__global__ void sqdiff_total_kernel(const double *__restrict__ part, int M, double *__restrict__ err) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double sn = 0.0, sd = 0.0;
  for (int t = 0; t < M; ++t) {
    sn += part[2 * t];
    sd += part[2 * t + 1];
  }
  err[0] = sn / sd;
  err[1] = sn;
  err[2] = sd;
}

// ---- Oracle ranking, Eq. (6) ------------------------------------------------------------------------
// With C_i[t] = w[t, slot] * E_i(h_t) for the slot that routes token t to expert i (zero otherwise) and the
// gold output O* = sum_i C_i, the error of a set S is ||O*||^2 - 2 sum_{i in S} b_i + sum_{i,j in S} G_ij
// with G_ij = sum_t <C_i[t], C_j[t]> and b_i = sum_j G_ij.  Adding i to S changes it by
// G_ii - 2 b_i + 2 sum_{j in S} G_ij, so the greedy choice needs only the Gram matrix.

// pair_gram[t, a, b] = w_a w_b <y[t k + a], y[t k + b]> for the surviving slots a, b of token t (0 otherwise),
// in fp64; thread i folds the elements i, i + 256, ... in ascending order, then thread 0 the 256 partial sums.
__global__ __launch_bounds__(256) void pair_gram_kernel(const float *__restrict__ y, int splits, size_t split_stride,
                                                        const int32_t *__restrict__ tok_ids,
                                                        const float *__restrict__ tok_w, int k, int d,
                                                        double *__restrict__ pair_gram) {
  __shared__ double part[256];
  const int t = blockIdx.x, tid = threadIdx.x;
  auto elem = [&](int slot, int j) {
    const float *p = y + ((size_t)t * k + slot) * d + j;
    float v = p[0];
    for (int sp = 1; sp < splits; ++sp) v += p[sp * split_stride];  // same order as the combine
    return (double)v;
  };
  for (int a = 0; a < k; ++a)
    for (int b = a; b < k; ++b) {
      const bool live = tok_ids[(size_t)t * k + a] >= 0 && tok_ids[(size_t)t * k + b] >= 0;  // uniform
      double acc = 0.0;
      if (live)
        for (int j = tid; j < d; j += 256) acc += elem(a, j) * elem(b, j);
      part[tid] = acc;
      __syncthreads();
      if (tid == 0) {
        double s = 0.0;
        for (int i = 0; i < 256; ++i) s += part[i];
        s *= (double)tok_w[(size_t)t * k + a] * (double)tok_w[(size_t)t * k + b];
        pair_gram[((size_t)t * k + a) * k + b] = live ? s : 0.0;
        pair_gram[((size_t)t * k + b) * k + a] = live ? s : 0.0;
      }
      __syncthreads();
    }
}

// One workgroup: Gram matrix (tokens added in ascending order), then the greedy selection.
// gram: [N, N] matrix, then b[N], cross[N], taken[N] (as doubles).
__global__ __launch_bounds__(kAnalysisThreads) void oracle_greedy_kernel(const double *__restrict__ pair_gram,
                                                                         const int32_t *__restrict__ tok_ids, int M,
                                                                         int N, int k, int B, double *gram,
                                                                         int32_t *__restrict__ ranking,
                                                                         double *__restrict__ err) {
  __shared__ double val[kAnalysisThreads];
  __shared__ int32_t idx[kAnalysisThreads];
  __shared__ double total_s, err_s;
  double *G = gram, *bvec = gram + (size_t)N * N, *cross = bvec + N, *taken = cross + N;
  const int tid = threadIdx.x, nt = blockDim.x;
  for (size_t i = tid; i < (size_t)N * (N + 3); i += nt) gram[i] = 0.0;
  __syncthreads();
  for (int t = 0; t < M; ++t) {  // experts of one token are distinct: no two threads meet on an entry
    for (int p = tid; p < k * k; p += nt) {
      const int ea = tok_ids[(size_t)t * k + p / k], eb = tok_ids[(size_t)t * k + p % k];
      if (ea >= 0 && eb >= 0 && ea < N && eb < N) G[(size_t)ea * N + eb] += pair_gram[(size_t)t * k * k + p];
    }
    __syncthreads();
  }
  for (int i = tid; i < N; i += nt) {
    double s = 0.0;
    for (int j = 0; j < N; ++j) s += G[(size_t)i * N + j];
    bvec[i] = s;
  }
  __syncthreads();
  if (tid == 0) {
    double s = 0.0;
    for (int i = 0; i < N; ++i) s += bvec[i];
    total_s = s;  // ||O*||^2
    err_s = s;    // error of the empty set
  }
  __syncthreads();
  for (int step = 0; step < B; ++step) {
    // candidate of this thread: the best of i = tid, tid + nt, ... (smaller change first, then lower id)
    double best = INFINITY;
    int besti = 0x7fffffff;
    for (int i = tid; i < N; i += nt)
      if (taken[i] == 0.0) {
        const double delta = G[(size_t)i * N + i] - 2.0 * bvec[i] + 2.0 * cross[i];
        if (delta < best || (delta == best && i < besti)) {
          best = delta;
          besti = i;
        }
      }
    val[tid] = best;
    idx[tid] = besti;
    __syncthreads();
    for (int s = nt >> 1; s > 0; s >>= 1) {
      if (tid < s) {
        const double o = val[tid + s];
        const int oi = idx[tid + s];
        if (o < val[tid] || (o == val[tid] && oi < idx[tid])) {
          val[tid] = o;
          idx[tid] = oi;
        }
      }
      __syncthreads();
    }
    const int pick = idx[0];
    if (tid == 0) {
      err_s += val[0];
      ranking[step] = pick;
      err[step] = err_s / total_s;
      taken[pick] = 1.0;
    }
    for (int i = tid; i < N; i += nt) cross[i] += G[(size_t)i * N + pick];
    __syncthreads();
  }
}

hipError_t launch_oracle_ranking(const moespec_desc &ds, const float *y, int splits, size_t split_stride,
                                 const int32_t *tok_ids, const float *tok_w, int M, int B, double *pair_gram,
                                 double *gram, int32_t *ranking, double *err, hipStream_t st) {
  pair_gram_kernel<<<M, 256, 0, st>>>(y, splits, split_stride, tok_ids, tok_w, ds.top_k, ds.d, pair_gram);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  oracle_greedy_kernel<<<1, kAnalysisThreads, 0, st>>>(pair_gram, tok_ids, M, ds.n_experts, ds.top_k, B, gram, ranking,
                                                       err);
  return hipGetLastError();
}

hipError_t launch_calibration_count(const int32_t *topk_ids, int M, int k, int N, int64_t *counts, hipStream_t st) {
  const int n = M * k;
  int blocks = (n + 255) / 256;
  blocks = blocks > 1024 ? 1024 : blocks;
  calibration_count_kernel<<<blocks, 256, 0, st>>>(topk_ids, n, N, reinterpret_cast<unsigned long long *>(counts));
  return hipGetLastError();
}

hipError_t launch_static_shortlist(const int64_t *counts, int N, int B, int32_t *shortlist, hipStream_t st) {
  static_shortlist_kernel<<<1, kAnalysisThreads, 0, st>>>(reinterpret_cast<const long long *>(counts), N, B,
                                                          shortlist);
  return hipGetLastError();
}

hipError_t launch_coverage_curve(const double *scores, int N, double *curve, hipStream_t st) {
  coverage_curve_kernel<<<1, kAnalysisThreads, 0, st>>>(scores, N, curve);
  return hipGetLastError();
}

hipError_t launch_reconstruction_error(const moespec_desc &ds, const void *out_budgeted, const void *out_full, int M,
                                       double *part, double *err, hipStream_t st) {
  if (ds.dtype == MOESPEC_BF16)
    sqdiff_rows_kernel<uint16_t><<<M, 256, 0, st>>>(static_cast<const uint16_t *>(out_budgeted),
                                                    static_cast<const uint16_t *>(out_full), ds.d, part);
  else
    sqdiff_rows_kernel<float><<<M, 256, 0, st>>>(static_cast<const float *>(out_budgeted),
                                                 static_cast<const float *>(out_full), ds.d, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  sqdiff_total_kernel<<<1, 64, 0, st>>>(part, M, err);
  return hipGetLastError();
}

// ---- streaming read (measurement aid): every 16-byte piece of the buffer once, eight loads in flight per lane --
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ p, size_t n16,
                                                          uint32_t *__restrict__ checksum) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  constexpr int U = 8;  // 16-byte loads in flight per lane
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u].x + v[u].y + v[u].z + v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = p[i];
    acc += a.x + a.y + a.z + a.w;
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s, kWave);
  // one word per workgroup and a single writer per word: no atomics on the way out (thousands of atomics on
  // one address would take longer than the read itself)
  __shared__ uint32_t part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) checksum[blockIdx.x] += part[0] + part[1] + part[2] + part[3];
}

hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *checksum, hipStream_t st) {
  const size_t n16 = bytes / 16;
  // One workgroup per compute unit with 8 loads in flight per lane (8 MB in flight on the chip) measured
  // fastest: 6.4 TB/s on a 2 GiB buffer, against 6.3 with 512 workgroups x 4 loads and 5.3-5.6 with 16 MB in
  // flight (2048 x 4 or 512 x 16).
  const size_t want = (n16 + 255) / 256;
  const int blocks = (int)(want < MOESPEC_STREAM_READ_WORDS ? want : MOESPEC_STREAM_READ_WORDS);
  stream_read_kernel<<<blocks, 256, 0, st>>>(static_cast<const uint4 *>(buf), n16, checksum);
  return hipGetLastError();
}

}  // namespace moespec
