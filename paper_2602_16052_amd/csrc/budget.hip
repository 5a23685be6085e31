// Stages 2-3 of Algorithm 1 without the expert maths: per-expert aggregation of routing
// probability over the tree (Eq. (5)), top-B shortlist (Section 3.2), restriction of every token's
// routing by truncation (Eq. (7)) or substitution (Eq. (8)), and the grouping of the surviving
// (token, slot) pairs into per-expert segments.  All decisions in fp64, ties to the lowest id.
#include "common.h"

namespace moespec {

constexpr int kBudgetThreads = 1024;
constexpr int kRedundantScoreTokens = 256;

// s_i = sum over t = 0..M-1 of probs[t, i], added strictly in ascending t; the loads of up to 32 rows
// are issued together so that the chain is bound by the adds, not by memory latency.
__device__ __forceinline__ double column_sum(const double *__restrict__ probs, int M, int N, int i) {
  double acc = 0.0;
  for (int t = 0; t < M; t += 32) {
    double v[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) v[u] = t + u < M ? probs[(size_t)(t + u) * N + i] : 0.0;
#pragma unroll
    for (int u = 0; u < 32; ++u) acc += v[u];  // rows past M add +0.0, which leaves the sum unchanged
  }
  return acc;
}

// The same sums for all N columns by a whole workgroup (N <= blockDim.x): the rows are fetched `rows_per_chunk`
// at a time with every thread loading (contiguous, one latency per chunk, the next chunk already in flight),
// parked in LDS, and thread i then adds column i row by row - the additions keep the strict ascending order,
// only the memory latency leaves the chain.  tab: rows_per_chunk * N doubles of LDS.  Synchronises.
constexpr int kScoreLoads = 4;  // values per thread and chunk
__device__ __forceinline__ double column_sums_staged(const double *__restrict__ probs, int M, int N,
                                                     int rows_per_chunk, double *tab) {
  const int tid = threadIdx.x, nt = blockDim.x;
  double nxt[kScoreLoads];
  auto fetch = [&](int t0) {
    const int n = (M - t0 < rows_per_chunk ? M - t0 : rows_per_chunk) * N;
#pragma unroll
    for (int u = 0; u < kScoreLoads; ++u) {
      const int idx = tid + u * nt;
      nxt[u] = idx < n ? probs[(size_t)t0 * N + idx] : 0.0;
    }
  };
  double acc = 0.0;
  fetch(0);
  for (int t0 = 0; t0 < M; t0 += rows_per_chunk) {
    const int rows = M - t0 < rows_per_chunk ? M - t0 : rows_per_chunk;
#pragma unroll
    for (int u = 0; u < kScoreLoads; ++u) {
      const int idx = tid + u * nt;
      if (idx < rows * N) tab[idx] = nxt[u];
    }
    __syncthreads();
    if (t0 + rows_per_chunk < M) fetch(t0 + rows_per_chunk);
    if (tid < N)
      for (int r = 0; r < rows; ++r) acc += tab[r * N + tid];
    __syncthreads();
  }
  return acc;
}

// Groups the surviving (token, slot) pairs by expert: segment i holds the pairs routed to
// seg_expert[i], tokens ascending.  Run by one whole workgroup; one wave per segment at a time,
// 64 tokens per ballot.  The routing table is staged in LDS slot-major (lanes read consecutive
// words) when it fits.  items receives the work items of the expert passes: the non-empty segments
// ordered by size, largest first (ties: lower segment first), each cut into piece_count(size) pieces of
// (almost) equal size; items[0].x = number of pieces, items[1 + r] = (segment, expert, offset, size) of
// piece r - the order in which the expert passes hand them out.
// lds: (3 B + 1 + (staged ? M k : 0)) int32.
__device__ void build_segments(const int32_t *tok_ids, int M, int k, int B, int staged, const int32_t *seg_expert,
                               int32_t *seg_off, int32_t *perm, int32_t *n_loaded, int4 *items, int32_t *lds) {
  int32_t *cnt = lds;           // [B + 1] exclusive offsets
  int32_t *sexp = cnt + B + 1;  // [B] seg_expert
  int32_t *sz = sexp + B;       // [B] sizes
  int32_t *copy = sz + B;       // [k][M] routing table, slot-major (if staged)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwave = blockDim.x >> 6;
  for (int i = tid; i < B; i += blockDim.x) sexp[i] = seg_expert[i];
  if (staged)
    for (int i = tid; i < M * k; i += blockDim.x) copy[(i % k) * M + i / k] = tok_ids[i];
  __syncthreads();
  auto id_at = [&](int t, int j) { return staged ? copy[j * M + t] : tok_ids[(size_t)t * k + j]; };

  for (int i = wave; i < B; i += nwave) {
    const int e = sexp[i];
    int c = 0;
    for (int t0 = 0; e >= 0 && t0 < M; t0 += kWave) {
      const int t = t0 + lane;
      bool has = false;
      if (t < M)
        for (int j = 0; j < k; ++j) has |= (id_at(t, j) == e);
      c += __popcll(__ballot(has));
    }
    if (lane == 0) sz[i] = c;
  }
  __syncthreads();
  if (wave == 0) {  // exclusive scan of the sizes, 64 segments per step
    int run = 0, loaded = 0, pieces = 0;
    for (int i0 = 0; i0 < B; i0 += kWave) {
      const int i = i0 + lane;
      const int c = i < B ? sz[i] : 0;
      pieces += piece_count(c);
      int incl = c;
#pragma unroll
      for (int sft = 1; sft < kWave; sft <<= 1) {
        const int v = __shfl_up(incl, sft, kWave);
        if (lane >= sft) incl += v;
      }
      if (i < B) {
        seg_off[i] = run + incl - c;
        cnt[i] = run + incl - c;
      }
      run += __shfl(incl, kWave - 1, kWave);
      loaded += __popcll(__ballot(c > 0));
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) pieces += __shfl_xor(pieces, sft, kWave);
    if (lane == 0) {
      seg_off[B] = run;
      items[0] = int4{pieces, 0, 0, 0};
      if (n_loaded) *n_loaded = loaded;
      cnt[B] = run;
    }
  }
  __syncthreads();
  for (int i = tid; i < B; i += blockDim.x) {
    const int c = sz[i];
    if (c > 0) {
      int first = 0;  // pieces of the segments that rank before this one
      for (int j = 0; j < B; ++j) first += (sz[j] > c || (sz[j] == c && j < i)) ? piece_count(sz[j]) : 0;
      const int q = piece_count(c), len = (c + q - 1) / q;
      for (int p = 0; p < q; ++p) items[1 + first + p] = int4{i, sexp[i], cnt[i] + p * len, min(len, c - p * len)};
    }
  }
  const int P = cnt[B];
  for (int p = P + tid; p < M * k; p += blockDim.x) perm[p] = -1;
  for (int i = wave; i < B; i += nwave) {
    const int e = sexp[i];
    int base = cnt[i];
    for (int t0 = 0; e >= 0 && t0 < M; t0 += kWave) {
      const int t = t0 + lane;
      int slot = -1;
      if (t < M)
        for (int j = 0; j < k; ++j)
          if (id_at(t, j) == e) slot = j;
      const unsigned long long mask = __ballot(slot >= 0);
      if (slot >= 0) perm[base + __popcll(mask & ((1ull << lane) - 1ull))] = t * k + slot;
      base += __popcll(mask);
    }
  }
}

// Bytes of the selection arrays at the start of the budget kernel's LDS (the score staging follows), and the
// rows of one staging chunk: kBudgetThreads * kScoreLoads values, at most 64 rows.
__host__ __device__ inline size_t budget_sel_bytes(int N, int k, int B) {
  const size_t b = sizeof(double) * (2 * (size_t)N + ((k + 1) & ~1) + 2) + sizeof(int32_t) * ((size_t)k + B + 2 * N + 1) + N;
  return (b + 15) & ~(size_t)15;
}
__host__ __device__ inline int budget_rows_per_chunk(int N) {
  const int r = kBudgetThreads * kScoreLoads / N;
  return r > 64 ? 64 : (r < 1 ? 1 : r);
}

// One workgroup per tree token.  Every workgroup recomputes the (tiny) scores and shortlist so that
// no grid-wide synchronisation is needed; workgroup 0 also writes them out.  The workgroup that
// finishes last (ticket counter done[0], zero at launch) builds the segments from everybody's rows,
// if they are wanted.  done[1 + r] (zero at launch) receives the number of surviving pairs of the expert
// with shortlist rank r.
__global__ __launch_bounds__(kBudgetThreads) void budget_kernel(
    const double *__restrict__ probs, int M, int N, int k, int B, int policy, int renorm,
    const int32_t *__restrict__ ext_shortlist, double *__restrict__ scores, int32_t *__restrict__ budget_ids,
    int32_t *__restrict__ seg_expert, int32_t *tok_ids, float *__restrict__ tok_w, int32_t *__restrict__ seg_off,
    int32_t *__restrict__ perm, int32_t *__restrict__ n_loaded, int4 *__restrict__ items, int staged,
    int want_segments, const double *__restrict__ scores_in, int32_t *done) {
  extern __shared__ __align__(16) unsigned char smem[];
  double *s = reinterpret_cast<double *>(smem);                  // [N] aggregate scores
  double *g = s + N;                                              // [N] this token's probabilities
  double *wsel = g + N;                                           // [k, even] + denominator
  int32_t *sel = reinterpret_cast<int32_t *>(wsel + ((k + 1) & ~1) + 2);  // [k]
  int32_t *S = sel + k;                                           // [B] shortlist in rank order
  int32_t *rank = S + B;                                          // [N] scratch of the selections
  int32_t *pos = rank + N;                                        // [N] shortlist rank of every expert
  int32_t *flag = pos + N;                                        // [1] "this workgroup is the last one"
  uint8_t *inS = reinterpret_cast<uint8_t *>(flag + 1);           // [N] membership
  double *tab = reinterpret_cast<double *>(smem + budget_sel_bytes(N, k, B));  // [rows_per_chunk, N] score staging
  const int rows_per_chunk = budget_rows_per_chunk(N);

  const int t = blockIdx.x, tid = threadIdx.x;

  for (int i = tid; i < N; i += blockDim.x) {
    g[i] = probs[(size_t)t * N + i];
    inS[i] = 0;
    pos[i] = 0x7fffffff;
  }
  if (ext_shortlist == nullptr) {
    // Eq. (5): s_i = sum over the M tree tokens of g_i(h_t), tokens in ascending order.
    // (large trees: summed once by scores_kernel instead of by every workgroup)
    if (scores_in) {
      for (int i = tid; i < N; i += blockDim.x) s[i] = scores_in[i];
    } else {
      const double acc = column_sums_staged(probs, M, N, rows_per_chunk, tab);
      if (tid < N) s[tid] = acc;
    }
    __syncthreads();
    select_topk(s, nullptr, N, B, S, rank);
  } else {
    for (int r = tid; r < B; r += blockDim.x) S[r] = ext_shortlist[r];
    if (scores && t == 0)  // uniform in the workgroup
      for (int i = tid; i < N; i += blockDim.x) s[i] = scores_in ? scores_in[i] : column_sum(probs, M, N, i);
  }
  __syncthreads();
  for (int r = tid; r < B; r += blockDim.x)
    if ((uint32_t)S[r] < (uint32_t)N) {  // ids outside [0, N) in an external shortlist are ignored
      inS[S[r]] = 1;
      atomicMin(&pos[S[r]], r);  // an expert named twice counts at its first rank
    }
  __syncthreads();

  if (t == 0) {
    for (int i = tid; i < N; i += blockDim.x) {
      if (scores) scores[i] = s[i];
      if (inS[i]) {  // position of expert i among the shortlisted experts in ascending id
        int pos = 0;
        for (int j = 0; j < i; ++j) pos += inS[j];
        seg_expert[pos] = i;
      }
    }
    if (tid < B) {
      int n_member = 0;  // < B only if an external shortlist repeats or misnames an expert
      for (int j = 0; j < N; ++j) n_member += inS[j];
      for (int r = tid; r < B; r += blockDim.x) {
        if (r >= n_member) seg_expert[r] = -1;
        budget_ids[r] = S[r];
      }
    }
  }

  if (policy == MOESPEC_TRUNCATE) {
    // Natural top-k and its weights, then drop the slots outside S; kept weights are unchanged.
    select_topk(g, nullptr, N, k, sel, rank);
    __syncthreads();
    mixing_weights(g, sel, k, renorm, wsel, wsel + ((k + 1) & ~1));
    __syncthreads();
    for (int j = tid; j < k; j += blockDim.x) {
      const bool keep = (uint32_t)sel[j] < (uint32_t)N && inS[sel[j]] != 0;  // an unfilled slot (NaN scores) is dropped
      tok_ids[(size_t)t * k + j] = keep ? sel[j] : -1;
      tok_w[(size_t)t * k + j] = keep ? (float)wsel[j] : 0.0f;
      if (keep) atomicAdd(&done[1 + pos[sel[j]]], 1);
    }
  } else {
    // Top-k inside S by g_i(h_t); weights over the constrained selection.  Slots stay unfilled (-1)
    // only when an external shortlist names fewer than k valid experts.
    select_topk(g, inS, N, k, sel, rank);
    __syncthreads();
    mixing_weights(g, sel, k, renorm, wsel, wsel + ((k + 1) & ~1));
    __syncthreads();
    for (int j = tid; j < k; j += blockDim.x) {
      const bool filled = (uint32_t)sel[j] < (uint32_t)N;
      tok_ids[(size_t)t * k + j] = filled ? sel[j] : -1;
      tok_w[(size_t)t * k + j] = filled ? (float)wsel[j] : 0.0f;
      if (filled) atomicAdd(&done[1 + pos[sel[j]]], 1);
    }
  }

  if (!want_segments) return;
  // Last workgroup to arrive groups the pairs of all tokens.  One thread publishes the workgroup's
  // rows (the barrier before it orders everybody's stores first) and takes the ticket; device-scope
  // fences are expensive, so they are not executed by every wave.
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    const bool is_last = atomicAdd(done, 1) == (int)gridDim.x - 1;
    if (is_last) __threadfence();
    *flag = is_last;
  }
  __syncthreads();
  const bool last = *flag != 0;
  __syncthreads();  // everybody has read the flag before the LDS is reused below
  if (!last) return;
  build_segments(tok_ids, M, k, B, staged, seg_expert, seg_off, perm, n_loaded, items,
                 reinterpret_cast<int32_t *>(smem));
}

// Eq. (5) once for the whole tree (same order of additions): used when the tree is so large that recomputing
// the scores in every workgroup of budget_kernel (M^2 N loads in total) would dominate.  One workgroup.
__global__ __launch_bounds__(kBudgetThreads) void scores_kernel(const double *__restrict__ probs, int M, int N,
                                                                double *__restrict__ scores) {
  extern __shared__ __align__(16) unsigned char smem[];
  const double acc = column_sums_staged(probs, M, N, budget_rows_per_chunk(N), reinterpret_cast<double *>(smem));
  if ((int)threadIdx.x < N) scores[threadIdx.x] = acc;
}

__global__ void zero_words_kernel(int32_t *p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

hipError_t launch_budget(const moespec_desc &ds, const double *probs, int M, int B, int policy,
                         const int32_t *ext_shortlist, double *scores, int32_t *budget_ids, int32_t *tok_ids,
                         float *tok_w, int32_t *seg_expert, int32_t *seg_off, int32_t *perm, int32_t *n_loaded,
                         int4 *items, int32_t *done, bool done_is_zero, bool want_segments, double *score_scratch,
                         hipStream_t st) {
  const int N = ds.n_experts, k = ds.top_k;
  if (!done_is_zero) {
    zero_words_kernel<<<1, 256, 0, st>>>(done, 1 + N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // above this many tokens the redundant per-workgroup scoring (M^2 N loads in total) is replaced by one pass
  const double *scores_in = nullptr;
  if (M > kRedundantScoreTokens && (ext_shortlist == nullptr || scores != nullptr)) {
    scores_kernel<<<1, kBudgetThreads, sizeof(double) * budget_rows_per_chunk(N) * N, st>>>(probs, M, N,
                                                                                           score_scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    scores_in = score_scratch;
  }
  const int staged = (size_t)M * k <= 8192;
  const size_t smem_sel = budget_sel_bytes(N, k, B) + sizeof(double) * budget_rows_per_chunk(N) * N;
  const size_t smem_seg = sizeof(int32_t) * (3 * B + 1 + (staged ? (size_t)M * k : 0));
  budget_kernel<<<M, kBudgetThreads, smem_sel > smem_seg ? smem_sel : smem_seg, st>>>(
      probs, M, N, k, B, policy, ds.renorm, ext_shortlist, scores, budget_ids, seg_expert, tok_ids, tok_w, seg_off, perm,
      n_loaded, items, staged, want_segments ? 1 : 0, scores_in, done);
  return hipGetLastError();
}

}  // namespace moespec
