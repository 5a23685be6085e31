// Stages 1-3 of Algorithm 1 for the fused layer call on small trees, in two launches with no dependence
// between workgroups inside a launch:
//
//   logits_mfma_kernel    the router projection w_i . h_t of Eq. (1) for all tokens and experts on the fp64
//                         matrix cores, as partial sums over slices of the hidden dimension
//   route_budget_kernel   one workgroup per tree token.  EVERY workgroup rebuilds the whole M x N table of
//                         routing probabilities from those partial sums (bias, softmax or sigmoid gate of
//                         Eq. (1)), the aggregate scores of Eq. (5) and the top-B shortlist (Section 3.2) in its
//                         LDS - a few thousand exponentials, cheaper than a second pass over global memory and a
//                         grid-wide wait - then restricts its own token's routing (Eq. (7) / Eq. (8)) and
//                         writes the pair lists of the shortlist ranks it is responsible for: for every loaded
//                         expert the (token, slot) pairs routed to it, tokens ascending, which is what the
//                         expert passes consume.
//
// Every decision in fp64, ties to the lowest expert id, as in the staged kernels of route.hip / budget.hip,
// which remain the path of the stage calls, of fp32 layers and of trees whose table does not fit the LDS.
#include "common.h"

namespace moespec {

typedef __attribute__((ext_vector_type(4))) double f64x4;

constexpr int kLogitWaves = 4;
constexpr int kPrologueThreads = 1024;
constexpr int kSoftmaxSegs = 16;  // threads that share one row of the table in the softmax
// Tables above this many entries get their softmax in a launch of its own (measured on MI355X: 4032 entries are
// 0.6 us faster rebuilt in every workgroup, 8128 entries 0.9 us and 16256 entries 2.3 us faster with the extra launch).
constexpr long long kSplitSoftmaxAbove = 6000;

__device__ __forceinline__ double bf16_to_f64(uint32_t word, int hi) {
  return (double)__uint_as_float(hi ? (word & 0xffff0000u) : (word << 16));
}

// partial[q][t][e] = sum over the q-th slice of the hidden dimension of h[t][j] * w_r[e][j], in fp64.
// Workgroup (x, q): x = output tile (16 tokens x 16 experts), q = slice; its 4 waves cut the slice again into
// runs of 32-element blocks and add their results through LDS in wave order.  v_mfma_f64_16x16x4: lane (i, g)
// = (lane % 16, lane / 16) supplies A[i][g] and B[g][i] and receives D[g + 4 r][i] in accumulator r.  A lane
// loads 8 consecutive elements (16 bytes) of its token row and of its expert row per block; which of the 32
// elements of a block meet in one instruction is immaterial, the sum over the block is complete after 8 of them.
__global__ __launch_bounds__(kLogitWaves *kWave) void logits_mfma_kernel(const uint16_t *__restrict__ h,
                                                                          const uint16_t *__restrict__ w_r, int M,
                                                                          int N, int d, int n_slices,
                                                                          double *__restrict__ partial) {
  __shared__ double red[kLogitWaves][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e_tiles = (N + 15) / 16;
  const int tt = blockIdx.x / e_tiles, et = blockIdx.x % e_tiles, q = blockIdx.y;
  const int i = lane & 15, g = lane >> 4;
  const int t = min(tt * 16 + i, M - 1), e = min(et * 16 + i, N - 1);  // pad rows repeat the last one, never stored
  const int n_blocks = d / 32, parts = n_slices * kLogitWaves, part = q * kLogitWaves + wave;
  const int b0 = (int)((long long)part * n_blocks / parts), b1 = (int)((long long)(part + 1) * n_blocks / parts);
  const uint16_t *ha = h + (size_t)t * d + g * 8, *wb = w_r + (size_t)e * d + g * 8;
  f64x4 acc = {0.0, 0.0, 0.0, 0.0};
  constexpr int PB = 4;  // blocks in flight
  for (int b = b0; b < b1; b += PB) {
    uint4 A[PB], Bv[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int bb = min(b + u, b1 - 1);
      A[u] = *reinterpret_cast<const uint4 *>(ha + (size_t)bb * 32);
      Bv[u] = *reinterpret_cast<const uint4 *>(wb + (size_t)bb * 32);
    }
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      if (b + u < b1) {  // uniform in the wave
        const uint32_t *a = reinterpret_cast<const uint32_t *>(&A[u]);
        const uint32_t *bw = reinterpret_cast<const uint32_t *>(&Bv[u]);
#pragma unroll
        for (int m = 0; m < 8; ++m)
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(bf16_to_f64(a[m >> 1], m & 1), bf16_to_f64(bw[m >> 1], m & 1), acc,
                                                     0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) red[wave][(g + 4 * r) * 16 + i] = acc[r];
  __syncthreads();
  const int x = threadIdx.x, row = tt * 16 + x / 16, col = et * 16 + x % 16;
  if (row < M && col < N) {
    double a = red[0][x];
#pragma unroll
    for (int w = 1; w < kLogitWaves; ++w) a += red[w][x];
    partial[((size_t)q * M + row) * N + col] = a;
  }
}

// ---- 16-lane all-reductions through DPP (no LDS, no barrier).  Every lane of a row of 16 ends with the same
// bits: each step combines a value with its partner's, and the operations used are commutative.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
__device__ __forceinline__ double row16_max(double v) {
  v = fmax(v, dpp_f64<kDppXor1>(v));
  v = fmax(v, dpp_f64<kDppXor2>(v));
  v = fmax(v, dpp_f64<kDppHalfMirror>(v));
  return fmax(v, dpp_f64<kDppMirror>(v));
}
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_f64<kDppXor1>(v);
  v += dpp_f64<kDppXor2>(v);
  v += dpp_f64<kDppHalfMirror>(v);
  return v + dpp_f64<kDppMirror>(v);
}
__device__ __forceinline__ int row16_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, kDppXor1, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppXor2, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppHalfMirror, 0xf, 0xf, false);
  return v + __builtin_amdgcn_update_dpp(0, v, kDppMirror, 0xf, 0xf, false);
}

// exp(x) for x <= 0 (the max-subtracted argument of a softmax): x = n ln 2 + r with |r| <= ln 2 / 2, the Taylor
// polynomial of degree 12 in r (truncation error below 2e-16 relative) and a scaling by 2^n.  Every workgroup of
// the kernel below evaluates the whole table, so the two dozen instructions of this form matter; arguments
// below -800 give 0, NaN gives NaN further on (0 * inf in the normalisation).
__device__ __forceinline__ double exp_nonpos(double x) {
  x = fmax(x, -800.0);
  const double n = rint(x * 1.4426950408889634);
  double r = fma(n, -6.93147180369123816490e-01, x);
  r = fma(n, -1.90821492927058770002e-10, r);
  double p = 1.0 / 479001600.0;
  p = fma(p, r, 1.0 / 39916800.0);
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  return ldexp(p, (int)n);
}

// Eq. (1) row by row, for tables so large that rebuilding all of them in every workgroup of route_budget_kernel
// would cost more than one more launch: probs[t, :] = gate(sum of the slices of the router projection + bias).
// One wave per token; a lane holds up to 4 experts (N <= 256); 16-lane DPP reductions, then two cross-row steps.
template <int Q>
__global__ __launch_bounds__(kWave) void softmax_rows_kernel(const double *__restrict__ partial,
                                                            const float *__restrict__ bias, int M, int N,
                                                            int sigmoid_gate, double *__restrict__ probs,
                                                            int32_t *__restrict__ zero_words, int n_zero) {
  const int t = blockIdx.x, lane = threadIdx.x;
  if (zero_words && t == 0)  // counters of a later kernel, cleared here instead of by a launch of their own
    for (int i = lane; i < n_zero; i += kWave) zero_words[i] = 0;
  const size_t MN = (size_t)M * N;
  double val[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = lane + kWave * u;
    double a = -INFINITY;
    if (i < N) {
      a = partial[(size_t)t * N + i];
#pragma unroll
      for (int q = 1; q < Q; ++q) a += partial[q * MN + (size_t)t * N + i];
      a += bias ? (double)bias[i] : 0.0;
    }
    val[u] = a;
  }
  auto all_lanes = [](double v, auto op) {  // the 16-lane result of every row combined across the 4 rows
    v = op(v, __shfl_xor(v, 16, kWave));
    return op(v, __shfl_xor(v, 32, kWave));
  };
  if (sigmoid_gate) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (lane + kWave * u < N) probs[(size_t)t * N + lane + kWave * u] = 1.0 / (1.0 + exp(-val[u]));
    return;
  }
  double m = fmax(fmax(val[0], val[1]), fmax(val[2], val[3]));
  m = all_lanes(row16_max(m), [](double a, double b) { return fmax(a, b); });
  double a = 0.0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    val[u] = exp_nonpos(val[u] - m);  // lanes past the row end hold -inf: they come out as 0
    a += val[u];
  }
  const double inv = 1.0 / all_lanes(row16_sum(a), [](double x, double y) { return x + y; });
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (lane + kWave * u < N) probs[(size_t)t * N + lane + kWave * u] = val[u] * inv;
}

// LDS of route_budget_kernel.  Rows of the table are N + 1 doubles apart: lanes that walk down a column (one token
// per lane) then touch different banks.
struct PrologueLds {
  size_t g, s, red, S, cand, rank, pos, sel, inS, total;
};
__host__ __device__ inline PrologueLds prologue_lds(int M, int N, int k, int B) {
  PrologueLds L;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + 15) & ~(size_t)15;
    return at;
  };
  L.g = take(sizeof(double) * (size_t)M * (N + 1));
  L.s = take(sizeof(double) * N);
  L.red = take(sizeof(double) * kPrologueThreads);
  L.S = take(sizeof(int32_t) * B);
  L.cand = take(sizeof(int32_t) * (N + kWave));
  L.rank = take(sizeof(int32_t) * N);
  L.pos = take(sizeof(int32_t) * N);
  L.sel = take(sizeof(int32_t) * k);
  L.inS = take((size_t)N);
  L.total = off;
  return L;
}

// list_count[r] = number of pairs routed to the expert at shortlist rank r after the restriction;
// lists[r * list_stride + p] = flat id t * k + slot of its p-th pair, tokens ascending.
// Q = slices of the router projection, NE = ceil(N / 16) = elements of a table row per lane in the softmax (both
// compile-time so that the short loops unroll: a taken branch costs this hardware about as much as ten fp64
// operations).  Up to the shortlist the whole workgroup works on the table (16 consecutive lanes share a row and
// reduce through DPP; rank counts split the rivals of a candidate over the threads with the same index modulo a
// power of two and add up with integer LDS atomics).  Comparisons are written without short-circuit evaluation and
// loops in fixed blocks of four or eight, so that the code stays straight-line.
template <int Q, int NE>
__global__ __launch_bounds__(kPrologueThreads) void route_budget_kernel(
    const double *__restrict__ partial, const float *__restrict__ bias, int M, int N, int k, int B, int policy,
    int renorm, int sigmoid_gate, const int32_t *__restrict__ ext_shortlist, double *__restrict__ probs_out,
    double *__restrict__ scores_out, int32_t *__restrict__ budget_ids, int32_t *__restrict__ seg_expert,
    int32_t *__restrict__ tok_ids, float *__restrict__ tok_w, int32_t *__restrict__ list_count,
    int32_t *__restrict__ lists, int list_stride, int table_ready) {
  extern __shared__ __align__(16) unsigned char smem[];
  const PrologueLds L = prologue_lds(M, N, k, B);
  double *g = reinterpret_cast<double *>(smem + L.g);        // [M][N + 1] logits, then routing probabilities
  double *s = reinterpret_cast<double *>(smem + L.s);        // [N] aggregate scores
  double *red = reinterpret_cast<double *>(smem + L.red);    // [1024] partial column sums
  int32_t *S = reinterpret_cast<int32_t *>(smem + L.S);      // [B] shortlist in rank order
  int32_t *cand = reinterpret_cast<int32_t *>(smem + L.cand);  // [n_cand, padded to 64] a token's candidates
  int32_t *rank = reinterpret_cast<int32_t *>(smem + L.rank);
  int32_t *pos = reinterpret_cast<int32_t *>(smem + L.pos);  // [N] shortlist rank of every expert
  volatile int32_t *sel = reinterpret_cast<int32_t *>(smem + L.sel);  // [k] this token's selection (wave 0 only)
  uint8_t *inS = smem + L.inS;
  constexpr int nt = kPrologueThreads;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int own = blockIdx.x;  // this workgroup's token
  const int NS = N + 1;

  // logits: the slices of the hidden dimension added in slice order, plus the router bias
  // (table_ready: `partial` already holds the finished routing probabilities, one slice, and Eq. (1) is skipped)
  const int MN = M * N;
  const bool fixed_col = nt % N == 0;  // then element tid + u nt always lies in column tid % N
  const int col0 = tid % N, row0 = tid / N, rows_per_step = nt / N;
  const double own_bias = (bias && fixed_col) ? (double)bias[col0] : 0.0;
  for (int x0 = 0; x0 < MN; x0 += 4 * nt) {
    double v[4][Q];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int x = x0 + u * nt + tid;
        v[u][q] = x < MN ? partial[(size_t)q * MN + x] : 0.0;
      }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int x = x0 + u * nt + tid;
      if (x < MN) {
        double a = v[u][0];
#pragma unroll
        for (int q = 1; q < Q; ++q) a += v[u][q];
        const int t = fixed_col ? (x0 / nt + u) * rows_per_step + row0 : x / N;
        const int i = fixed_col ? col0 : x % N;
        g[t * NS + i] = a + (fixed_col ? own_bias : (bias ? (double)bias[i] : 0.0));
      }
    }
  }
  for (int i = tid; i < N; i += nt) {
    inS[i] = 0;
    pos[i] = 0x7fffffff;
    rank[i] = 0;
  }
  __syncthreads();

  // Eq. (1): 16 lanes per row, 64 rows per round; a lane holds its NE elements of the row in registers
  const int seg = tid & 15;
  for (int t0 = 0; t0 < M && !table_ready; t0 += nt / 16) {
    const int t = t0 + (tid >> 4);
    double *row = g + (t < M ? t : M - 1) * NS;
    double val[NE];
#pragma unroll
    for (int u = 0; u < NE; ++u) val[u] = (t < M && seg + 16 * u < N) ? row[seg + 16 * u] : -INFINITY;
    if (sigmoid_gate) {
#pragma unroll
      for (int u = 0; u < NE; ++u)
        if (t < M && seg + 16 * u < N) row[seg + 16 * u] = 1.0 / (1.0 + exp(-val[u]));
    } else {
      double m = val[0];
#pragma unroll
      for (int u = 1; u < NE; ++u) m = fmax(m, val[u]);
      m = row16_max(m);
      double a = 0.0;
#pragma unroll
      for (int u = 0; u < NE; ++u) {
        val[u] = exp_nonpos(val[u] - m);  // elements past the row end are -inf: they come out as 0
        a += val[u];
      }
      const double inv = 1.0 / row16_sum(a);
#pragma unroll
      for (int u = 0; u < NE; ++u)
        if (t < M && seg + 16 * u < N) row[seg + 16 * u] = val[u] * inv;
    }
  }
  __syncthreads();
  if (probs_out && !table_ready)  // (a finished table was written where the caller wants it)
    for (int i = tid; i < N; i += nt) probs_out[(size_t)own * N + i] = g[own * NS + i];

  // Eq. (5): s_i = sum_t g_i(h_t).  16 lanes share a column: lane p adds tokens p, p + 16, ... in ascending order
  // and the 16 partial sums are folded through DPP; 64 columns per round.
  int np2 = 1, np2_log = 0;
  while (np2 < N) np2 <<= 1, ++np2_log;
  const int parts = nt >> np2_log;  // N <= 256: at least 4
  const int ci = tid & (np2 - 1), cp = tid >> np2_log;
  if (ext_shortlist == nullptr || scores_out != nullptr) {
    for (int c0 = 0; c0 < N; c0 += nt / 16) {
      const int col = min(c0 + (tid >> 4), N - 1);
      double a = 0.0;
      for (int t = seg; t < M; t += 64) {  // fixed blocks of 4 tokens: the loads go out together
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = t + 16 * u < M ? g[(t + 16 * u) * NS + col] : 0.0;
#pragma unroll
        for (int u = 0; u < 4; ++u) a += v[u];  // rows past the end add +0.0, which leaves the sum unchanged
      }
      a = row16_sum(a);
      if (seg == 0 && c0 + (tid >> 4) < N) s[col] = a;
    }
    __syncthreads();
  }
  // Section 3.2: the B highest aggregate scores, ties to the lowest id - or the caller's shortlist
  if (ext_shortlist == nullptr) {
    const int per = (N + parts - 1) / parts;
    if (ci < N) {
      const double vi = s[ci];
      const int j1 = min(N, (cp + 1) * per);
      int c = 0;
      for (int j = cp * per; j < j1; j += 4) {
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = s[min(j + u, N - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) c += (j + u < j1 && ranks_before(v[u], j + u, vi, ci)) ? 1 : 0;
      }
      if (c) atomicAdd(&rank[ci], c);
    }
    for (int r = tid; r < B; r += nt) S[r] = -1;  // NaN scores: several experts count rank 0, slots stay unfilled
    __syncthreads();
    if (tid < N && rank[tid] < B) {
      S[rank[tid]] = tid;
      pos[tid] = rank[tid];
      inS[tid] = 1;
    }
  } else {
    for (int r = tid; r < B; r += nt) {
      const int e = ext_shortlist[r];
      S[r] = e;
      if ((uint32_t)e < (uint32_t)N) {  // ids outside [0, N) are ignored
        inS[e] = 1;
        atomicMin(&pos[e], r);  // an expert named twice counts at its first rank
      }
    }
  }
  for (int j = tid; j < k; j += nt) sel[j] = -1;
  __syncthreads();
  for (int i = tid; i < N; i += nt) rank[i] = 0;  // reused for this token's candidate ranks below
  // a token's candidates: all experts under truncation (Eq. (7) restricts the natural top-k afterwards), the
  // shortlist in rank order under substitution (Eq. (8)); -1 marks an entry of an external shortlist that is out of
  // range or a repeat, and the padding up to a multiple of 64
  const bool truncate = policy == MOESPEC_TRUNCATE;
  const int n_cand = truncate ? N : B;
  const int n_cand_pad = (n_cand + kWave - 1) & ~(kWave - 1);
  for (int x = tid; x < n_cand_pad; x += nt) {
    int j = -1;
    if (x < n_cand) {
      j = truncate ? x : S[x];
      if (!truncate && !((uint32_t)j < (uint32_t)N && pos[j] == x)) j = -1;
    }
    cand[x] = j;
  }
  // copies for the caller and for the expert passes, written by the last workgroup (on trees of more tokens than
  // shortlisted experts it has no pair list to build)
  if (own == (int)gridDim.x - 1) {
    for (int i = tid; i < N; i += nt) {
      if (scores_out) scores_out[i] = s[i];
      if (seg_expert && inS[i]) {  // position of expert i among the shortlisted experts in ascending id
        int at = 0;
        for (int j = 0; j < i; ++j) at += inS[j];
        seg_expert[at] = i;
      }
    }
    if (tid < B) {
      int n_member = 0;  // < B only if an external shortlist repeats or misnames an expert
      if (seg_expert)
        for (int j = 0; j < N; ++j) n_member += inS[j];
      for (int r = tid; r < B; r += nt) {
        if (seg_expert && r >= n_member) seg_expert[r] = -1;
        budget_ids[r] = S[r];
      }
    }
  }
  __syncthreads();

  // "x goes before y" in a ranking by (probability descending, id ascending), without short-circuit evaluation
  // (which would turn into divergent control flow)
  auto before = [](double vx, int jx, double vy, int jy) { return (vx > vy) | ((vx == vy) & (jx < jy)); };

  // This token's restricted routing.  Eq. (7) keeps the natural top-k slots that fall inside S with their weights
  // unchanged; Eq. (8) takes the top-k inside S and weights over that selection.  A candidate's rank is the number
  // of candidates that go before it; rank r < k fills slot r.  Thread (x, p): candidate x against the p-th share
  // of the rivals.
  int cand_j = -1;
  {
    const double *grow = g + own * NS;
    int cp2 = 64, cp2_log = 6;  // candidates rounded up to a power of two, at least one wave
    while (cp2 < n_cand) cp2 <<= 1, ++cp2_log;
    const int rparts = nt >> cp2_log, x = tid & (cp2 - 1), p = tid >> cp2_log;
    const int rper = (n_cand + rparts - 1) / rparts;
    const int j = x < n_cand_pad ? cand[x] : -1;
    const double v = grow[j < 0 ? 0 : j];
    const int y1 = min(n_cand, (p + 1) * rper);
    int c = 0;
    for (int y = p * rper; y < y1; y += 4) {
      int jy[4];
      double vy[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) jy[u] = cand[min(y + u, n_cand_pad - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u) vy[u] = grow[jy[u] < 0 ? 0 : jy[u]];
#pragma unroll
      for (int u = 0; u < 4; ++u) c += (int)((y + u < y1) & (jy[u] >= 0) & before(vy[u], jy[u], v, j));
    }
    if (c && j >= 0) atomicAdd(&rank[x], c);  // rank[] is zero again here; j >= 0 implies x < n_cand <= N
    cand_j = j;
  }
  // the two remaining steps of the token's routing wait for one barrier each; they ride on the barriers of the first
  // pair-list round below when this workgroup has one
  auto token_fill_slots = [&]() {
    if (tid < n_cand && cand_j >= 0 && rank[tid] < k) sel[rank[tid]] = cand_j;
  };
  auto token_write = [&]() {
    if (tid < k) {
      const double *grow = g + own * NS;
      double denom = 0.0;  // over the selected set in slot order (before any slot is dropped: Eq. (7))
      for (int sl = 0; sl < k; ++sl) {
        const int e = sel[sl];
        denom += e >= 0 ? grow[e] : 0.0;
      }
      const int e = sel[tid];
      const bool keep = e >= 0 && inS[e] != 0;  // an unfilled slot (NaN scores) is dropped
      const double w = keep ? (renorm ? grow[e] / denom : grow[e]) : 0.0;
      tok_ids[(size_t)own * k + tid] = keep ? e : -1;
      tok_w[(size_t)own * k + tid] = (float)w;
    }
  };
  bool token_done = false;

  // Pair lists of the shortlist ranks own, own + M, ...: token t is routed to expert e = S[r] iff e ranks among the
  // first k of t's candidates; its rank is the slot.  16 lanes share a token and split its rivals; 64 tokens per
  // round; the routed tokens of a round are compacted in token order with one ballot per wave.
  for (int r = own; r < B; r += gridDim.x) {
    const int e = S[r];
    const bool real = (uint32_t)e < (uint32_t)N && pos[e] == r;  // not a repeat, not out of range
    int base = 0;
    for (int t0 = 0; t0 < M; t0 += nt / 16) {
      const int t = min(t0 + (tid >> 4), M - 1);
      const double *row = g + t * NS;
      const double ge = row[real ? e : 0];
      int c = 0;
      for (int y = seg; y < n_cand; y += 64) {  // rivals seg, seg + 16, ... four at a time
        int jy[4];
        double vy[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) jy[u] = cand[min(y + 16 * u, n_cand_pad - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) vy[u] = row[jy[u] < 0 ? 0 : jy[u]];
#pragma unroll
        for (int u = 0; u < 4; ++u) c += (int)((y + 16 * u < n_cand) & (jy[u] >= 0) & before(vy[u], jy[u], ge, e));
      }
      c = row16_sum(c);
      const bool routed = real & (t0 + (tid >> 4) < M) & (seg == 0) & (c < k) & (ge == ge);  // NaN ranks nowhere
      const unsigned long long mask = __ballot(routed);
      __syncthreads();  // the wave counts of the previous round have been read (and the rank counts are complete)
      if (!token_done) token_fill_slots();
      if (lane == 0) red[wave] = (double)__popcll(mask);
      __syncthreads();
      if (!token_done) token_write();
      token_done = true;
      int at = base, total = 0;
#pragma unroll
      for (int w = 0; w < nt / kWave; ++w) {
        const int cw = (int)red[w];
        at += w < wave ? cw : 0;
        total += cw;
      }
      at += __popcll(mask & ((1ull << lane) - 1ull));
      if (routed) lists[(size_t)r * list_stride + at] = t * k + c;
      base += total;
    }
    if (tid == 0) list_count[r] = base;
  }
  if (!token_done) {  // a workgroup without a pair list
    __syncthreads();
    token_fill_slots();
    __syncthreads();
    token_write();
  }
}

// seg_expert / seg_off / perm / n_loaded from the pair lists (only when a caller asks for those arrays):
// segments in ascending expert id, each list copied in order.  One workgroup; N <= 256.
__global__ __launch_bounds__(256) void lists_to_segments_kernel(const int32_t *__restrict__ budget_ids,
                                                                const int32_t *__restrict__ list_count,
                                                                const int32_t *__restrict__ lists, int list_stride,
                                                                int B, int N, int n_pairs,
                                                                int32_t *__restrict__ seg_off,
                                                                int32_t *__restrict__ perm,
                                                                int32_t *__restrict__ n_loaded) {
  __shared__ int32_t rank_of[kSelfMaxExperts];  // expert -> first shortlist rank, or -1
  __shared__ int32_t seg_rank[kSelfMaxExperts];  // segment (ascending expert id) -> shortlist rank
  __shared__ int32_t off[kSelfMaxExperts + 1];
  __shared__ int32_t n_member;
  const int tid = threadIdx.x;
  for (int i = tid; i < N; i += blockDim.x) rank_of[i] = 0x7fffffff;
  __syncthreads();
  for (int r = tid; r < B; r += blockDim.x)
    if ((uint32_t)budget_ids[r] < (uint32_t)N) atomicMin(&rank_of[budget_ids[r]], r);
  __syncthreads();
  for (int i = tid; i < N; i += blockDim.x)
    if (rank_of[i] != 0x7fffffff) {
      int at = 0;
      for (int j = 0; j < i; ++j) at += rank_of[j] != 0x7fffffff;
      seg_rank[at] = rank_of[i];
    }
  if (tid == 0) {
    int n = 0;
    for (int j = 0; j < N; ++j) n += rank_of[j] != 0x7fffffff;
    n_member = n;
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0, loaded = 0;
    for (int sg = 0; sg < B; ++sg) {
      off[sg] = run;
      const int c = sg < n_member ? list_count[seg_rank[sg]] : 0;
      run += c;
      loaded += c > 0;
    }
    off[B] = run;
    if (n_loaded) *n_loaded = loaded;
  }
  __syncthreads();
  if (seg_off)
    for (int sg = tid; sg <= B; sg += blockDim.x) seg_off[sg] = off[sg];
  if (perm) {
    for (int sg = 0; sg < n_member; ++sg) {
      const int r = seg_rank[sg], c = off[sg + 1] - off[sg];
      for (int p = tid; p < c; p += blockDim.x) perm[off[sg] + p] = lists[(size_t)r * list_stride + p];
    }
    for (int p = off[B] + tid; p < n_pairs; p += blockDim.x) perm[p] = -1;
  }
}

// The fused prologue covers bf16 layers whose M x N table of doubles fits the LDS of one workgroup beside the
// selection scratch, with at most kSelfMaxExperts experts (one thread per shortlist rank in the expert passes).
bool fused_prologue_ok(const moespec_desc &ds, int M) {
  if (ds.dtype != MOESPEC_BF16 || ds.n_experts > kSelfMaxExperts || M > kSelfMaxTokens) return false;
  return prologue_lds(M, ds.n_experts, ds.top_k, ds.n_experts).total <= 160 * 1024;
}

// Slices of the hidden dimension (1, 2, 4 or 8): more slices spread the matrix work over more compute units
// (a wave issues one fp64 matrix instruction per 64 cycles), but the consumer re-reads one partial table per
// slice: every workgroup of the fused kernel the whole table (whole_table), the row-wise gate kernel one row.
// Picks the count with the smallest estimated sum of the two (rates measured on MI355X: 2.4 GHz, about 150 GB/s
// from L2 into one compute unit).
int logit_slices(const moespec_desc &ds, int M, bool whole_table) {
  const double tiles = ((M + 15) / 16) * ((ds.n_experts + 15) / 16), n_blocks = ds.d / 32;
  int best = 1;
  double best_us = 1e30;
  for (int q = 1; q <= kMaxLogitSlices; q *= 2) {
    if (q > 1 && n_blocks < 2.0 * q * kLogitWaves) break;  // at least two 32-element blocks per wave
    const double waves_per_simd = tiles * q * kLogitWaves / 1024.0;  // 256 compute units x 4 SIMDs
    const double mfma_us = (n_blocks / (q * kLogitWaves)) * 8 * 64 / 2400.0 * (waves_per_simd > 1 ? waves_per_simd : 1);
    const double read_us = q * 8.0 * (whole_table ? M : 1) * ds.n_experts / 150e3;
    if (mfma_us + read_us < best_us) {
      best_us = mfma_us + read_us;
      best = q;
    }
  }
  return best;
}

// Stage 1 alone for bf16 layers whose table does not fit the fused kernel's LDS: matrix-core projection, then the
// row-wise gate; also clears n_zero counters for the staged budget kernel.
bool mfma_route_ok(const moespec_desc &ds, int M) {
  return ds.dtype == MOESPEC_BF16 && ds.n_experts <= kSelfMaxExperts && M <= kSelfMaxTokens;
}
hipError_t launch_mfma_route(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, double *partial,
                             double *probs, int32_t *zero_words, int n_zero, hipStream_t st) {
  const int N = ds.n_experts, q = logit_slices(ds, M, false), sig = ds.gate == MOESPEC_GATE_SIGMOID ? 1 : 0;
  dim3 grid(((M + 15) / 16) * ((N + 15) / 16), q);
  logits_mfma_kernel<<<grid, kLogitWaves * kWave, 0, st>>>(static_cast<const uint16_t *>(h),
                                                          static_cast<const uint16_t *>(wt.w_router), M, N, ds.d, q,
                                                          partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  switch (q) {
    case 1: softmax_rows_kernel<1><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, zero_words, n_zero); break;
    case 2: softmax_rows_kernel<2><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, zero_words, n_zero); break;
    case 4: softmax_rows_kernel<4><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, zero_words, n_zero); break;
    default: softmax_rows_kernel<8><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, zero_words, n_zero); break;
  }
  return hipGetLastError();
}

hipError_t launch_fused_prologue(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, int B,
                                 int policy, const int32_t *ext_shortlist, double *partial, double *probs_ws,
                                 double *probs_out,
                                 double *scores_out, int32_t *budget_ids, int32_t *seg_expert, int32_t *tok_ids,
                                 float *tok_w, int32_t *list_count, int32_t *lists, int list_stride,
                                 int32_t *seg_off, int32_t *perm, int32_t *n_loaded, hipStream_t st) {
  const int N = ds.n_experts, k = ds.top_k;
  // Large tables: the routing probabilities are finished row by row in a launch of their own and the last kernel
  // only loads them; small tables: every workgroup of the last kernel rebuilds the table itself.
  const bool split = (long long)M * N > kSplitSoftmaxAbove;
  const int q = logit_slices(ds, M, !split);
  dim3 grid(((M + 15) / 16) * ((N + 15) / 16), q);
  logits_mfma_kernel<<<grid, kLogitWaves * kWave, 0, st>>>(static_cast<const uint16_t *>(h),
                                                          static_cast<const uint16_t *>(wt.w_router), M, N, ds.d, q,
                                                          partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t smem = prologue_lds(M, N, k, B).total;
  const int sig = ds.gate == MOESPEC_GATE_SIGMOID ? 1 : 0;
  const double *table = partial;
  const float *table_bias = wt.b_router;
  int slices = q;
  if (split) {
    double *probs = probs_out ? probs_out : probs_ws;
    switch (q) {
      case 1: softmax_rows_kernel<1><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, nullptr, 0); break;
      case 2: softmax_rows_kernel<2><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, nullptr, 0); break;
      case 4: softmax_rows_kernel<4><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, nullptr, 0); break;
      default: softmax_rows_kernel<8><<<M, kWave, 0, st>>>(partial, wt.b_router, M, N, sig, probs, nullptr, 0); break;
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    table = probs;
    table_bias = nullptr;
    slices = 1;
  }
  // instantiation for (slices, elements of a table row per lane = ceil(N / 16) rounded up to a power of two)
  auto run = [&](auto kern) -> hipError_t {
    if (smem > 64 * 1024) {  // beyond the default limit of a launch
      hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (err != hipSuccess) return err;
    }
    kern<<<M, kPrologueThreads, smem, st>>>(table, table_bias, M, N, k, B, policy, ds.renorm, sig, ext_shortlist,
                                            probs_out, scores_out, budget_ids, seg_expert, tok_ids, tok_w, list_count,
                                            lists, list_stride, split ? 1 : 0);
    return hipGetLastError();
  };
  const int ne = (N + 15) / 16;
#define MOESPEC_RB_NE(QQ)                                                                        \
  (ne <= 1 ? run(route_budget_kernel<QQ, 1>) : ne <= 2 ? run(route_budget_kernel<QQ, 2>)         \
   : ne <= 4 ? run(route_budget_kernel<QQ, 4>) : ne <= 8 ? run(route_budget_kernel<QQ, 8>)       \
                                                         : run(route_budget_kernel<QQ, 16>))
  e = slices == 1 ? MOESPEC_RB_NE(1) : slices == 2 ? MOESPEC_RB_NE(2) : slices == 4 ? MOESPEC_RB_NE(4) : MOESPEC_RB_NE(8);
#undef MOESPEC_RB_NE
  if (e != hipSuccess) return e;
  if (seg_off || perm || n_loaded) {
    lists_to_segments_kernel<<<1, 256, 0, st>>>(budget_ids, list_count, lists, list_stride, B, N, M * k, seg_off, perm,
                                                n_loaded);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace moespec
