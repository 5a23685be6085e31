// Shared device/host helpers of the moespec kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moespec.h"

namespace moespec {

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// bfloat16 bit pattern <-> float.  Storage tensors hold raw uint16 patterns.
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// Round-to-nearest-even; NaN stays NaN.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
  static __device__ __forceinline__ float stored(float v) { return v; }  // the value a store of v leaves behind
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t *p, float v) { *p = float_to_bf16_bits(v); }
  static __device__ __forceinline__ float stored(float v) { return bf16_bits_to_float(float_to_bf16_bits(v)); }
};

// Ranking order used by every selection: larger value first, then lower index.
__device__ __forceinline__ bool ranks_before(double vj, int j, double vi, int i) {
  return vj > vi || (vj == vi && j < i);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kWave);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kWave);
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v = fmax(v, __shfl_xor(v, s, kWave));
  return v;
}

// x = row / sqrt(mean of squares) in fp32 for one row held by a workgroup of kRmsThreads threads: thread i holds the
// elements (c * kRmsThreads + i) * 4 .. + 3 of chunk c = 0 .. kRmsChunks-1 in v[c][0..3] (zeros past the row end;
// the hidden size is at most 8192).  Squares are
// added chunk by chunk and element by element per thread, the per-thread sums pairwise through LDS (a fixed tree):
// the result depends on the values alone.  Used by rms_scale_kernel and by the combine that also writes the next
// layer's input, which therefore agree bit for bit.  part: kRmsThreads floats of LDS.  Synchronises.
constexpr int kRmsThreads = 1024, kRmsChunks = 2;
__device__ inline float rms_scale_of_row(const float (&v)[kRmsChunks][4], int d, float *part) {
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < kRmsChunks; ++c)
#pragma unroll
    for (int i = 0; i < 4; ++i) ss = fmaf(v[c][i], v[c][i], ss);
  part[threadIdx.x] = ss;
  __syncthreads();
  for (int s = kRmsThreads / 2; s >= 1; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  return 1.0f / sqrtf(part[0] / (float)d);
}

// Rank-count selection of the k best of v[0..n) restricted to candidates with member[i] != 0
// (member == nullptr: all).  sel[r] receives the index with rank r < k.  Equivalent to sorting by
// (value descending, index ascending) and keeping the first k.  v, member, sel and the scratch
// rank[n] live in LDS.  Called by every thread of the workgroup (it synchronises); the caller
// synchronises again before reading sel.  The n x n comparisons are spread over the whole workgroup:
// thread (i, part) counts the rivals of candidate i inside its part of the index range and adds its
// count to rank[i] with an integer LDS atomic (order-independent, hence deterministic).
// Every slot of sel is first set to -1: when a value is NaN no comparison holds, several candidates then
// count rank 0 and some slots are never claimed; those stay -1 (an unfilled slot) instead of stale LDS.
__device__ inline void select_topk(const double *v, const uint8_t *member, int n, int k, int32_t *sel, int32_t *rank) {
  const int nt = blockDim.x, tid = threadIdx.x;
  int np2 = 1;
  while (np2 < n) np2 <<= 1;
  for (int x = tid; x < n; x += nt) rank[x] = 0;
  for (int x = tid; x < k; x += nt) sel[x] = -1;
  __syncthreads();
  const int parts = np2 <= nt ? nt / np2 : 1;
  const int chunk = (n + parts - 1) / parts;
  for (int i = np2 <= nt ? (tid & (np2 - 1)) : tid; i < n; i += np2 <= nt ? n : nt) {
    const int part = np2 <= nt ? tid / np2 : 0;
    if (member && !member[i]) continue;
    const int j0 = part * chunk, j1 = min(n, j0 + chunk);
    const double vi = v[i];
    int cnt = 0;
    if (member) {
#pragma unroll 4
      for (int j = j0; j < j1; ++j) cnt += (member[j] && ranks_before(v[j], j, vi, i)) ? 1 : 0;
    } else {
#pragma unroll 4
      for (int j = j0; j < j1; ++j) cnt += ranks_before(v[j], j, vi, i) ? 1 : 0;
    }
    if (cnt) atomicAdd(&rank[i], cnt);
  }
  __syncthreads();
  for (int x = tid; x < n; x += nt)
    if ((!member || member[x]) && rank[x] < k) sel[rank[x]] = x;
}

// Mixing weights of the slots sel[0..k): raw g or g / sum over the slots (summed in slot order).
// An unfilled slot (sel < 0) gets weight 0.  Called by every thread (it synchronises); denom is one
// LDS double of scratch.
__device__ inline void mixing_weights(const double *g, const int32_t *sel, int k, int renorm, double *w,
                                      double *denom) {
  if (threadIdx.x == 0 && renorm) {
    double acc = 0.0;
    for (int s = 0; s < k; ++s)
      if (sel[s] >= 0) acc += g[sel[s]];
    *denom = acc;
  }
  __syncthreads();
  for (int s = threadIdx.x; s < k; s += blockDim.x)
    w[s] = sel[s] < 0 ? 0.0 : (renorm ? g[sel[s]] / *denom : g[sel[s]]);
}

constexpr int kMaxDownSplits = 4;  // K-split copies of the per-pair outputs y

// The LDS-tiled expert passes take up to 128 pairs (8 token tiles of 16) per walk over an expert's weights.
// A longer segment is cut into ceil(c / 128) pieces of (almost) equal size, each a work item of its own, so
// that its walks run side by side on different compute units instead of one after the other.
constexpr int kPiecePairs = 128;
__host__ __device__ inline int piece_count(int c) { return (c + kPiecePairs - 1) / kPiecePairs; }
// Upper bound on the pieces of n_seg well-formed segments (disjoint, at most one pair per token each).
inline int items_capacity(int n_seg, int64_t M, int64_t k) {
  const int64_t a = (int64_t)n_seg * ((M + kPiecePairs - 1) / kPiecePairs), b = n_seg + M * k / kPiecePairs;
  return (int)(a < b ? a : b);
}
constexpr int kMaxLogitSlices = 8;    // slices of the hidden dimension in the fused prologue's router projection
constexpr int kSelfMaxTokens = 1024;  // largest tree for which the expert passes derive their segments themselves
constexpr int kSelfMaxExperts = 256;  // ... and the largest shortlist

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace carve-up shared by all entry points (host).
struct Workspace {
  double *probs;      // [M, N]
  double *scores;     // [N]
  int32_t *budget_ids;  // [N]
  int32_t *tok_ids;   // [M, k]
  float *tok_w;       // [M, k]
  int32_t *seg_expert;  // [N]
  int32_t *seg_off;   // [N + 1]
  int32_t *perm;      // [M * k]
  int4 *items;        // [items_capacity(N, M, k) + 1] count, then (segment, expert, offset, size) of every piece
  int4 *pub_items;    // [as items] the same table as published by a self-segmenting gate/up pass
  int32_t *pub_lists; // [work items of that mode, kPiecePairs] its pair lists
  int32_t *n_loaded;  // [1]
  int32_t *done;      // [1 + N] ticket counter of the budget stage, then surviving pairs per shortlist rank
  void *act;          // [M * k, F] dtype
  float *y;           // [kMaxDownSplits][M * k, d]
  double *gram;       // [N, N + 3] scratch of the oracle ranking
  double *partial;    // [kMaxLogitSlices, M, N] partial router projections of the fused prologue
  int32_t *list_count;  // [N] pairs per shortlist rank (fused prologue)
  int32_t *lists;     // [N, M] their pair lists (only for shapes the fused prologue covers)
  void *xnorm;        // [M, d] dtype: the scaled layer input of the layer stack
  size_t bytes;
};

inline Workspace carve_workspace(const moespec_desc &ds, int64_t M, void *base) {
  Workspace w;
  size_t off = 0;
  char *b = static_cast<char *>(base);
  auto take = [&](size_t n) {
    void *p = b ? b + off : nullptr;
    off += align_up(n, 256);
    return p;
  };
  const int64_t N = ds.n_experts, k = ds.top_k, F = ds.d_ff, d = ds.d;
  const size_t es = ds.dtype == MOESPEC_BF16 ? 2 : 4;
  w.probs = static_cast<double *>(take(sizeof(double) * M * N));
  w.scores = static_cast<double *>(take(sizeof(double) * N));
  w.budget_ids = static_cast<int32_t *>(take(sizeof(int32_t) * N));
  w.tok_ids = static_cast<int32_t *>(take(sizeof(int32_t) * M * k));
  w.tok_w = static_cast<float *>(take(sizeof(float) * M * k));
  w.seg_expert = static_cast<int32_t *>(take(sizeof(int32_t) * N));
  w.seg_off = static_cast<int32_t *>(take(sizeof(int32_t) * (N + 1)));
  w.perm = static_cast<int32_t *>(take(sizeof(int32_t) * M * k));
  w.items = static_cast<int4 *>(take(sizeof(int4) * (items_capacity((int)N, M, k) + 1)));
  w.pub_items = static_cast<int4 *>(take(sizeof(int4) * (items_capacity((int)N, M, k) + 1)));
  w.pub_lists = static_cast<int32_t *>(
      take(sizeof(int32_t) * kPiecePairs *
           items_capacity((int)(N < kSelfMaxExperts ? N : kSelfMaxExperts), M < kSelfMaxTokens ? M : kSelfMaxTokens, k)));
  w.n_loaded = static_cast<int32_t *>(take(sizeof(int32_t)));
  w.done = static_cast<int32_t *>(take(sizeof(int32_t) * (1 + N)));
  w.act = take(es * M * k * F);
  w.y = static_cast<float *>(take(sizeof(float) * kMaxDownSplits * M * k * d));
  w.gram = static_cast<double *>(take(sizeof(double) * N * (N + 3)));
  const bool small = N <= kSelfMaxExperts && M <= kSelfMaxTokens;
  w.partial = static_cast<double *>(take(small ? sizeof(double) * kMaxLogitSlices * M * N : 0));
  w.list_count = static_cast<int32_t *>(take(sizeof(int32_t) * N));
  w.lists = static_cast<int32_t *>(take(small ? sizeof(int32_t) * N * M : 0));
  w.xnorm = take(es * M * d);
  w.bytes = off;
  return w;
}

// Launchers (defined in the .hip files).  Each returns hipGetLastError() after its launches.
// zero_words (may be NULL): n_zero int32 that the route stage sets to 0 (the counters of the budget stage).
hipError_t launch_route(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, double *probs,
                        int32_t *topk_ids, float *topk_w, int32_t *zero_words, int n_zero, hipStream_t st);
// done: [1 + N] counters (ticket, then the number of surviving pairs of the expert at each shortlist
// rank), zero at launch or zeroed first (done_is_zero == false).  budget_ids must not be NULL.
// want_segments == false skips seg_off / perm / n_loaded / items: the expert passes can then only run in
// the mode that derives its segments from done + 1, budget_ids and tok_ids.  score_scratch: N doubles.
hipError_t launch_budget(const moespec_desc &ds, const double *probs, int M, int B, int policy,
                         const int32_t *ext_shortlist, double *scores, int32_t *budget_ids, int32_t *tok_ids,
                         float *tok_w, int32_t *seg_expert, int32_t *seg_off, int32_t *perm, int32_t *n_loaded,
                         int4 *items, int32_t *done, bool done_is_zero, bool want_segments, double *score_scratch,
                         hipStream_t st);
// items: table of the work items ([items_capacity(n_seg, M, k) + 1] int4 of scratch: the non-empty segments,
// those above kPiecePairs pairs cut into pieces); items_ready says that the budget stage has already filled
// it from the same segment arrays, otherwise it is built first.
// rank_count, shortlist (may be NULL): the shortlist in rank order ([n_seg]) and the surviving pairs of each
// of its experts, from the budget stage; when given and the shape allows (expert_ffn_self_segmenting),
// every workgroup derives its segment from them and tok_ids itself, and seg_expert / seg_off / perm /
// items are not read.  pub_items (like items) and pub_lists ([work items, kPiecePairs] int32) are scratch in
// which the gate/up pass of that mode leaves its work items for the down pass (NULL: the down pass derives
// them again).
// trace (may be NULL): 3 events recorded after the gate/up pass, the down pass and the combine.
// x_next (may be NULL): [M, d] dtype; the combine then also writes out scaled row by row to unit root-mean-square,
// the next layer's input in a stack (d <= 8192).
hipError_t launch_expert_ffn(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, int n_seg,
                             const int32_t *seg_expert, const int32_t *seg_off, const int32_t *perm,
                             const int32_t *tok_ids, const float *tok_w, const void *residual, void *out, void *act,
                             float *y, int4 *items, bool items_ready, const int32_t *rank_count,
                             const int32_t *shortlist, int4 *pub_items, int32_t *pub_lists, hipStream_t st,
                             void *const *trace = nullptr, const int32_t *lists = nullptr, int list_stride = 0,
                             void *x_next = nullptr);
// The fused prologue of the layer call (prologue.hip): router projection on the fp64 matrix cores, then one
// launch that leaves the shortlist (budget_ids), the restricted routing (tok_ids, tok_w) and, for every shortlist
// rank r, the pairs routed to its expert (list_count[r]; lists[r * list_stride ..], flat ids t * k + slot, tokens
// ascending).  partial: [logit_slices, M, N] doubles of scratch.  probs_out, scores_out, seg_expert, seg_off,
// perm, n_loaded are optional copies for the caller (the last three cost one more small launch).
bool fused_prologue_ok(const moespec_desc &ds, int M);
// Stage 1 on the matrix cores for bf16 layers of up to kSelfMaxExperts experts and kSelfMaxTokens tokens, whatever the
// size of the table: probs [M, N] out, partial as above, zero_words cleared like launch_route does.
bool mfma_route_ok(const moespec_desc &ds, int M);
hipError_t launch_mfma_route(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, double *partial,
                             double *probs, int32_t *zero_words, int n_zero, hipStream_t st);
int logit_slices(const moespec_desc &ds, int M, bool whole_table);
hipError_t launch_fused_prologue(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, int B,
                                 int policy, const int32_t *ext_shortlist, double *partial, double *probs_ws,
                                 double *probs_out,
                                 double *scores_out, int32_t *budget_ids, int32_t *seg_expert, int32_t *tok_ids,
                                 float *tok_w, int32_t *list_count, int32_t *lists, int list_stride,
                                 int32_t *seg_off, int32_t *perm, int32_t *n_loaded, hipStream_t st);
bool expert_ffn_self_segmenting(const moespec_desc &ds, int M);
// Number of K-split copies of y that launch_expert_ffn writes for n_seg segments; out == NULL there skips
// the combine and leaves the per-pair expert outputs in y.
int down_splits(const moespec_desc &ds, int n_seg);
// Analysis kernels (analysis.hip).  part: 2 M doubles of scratch.
hipError_t launch_calibration_count(const int32_t *topk_ids, int M, int k, int N, int64_t *counts, hipStream_t st);
hipError_t launch_static_shortlist(const int64_t *counts, int N, int B, int32_t *shortlist, hipStream_t st);
hipError_t launch_coverage_curve(const double *scores, int N, double *curve, hipStream_t st);
// Greedy oracle ranking on the per-pair outputs y (splits copies, split_stride floats apart) of a run with
// natural routing (tok_ids / tok_w = natural top-k).  pair_gram: M k k doubles, gram: N N + 3 N doubles of scratch.
hipError_t launch_oracle_ranking(const moespec_desc &ds, const float *y, int splits, size_t split_stride,
                                 const int32_t *tok_ids, const float *tok_w, int M, int B, double *pair_gram,
                                 double *gram, int32_t *ranking, double *err, hipStream_t st);
// x[t] = h[t] / rms(h[t]) (stack.hip); x may alias h.
hipError_t launch_rms_scale(const moespec_desc &ds, const void *h, int M, void *x, hipStream_t st);
hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *checksum, hipStream_t st);
hipError_t launch_reconstruction_error(const moespec_desc &ds, const void *out_budgeted, const void *out_full, int M,
                                       double *part, double *err, hipStream_t st);

}  // namespace moespec
