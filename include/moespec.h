/*
 * moespec.h - C ABI of the budgeted MoE-layer forward that verifies an M-token draft tree
 * (MoE-Spec expert budgeting), implemented as HIP kernels for gfx950 (MI355X).
 *
 * The calls take the inputs and produce the output of Algorithm 1 (the M hidden rows of the draft tree, the
 * budget and the coverage policy in; one MoE output row per token out), split at its three stages:
 *
 *   moespec_route          Eq. (1) router softmax, Section 2.1 per-token top-k and mixing weights
 *   moespec_budget         Eq. (5) per-expert aggregation, top-B shortlist (Section 3.2), Eq. (7)/(8)
 *                          restriction of every token's routing (Section 3.3), grouping into per-expert
 *                          segments
 *   moespec_expert_ffn     the expert networks of Eq. (2)/(7)/(8) run over the loaded experts only,
 *                          and the weighted combine
 *   moespec_layer_forward  all of the above in one call (Algorithm 1)
 *
 * and, around that path, the static ranking of Eq. (4) (moespec_calibration_count,
 * moespec_static_shortlist: a shortlist fixed from calibration data, passed in as ext_shortlist)
 * the Oracle ranking of Eq. (6) (moespec_oracle_ranking, an upper bound for analysis) and two analysis
 * quantities of Section 4 (moespec_coverage_curve, moespec_reconstruction_error).
 *
 * Conventions (all calls)
 *   Pointers  Every buffer pointer is a DEVICE pointer unless it is a descriptor struct
 *             (moespec_desc, moespec_weights are read on the host).  All tensors are row-major,
 *             contiguous and 16-byte aligned.  "dtype" tensors hold float (MOESPEC_F32) or bfloat16
 *             bit patterns (MOESPEC_BF16).
 *   Ownership The caller owns every buffer, workspace included.  The library allocates nothing,
 *             frees nothing and keeps no pointer after a call returns; it holds no global state.
 *   Execution A call validates its arguments on the host, enqueues kernels on `hip_stream`
 *             (a hipStream_t passed as void*; NULL = the default stream) and returns without
 *             synchronising.  Nothing is copied to the host; data-dependent quantities (the number
 *             of loaded experts, segment sizes) stay on the device.
 *   Sizes     1 <= M <= 65535 tree tokens per call, and M * top_k * max(d, d_ff) < 2^31
 *             (MOESPEC_ERR_UNSUPPORTED_SHAPE beyond that).
 *   Workspace `ws` must hold at least moespec_workspace_bytes(desc, M) bytes, 256-byte aligned.
 *             Its contents are scratch: undefined before and after a call.  Calls that share a
 *             workspace must be ordered on one stream.
 *   Errors    Every call returns a moespec_status.  Argument errors are detected before any launch
 *             and leave all buffers untouched.  HIP launch failures are reported as
 *             MOESPEC_ERR_HIP.  Nothing throws or aborts across this boundary.
 *   Decisions Routing probabilities, aggregate scores and every ranking are computed in fp64;
 *             every tie goes to the lowest expert id.  Rankings compare routing probabilities.
 *   Determinism  Same inputs give bit-identical outputs on every call (no floating-point atomics).
 */
#ifndef MOESPEC_H
#define MOESPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOESPEC_OK = 0,
  MOESPEC_ERR_INVALID_ARG = 1,       /* null pointer, size out of range, B < k under substitution, ... */
  MOESPEC_ERR_UNSUPPORTED_SHAPE = 2, /* a shape the kernels do not cover (see moespec_check_desc)     */
  MOESPEC_ERR_WORKSPACE_TOO_SMALL = 3,
  MOESPEC_ERR_HIP = 4                /* a HIP runtime call failed (no device, launch error)           */
} moespec_status;

typedef enum { MOESPEC_F32 = 0, MOESPEC_BF16 = 1 } moespec_dtype;

/* Coverage policy of Section 3.3: Eq. (7) truncation or Eq. (8) substitution. */
typedef enum { MOESPEC_TRUNCATE = 0, MOESPEC_SUBSTITUTE = 1 } moespec_policy;

/* Gate of the router: the softmax over all experts of Eq. (1), or an independent sigmoid per expert
 * (the routing scheme the paper's limitations section names as an open case; T_k, Eq. (5) and
 * Eq. (7)/(8) are applied to the sigmoid scores unchanged). */
typedef enum { MOESPEC_GATE_SOFTMAX = 0, MOESPEC_GATE_SIGMOID = 1 } moespec_gate;

/* Shape of one MoE layer.  Host struct. */
typedef struct {
  int32_t d;         /* hidden size                                                         */
  int32_t n_experts; /* N                                                                   */
  int32_t top_k;     /* k, 1 <= k <= N                                                      */
  int32_t d_ff;      /* expert intermediate size F                                          */
  int32_t dtype;     /* moespec_dtype: storage of h, the weights, residual and out          */
  int32_t renorm;    /* 0: mixing weights are the raw g_i; 1: g_i / sum over the selected   */
                     /* set (which one applies is a property of the model, Section 2.1)     */
  int32_t gate;      /* moespec_gate                                                        */
} moespec_desc;

/* Weights of one MoE layer.  Host struct holding device pointers. */
typedef struct {
  const void  *w_router; /* [N, d]    dtype, row i is the routing vector w_i of Eq. (1)      */
  const float *b_router; /* [N] float or NULL; added to the router projection before softmax */
  const void  *w_gate;   /* [N, F, d] dtype                                                  */
  const void  *w_up;     /* [N, F, d] dtype                                                  */
  const void  *w_down;   /* [N, d, F] dtype;  E_i(x) = w_down_i (silu(w_gate_i x) * w_up_i x) */
} moespec_weights;

/* Library ABI version (bumped on any signature change). */
int32_t moespec_abi_version(void);

/* Human-readable name of a status code; never NULL. */
const char *moespec_status_string(int32_t status);

/*
 * Checks that the kernels cover this layer shape: d and d_ff multiples of 32 (bf16) or 4 (f32),
 * d <= 8192, d_ff <= 2^20, 1 <= top_k <= n_experts <= 1024, top_k <= 64, n_experts * d_ff * d < 2^40, dtype and
 * renorm and gate valid.
 * Returns MOESPEC_OK, MOESPEC_ERR_INVALID_ARG or MOESPEC_ERR_UNSUPPORTED_SHAPE.  Host only.
 */
moespec_status moespec_check_desc(const moespec_desc *desc);

/*
 * Bytes of workspace any call below needs for trees of up to M_max tokens, 1 <= M_max <= 65535
 * (0 on an invalid descriptor or M_max out of range).  The workspace is scratch: its content need
 * not be initialised and is not preserved between calls; calls that share one workspace must not
 * overlap in time.  Host only.
 */
size_t moespec_workspace_bytes(const moespec_desc *desc, int32_t M_max);

/*
 * Stage 1 of Algorithm 1 - Eq. (1) and Section 2.1.
 *   h        [M, d] dtype   in   draft-tree hidden rows
 *   probs    [M, N] double  out  g_i(h_t), softmax over all N experts of w_i . h_t (+ b_i)
 *   topk_ids [M, k] int32   out  T_k(h_t), best first (ties: lowest id)
 *   topk_w   [M, k] float   out  mixing weights of those slots (raw or renormalised over T_k)
 * topk_ids and topk_w may both be NULL.  1 <= M <= 65535.
 */
moespec_status moespec_route(const moespec_desc *desc, const moespec_weights *weights,
                             const void *h, int32_t M,
                             double *probs, int32_t *topk_ids, float *topk_w,
                             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Stages 2-3 of Algorithm 1 without the expert maths - Eq. (5), Section 3.2, Eq. (7)/(8).
 *   probs         [M, N] double in   routing probabilities (as written by moespec_route)
 *   B                           in   expert budget, 1 <= B <= N; substitution needs B >= k
 *   ext_shortlist [B] int32     in   NULL = router-based ranking (Eq. (5)); otherwise B distinct
 *                                    expert ids fixed elsewhere (e.g. the static ranking of Eq. (4)),
 *                                    used as the shortlist S verbatim
 *   scores        [N] double    out  s_i = sum_t g_i(h_t)                      (may be NULL)
 *   budget_ids    [B] int32     out  S in rank order (best first)              (may be NULL)
 *   tok_ids       [M, k] int32  out  restricted routing; -1 marks a dropped slot.  Truncation keeps the
 *                                    natural slot order; substitution lists the top-k inside S best first
 *   tok_w         [M, k] float  out  mixing weights; truncation keeps the weights of the natural top-k
 *                                    unchanged, dropped slots get 0
 *   seg_expert    [B] int32     out  S in ascending expert id
 *   seg_off       [B+1] int32   out  offsets of each expert's segment in perm (empty segments allowed)
 *   perm          [M*k] int32   out  surviving (token, slot) pairs as flat indices t*k+slot, ordered by
 *                                    (expert id, token); entries past seg_off[B] are -1
 *   n_loaded      [1] int32     out  number of non-empty segments = experts loaded (may be NULL)
 */
moespec_status moespec_budget(const moespec_desc *desc, const double *probs, int32_t M, int32_t B,
                              int32_t policy, const int32_t *ext_shortlist,
                              double *scores, int32_t *budget_ids,
                              int32_t *tok_ids, float *tok_w,
                              int32_t *seg_expert, int32_t *seg_off, int32_t *perm, int32_t *n_loaded,
                              void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The expert networks over the loaded experts and the weighted combine - Eq. (2)/(7)/(8).
 * For every segment i with at least one pair, expert seg_expert[i] is applied to the hidden rows of
 * its pairs, streaming that expert's three matrices from memory once; then
 *   out[t] = (residual ? residual[t] : 0) + sum over surviving slots, in slot order, tok_w[t,slot] * E(h_t).
 * A token with no surviving slot gets exactly residual[t] (or 0).
 *   n_seg                       in   number of segments (the B of moespec_budget), 1 <= n_seg <= N
 *   seg_expert, seg_off, perm, tok_ids, tok_w   in   as written by moespec_budget
 *   residual [M, d] dtype       in   NULL or the residual stream to add
 *   out      [M, d] dtype       out
 */
moespec_status moespec_expert_ffn(const moespec_desc *desc, const moespec_weights *weights,
                                  const void *h, int32_t M, int32_t n_seg,
                                  const int32_t *seg_expert, const int32_t *seg_off, const int32_t *perm,
                                  const int32_t *tok_ids, const float *tok_w,
                                  const void *residual, void *out,
                                  void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Algorithm 1 end to end: route, aggregate, shortlist, restrict, experts, combine.
 * B = N is the unbudgeted layer of Eq. (2), which loads the expert union of Eq. (3).
 * The tap pointers (all optional, any may be NULL) receive copies of the intermediates with the
 * shapes documented above: probs [M,N], scores [N], budget_ids [B], tok_ids [M,k], tok_w [M,k],
 * seg_expert [B], seg_off [B+1], perm [M*k], n_loaded [1].  The grouping of the pairs into segments
 * (seg_off, perm, n_loaded) is an extra serial step that small trees only pay when one of those three
 * taps is given: without them the expert passes find their segments themselves.  The output is the
 * same, bit for bit, either way.
 */
typedef struct {
  double  *probs;
  double  *scores;
  int32_t *budget_ids;
  int32_t *tok_ids;
  float   *tok_w;
  int32_t *seg_expert;
  int32_t *seg_off;
  int32_t *perm;
  int32_t *n_loaded;
} moespec_taps;

moespec_status moespec_layer_forward(const moespec_desc *desc, const moespec_weights *weights,
                                     const void *h, int32_t M, int32_t B, int32_t policy,
                                     const int32_t *ext_shortlist,
                                     const void *residual, void *out,
                                     const moespec_taps *taps,
                                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Measurement aid, not part of the method: moespec_layer_forward (no taps) that also records HIP events on the
 * stream at its stage boundaries, so that a benchmark can time the stages of one call without a profiler.
 *   trace_events  HOST array of MOESPEC_TRACE_POINTS hipEvent_t handles created by the caller with timing
 *                 enabled (entries may be NULL): [0] start, [1] after the prologue (router, scores, shortlist,
 *                 restricted routing, pair grouping), [2] after the gate/up pass, [3] after the down pass,
 *                 [4] after the combine.
 * An event interval brackets the launches in it and includes their dispatch latency.
 */
#define MOESPEC_TRACE_POINTS 5
moespec_status moespec_layer_forward_traced(const moespec_desc *desc, const moespec_weights *weights,
                                            const void *h, int32_t M, int32_t B, int32_t policy,
                                            const int32_t *ext_shortlist,
                                            const void *residual, void *out, int32_t *n_loaded,
                                            void *const *trace_events,
                                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * moespec_layer_forward for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results
 * (bit for bit) as moespec_layer_forward without taps, but the scratch memory is a fixed device array inside
 * the library, MOESPEC_STATIC_SCRATCH_BYTES large, instead of a caller-owned workspace.  The call allocates and
 * frees nothing.
 *   Limit     moespec_workspace_bytes(desc, M) must not exceed MOESPEC_STATIC_SCRATCH_BYTES, otherwise
 *             MOESPEC_ERR_WORKSPACE_TOO_SMALL is returned before any launch (the OLMoE-like, 128-expert and
 *             Mixtral-like layer shapes fit up to 127 tree tokens).
 *   Set-up    The first call on a device looks up the array's device address (hipGetSymbolAddress, once per
 *             device, with that device current); make that first call outside any graph capture.
 *             MOESPEC_ERR_HIP if the look-up fails.
 *   Sharing   Every call on one GPU uses that GPU's one array, which keeps whatever the last call left in it
 *             (the kernels clear what they need cleared).  Calls that overlap in time on one GPU - different
 *             streams, different host threads - race on it: order them on one stream.
 * The array occupies MOESPEC_STATIC_SCRATCH_BYTES of every GPU the library is used on until the process ends.
 */
#define MOESPEC_STATIC_SCRATCH_BYTES (48u << 20)
moespec_status moespec_layer_forward_static(const moespec_desc *desc, const moespec_weights *weights,
                                            const void *h, int32_t M, int32_t B, int32_t policy,
                                            const int32_t *ext_shortlist,
                                            const void *residual, void *out, void *hip_stream);

/*
 * The layer stack of the coarse-expert workload: n_layers consecutive MoE layers joined by the residual stream.
 * For l = 0 .. n_layers-1:  x = pre_norm ? rms_scale(h) : h;  h <- h + MoE_S(x) with layer l's weights, every
 * layer being Algorithm 1 as in moespec_layer_forward (Section 3.3 notes that a token without a surviving expert
 * passes through on the residual connection alone).  pre_norm = 1 scales every row of the layer input to unit
 * root-mean-square (moespec_rms_scale) and leaves the residual stream itself unscaled; pre_norm = 0 is the plain
 * recurrence.
 *   layers     HOST array of n_layers moespec_weights (device pointers inside), 1 <= n_layers <= 4096
 *   h          [M, d] dtype  in/out  residual stream, updated in place
 *   budget_ids [n_layers, B] int32 out (may be NULL)  every layer's shortlist in rank order
 *   tok_ids    [n_layers, M, k] int32 out (may be NULL)  every layer's restricted routing
 * All layers share desc, B, policy and the workspace (size rule as for the other calls).
 */
moespec_status moespec_stack_forward(const moespec_desc *desc, const moespec_weights *layers, int32_t n_layers,
                                     void *h, int32_t M, int32_t B, int32_t policy, int32_t pre_norm,
                                     int32_t *budget_ids, int32_t *tok_ids,
                                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * x[t] = h[t] / sqrt(mean_j h[t, j]^2) for every row (fp32 arithmetic, fixed summation order): the input scaling
 * of moespec_stack_forward with pre_norm = 1, exported so that a stack can also be driven layer by layer.
 *   h, x [M, d] dtype (device); x may be the same buffer as h.  No workspace.
 */
moespec_status moespec_rms_scale(const moespec_desc *desc, const void *h, int32_t M, void *x, void *hip_stream);

/*
 * Static ranking - Eq. (4): c_i = number of calibration tokens h with i in T_k(h).
 *   topk_ids [M, k] int32  in     natural top-k ids of a batch of calibration tokens (moespec_route);
 *                                 entries outside [0, N) are ignored
 *   counts   [N] int64     in/out selection frequencies, incremented in place (zero them before the
 *                                 first batch; later batches accumulate)
 * Device pointers; asynchronous on hip_stream; no workspace.
 */
moespec_status moespec_calibration_count(const moespec_desc *desc, const int32_t *topk_ids, int32_t M,
                                         int64_t *counts, void *hip_stream);

/*
 * Static ranking - Eq. (4) and the sentence after it: the B experts with the highest c_i, most
 * frequent first, ties to the lowest id.  The result is what moespec_budget / moespec_layer_forward
 * take as ext_shortlist.
 *   counts [N] int64 in, shortlist [B] int32 out (device), 1 <= B <= N.
 */
moespec_status moespec_static_shortlist(const moespec_desc *desc, const int64_t *counts, int32_t B,
                                        int32_t *shortlist, void *hip_stream);

/*
 * Coverage analysis - Section 4.6: curve[B-1] = share of the tree's routing probability captured by
 * the B highest-scoring experts, B = 1..N, from the aggregate scores of Eq. (5).
 *   scores [N] double in (the scores tap), curve [N] double out (device).
 */
moespec_status moespec_coverage_curve(const moespec_desc *desc, const double *scores, double *curve,
                                      void *hip_stream);

/*
 * Reconstruction error - Section 4.5: ||O_S - O*||^2 / ||O*||^2 over all M tokens, O_S the budgeted
 * layer output and O* the full output of Eq. (2) (a layer call with B = N), accumulated in fp64.
 *   out_budgeted, out_full [M, d] dtype in;  err [3] double out: ratio, numerator, denominator.
 * Uses the workspace as scratch (same size rule as the other calls).
 */
moespec_status moespec_reconstruction_error(const moespec_desc *desc, const void *out_budgeted, const void *out_full,
                                            int32_t M, double *err, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Oracle ranking - Eq. (6): runs the layer with natural routing (every expert of the union), then
 * greedily builds the ordering that minimises the reconstruction error against the gold output
 * O* = sum_{i in T_k(h_t)} g-bar_i(h_t) E_i(h_t): starting from the empty set, B times add the expert i
 * outside S that minimises sum_t || O*_t - sum_{j in (S + {i}) and in T_k(h_t)} g-bar_j(h_t) E_j(h_t) ||^2
 * (ties to the lowest id).  Analysis only: it streams every expert of the union.
 *   ranking [B] int32  out  experts in the order they were added (an upper-bound shortlist, usable as
 *                           ext_shortlist)
 *   err     [B] double out  that error divided by ||O*||^2 after each addition
 * The selection runs in fp64 on the experts' fp32 outputs.  Requires top_k * 8 <= d_ff * sizeof(dtype)
 * (MOESPEC_ERR_UNSUPPORTED_SHAPE otherwise).
 */
moespec_status moespec_oracle_ranking(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                      int32_t M, int32_t B, int32_t *ranking, double *err,
                                      void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Measurement aid - the practical ceiling of the roofline that bounds the expert passes: a plain streaming
 * read of `bytes` bytes (16-byte loads, eight in flight per lane, every byte read once), timed by the caller.
 * The expert passes are bound by HBM bandwidth (Section 2.2 of the paper: loading the unique experts
 * dominates verification); this kernel shows how much of the published peak a read-only stream reaches on
 * the machine at hand.
 *   buf      [bytes] in (device), 16-byte aligned; bytes a multiple of 16, 16 <= bytes < 2^40
 *   checksum [MOESPEC_STREAM_READ_WORDS] uint32 in/out (device): workgroup b ADDS the sum modulo 2^32 of the
 *            32-bit words it has read to word b (one writer per word, no atomics); the sum of all words
 *            modulo 2^32 is the checksum of the buffer; the caller zeroes the array
 * Errors: MOESPEC_ERR_INVALID_ARG for a NULL or misaligned pointer or a size outside the range.
 */
#define MOESPEC_STREAM_READ_WORDS 256
moespec_status moespec_stream_read(const void *buf, size_t bytes, uint32_t *checksum, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOESPEC_H */
