// C ABI of the library: argument validation (host only, before any launch), workspace carve-up,
// and the sequencing of the kernel launchers.
#include <atomic>

#include "common.h"

using namespace moespec;

namespace {

constexpr int kMaxExperts = 1024;
constexpr int kMaxTopK = 64;
constexpr int kMaxHidden = 8192;
constexpr int kMaxInter = 1 << 20;
constexpr int kMaxTokens = 65535;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

moespec_status check_desc(const moespec_desc *ds) {
  if (!ds) return MOESPEC_ERR_INVALID_ARG;
  if (ds->dtype != MOESPEC_F32 && ds->dtype != MOESPEC_BF16) return MOESPEC_ERR_INVALID_ARG;
  if (ds->renorm != 0 && ds->renorm != 1) return MOESPEC_ERR_INVALID_ARG;
  if (ds->gate != MOESPEC_GATE_SOFTMAX && ds->gate != MOESPEC_GATE_SIGMOID) return MOESPEC_ERR_INVALID_ARG;
  if (ds->d < 1 || ds->d_ff < 1 || ds->n_experts < 1) return MOESPEC_ERR_INVALID_ARG;
  if (ds->top_k < 1 || ds->top_k > ds->n_experts) return MOESPEC_ERR_INVALID_ARG;
  if (ds->n_experts > kMaxExperts || ds->top_k > kMaxTopK || ds->d > kMaxHidden || ds->d_ff > kMaxInter)
    return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  const int mult = ds->dtype == MOESPEC_BF16 ? 32 : 4;
  if (ds->d % mult != 0 || ds->d_ff % mult != 0) return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  if ((int64_t)ds->n_experts * ds->d_ff * ds->d >= (int64_t)1 << 40) return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  return MOESPEC_OK;
}

moespec_status check_common(const moespec_desc *ds, int32_t M, const void *ws, size_t ws_bytes) {
  moespec_status s = check_desc(ds);
  if (s != MOESPEC_OK) return s;
  if (M < 1 || M > kMaxTokens) return MOESPEC_ERR_INVALID_ARG;
  // the kernels index the per-pair intermediates with 32-bit element offsets
  if ((int64_t)M * ds->top_k * (ds->d > ds->d_ff ? ds->d : ds->d_ff) >= ((int64_t)1 << 31))
    return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOESPEC_ERR_INVALID_ARG;
  if (ws_bytes < carve_workspace(*ds, M, nullptr).bytes) return MOESPEC_ERR_WORKSPACE_TOO_SMALL;
  return MOESPEC_OK;
}

moespec_status check_weights(const moespec_weights *wt, bool router, bool experts) {
  if (!wt) return MOESPEC_ERR_INVALID_ARG;
  if (router && (!wt->w_router || !aligned16(wt->w_router))) return MOESPEC_ERR_INVALID_ARG;
  if (experts && (!wt->w_gate || !wt->w_up || !wt->w_down || !aligned16(wt->w_gate) || !aligned16(wt->w_up) ||
                  !aligned16(wt->w_down)))
    return MOESPEC_ERR_INVALID_ARG;
  return MOESPEC_OK;
}

moespec_status check_budget(const moespec_desc *ds, int32_t B, int32_t policy) {
  if (policy != MOESPEC_TRUNCATE && policy != MOESPEC_SUBSTITUTE) return MOESPEC_ERR_INVALID_ARG;
  if (B < 1 || B > ds->n_experts) return MOESPEC_ERR_INVALID_ARG;
  if (policy == MOESPEC_SUBSTITUTE && B < ds->top_k) return MOESPEC_ERR_INVALID_ARG;
  return MOESPEC_OK;
}

moespec_status from_hip(hipError_t e) { return e == hipSuccess ? MOESPEC_OK : MOESPEC_ERR_HIP; }


// Scratch memory of moespec_layer_forward_static: the workspace of the other entry points as a file-scope
// device array, so that the call allocates nothing.  Every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the array's name is only a handle: the device address is resolved
// once per device with hipGetSymbolAddress and kept here; kernels are only ever given that address.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[MOESPEC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];

void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void *p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  scratch_ptr[dev].store(p, std::memory_order_release);  // every thread resolves the same address: no lock needed
  return p;
}

// The argument checks of the fused call other than those on the tree size and the workspace (desc is valid).
moespec_status check_layer_args(const moespec_desc *desc, const moespec_weights *weights, const void *h, int32_t B,
                                int32_t policy, const void *residual, const void *out) {
  moespec_status s = check_weights(weights, true, true);
  if (s != MOESPEC_OK) return s;
  if ((s = check_budget(desc, B, policy)) != MOESPEC_OK) return s;
  if (!h || !out || !aligned16(h) || !aligned16(out) || (residual && !aligned16(residual)))
    return MOESPEC_ERR_INVALID_ARG;
  return MOESPEC_OK;
}

moespec_status layer_forward(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                     int32_t M, int32_t B, int32_t policy, const int32_t *ext_shortlist,
                                     const void *residual, void *out, const moespec_taps *taps, void *ws,
                                     size_t ws_bytes, void *hip_stream, void *const *tr = nullptr,
                                     void *x_next = nullptr) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if ((s = check_layer_args(desc, weights, h, B, policy, residual, out)) != MOESPEC_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Workspace w = carve_workspace(*desc, M, ws);
  // A tap replaces the workspace slot of the same intermediate, so it is written in place.
  moespec_taps t = taps ? *taps : moespec_taps{};
  double *probs = t.probs ? t.probs : w.probs;
  int32_t *tok_ids = t.tok_ids ? t.tok_ids : w.tok_ids;
  float *tok_w = t.tok_w ? t.tok_w : w.tok_w;
  int32_t *seg_expert = t.seg_expert ? t.seg_expert : w.seg_expert;
  int32_t *seg_off = t.seg_off ? t.seg_off : w.seg_off;
  int32_t *perm = t.perm ? t.perm : w.perm;
  int32_t *budget_ids = t.budget_ids ? t.budget_ids : w.budget_ids;
  auto mark = [&](int i) {
    if (tr && tr[i]) (void)hipEventRecord(static_cast<hipEvent_t>(tr[i]), st);
  };
  mark(0);
  if (fused_prologue_ok(*desc, M) && expert_ffn_self_segmenting(*desc, M)) {
    // Small trees: two launches leave the shortlist, the restricted routing and every loaded expert's pair
    // list; the expert passes pick their work items from those lists.
    hipError_t e = launch_fused_prologue(*desc, *weights, h, M, B, policy, ext_shortlist, w.partial, w.probs, t.probs,
                                         t.scores,
                                         budget_ids, t.seg_expert, tok_ids, tok_w, w.list_count, w.lists, M,
                                         t.seg_off, t.perm, t.n_loaded, st);
    if (e != hipSuccess) return MOESPEC_ERR_HIP;
    mark(1);
    e = launch_expert_ffn(*desc, *weights, h, M, B, nullptr, nullptr, nullptr, tok_ids, tok_w, residual, out, w.act,
                          w.y, w.items, false, w.list_count, budget_ids, nullptr, nullptr, st, tr ? tr + 2 : nullptr,
                          w.lists, M, x_next);
    return from_hip(e);
  }
  // Other shapes: the expert passes derive their segments themselves where they can, and the budget stage groups
  // the pairs only if the caller asked for the segment arrays or the passes need them.
  const bool self_seg = expert_ffn_self_segmenting(*desc, M);
  const bool want_segments = !self_seg || t.seg_off || t.perm || t.n_loaded;
  hipError_t e = mfma_route_ok(*desc, M)
                     ? launch_mfma_route(*desc, *weights, h, M, w.partial, probs, w.done, 1 + desc->n_experts, st)
                     : launch_route(*desc, *weights, h, M, probs, nullptr, nullptr, w.done, 1 + desc->n_experts, st);
  if (e != hipSuccess) return MOESPEC_ERR_HIP;
  e = launch_budget(*desc, probs, M, B, policy, ext_shortlist, t.scores, budget_ids, tok_ids, tok_w, seg_expert,
                    seg_off, perm, t.n_loaded, w.items, w.done, true, want_segments, w.scores, st);
  if (e != hipSuccess) return MOESPEC_ERR_HIP;
  mark(1);
  e = launch_expert_ffn(*desc, *weights, h, M, B, seg_expert, seg_off, perm, tok_ids, tok_w, residual, out, w.act,
                        w.y, w.items, want_segments, self_seg ? w.done + 1 : nullptr, budget_ids, w.pub_items,
                        w.pub_lists, st, tr ? tr + 2 : nullptr, nullptr, 0, x_next);
  return from_hip(e);
}

}  // namespace

extern "C" {

int32_t moespec_abi_version(void) { return 5; }

const char *moespec_status_string(int32_t status) {
  switch (status) {
    case MOESPEC_OK: return "ok";
    case MOESPEC_ERR_INVALID_ARG: return "invalid argument";
    case MOESPEC_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case MOESPEC_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOESPEC_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

moespec_status moespec_check_desc(const moespec_desc *desc) { return check_desc(desc); }

size_t moespec_workspace_bytes(const moespec_desc *desc, int32_t M_max) {
  if (check_desc(desc) != MOESPEC_OK || M_max < 1 || M_max > kMaxTokens) return 0;
  return carve_workspace(*desc, M_max, nullptr).bytes;
}

moespec_status moespec_route(const moespec_desc *desc, const moespec_weights *weights, const void *h, int32_t M,
                             double *probs, int32_t *topk_ids, float *topk_w, void *ws, size_t ws_bytes,
                             void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if ((s = check_weights(weights, true, false)) != MOESPEC_OK) return s;
  if (!h || !probs || !aligned16(h)) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(
      launch_route(*desc, *weights, h, M, probs, topk_ids, topk_w, nullptr, 0, static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_budget(const moespec_desc *desc, const double *probs, int32_t M, int32_t B, int32_t policy,
                              const int32_t *ext_shortlist, double *scores, int32_t *budget_ids, int32_t *tok_ids,
                              float *tok_w, int32_t *seg_expert, int32_t *seg_off, int32_t *perm, int32_t *n_loaded,
                              void *ws, size_t ws_bytes, void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if ((s = check_budget(desc, B, policy)) != MOESPEC_OK) return s;
  if (!probs || !tok_ids || !tok_w || !seg_expert || !seg_off || !perm) return MOESPEC_ERR_INVALID_ARG;
  Workspace w = carve_workspace(*desc, M, ws);
  return from_hip(launch_budget(*desc, probs, M, B, policy, ext_shortlist, scores,
                                budget_ids ? budget_ids : w.budget_ids, tok_ids, tok_w,
                                seg_expert, seg_off, perm, n_loaded, w.items, w.done, false, true,
                                w.scores, static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_expert_ffn(const moespec_desc *desc, const moespec_weights *weights, const void *h, int32_t M,
                                  int32_t n_seg, const int32_t *seg_expert, const int32_t *seg_off,
                                  const int32_t *perm, const int32_t *tok_ids, const float *tok_w,
                                  const void *residual, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if ((s = check_weights(weights, false, true)) != MOESPEC_OK) return s;
  if (n_seg < 1 || n_seg > desc->n_experts) return MOESPEC_ERR_INVALID_ARG;
  if (!h || !seg_expert || !seg_off || !perm || !tok_ids || !tok_w || !out) return MOESPEC_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(out) || (residual && !aligned16(residual))) return MOESPEC_ERR_INVALID_ARG;
  Workspace w = carve_workspace(*desc, M, ws);
  return from_hip(launch_expert_ffn(*desc, *weights, h, M, n_seg, seg_expert, seg_off, perm, tok_ids, tok_w, residual,
                                    out, w.act, w.y, w.items, false, nullptr, nullptr, nullptr, nullptr,
                                    static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_layer_forward(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                     int32_t M, int32_t B, int32_t policy, const int32_t *ext_shortlist,
                                     const void *residual, void *out, const moespec_taps *taps, void *ws,
                                     size_t ws_bytes, void *hip_stream) {
  return layer_forward(desc, weights, h, M, B, policy, ext_shortlist, residual, out, taps, ws, ws_bytes, hip_stream);
}

moespec_status moespec_layer_forward_traced(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                            int32_t M, int32_t B, int32_t policy, const int32_t *ext_shortlist,
                                            const void *residual, void *out, int32_t *n_loaded,
                                            void *const *trace_events, void *ws, size_t ws_bytes, void *hip_stream) {
  moespec_taps t{};
  t.n_loaded = n_loaded;
  return layer_forward(desc, weights, h, M, B, policy, ext_shortlist, residual, out, &t, ws, ws_bytes, hip_stream,
                       trace_events);
}

moespec_status moespec_layer_forward_static(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                            int32_t M, int32_t B, int32_t policy, const int32_t *ext_shortlist,
                                            const void *residual, void *out, void *hip_stream) {
  // shapes first: a descriptor error is reported as such, a layer that does not fit the array as a workspace error
  moespec_status s = check_desc(desc);
  if (s != MOESPEC_OK) return s;
  if (M < 1 || M > kMaxTokens) return MOESPEC_ERR_INVALID_ARG;
  if ((int64_t)M * desc->top_k * (desc->d > desc->d_ff ? desc->d : desc->d_ff) >= ((int64_t)1 << 31))
    return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  if (carve_workspace(*desc, M, nullptr).bytes > (size_t)MOESPEC_STATIC_SCRATCH_BYTES)
    return MOESPEC_ERR_WORKSPACE_TOO_SMALL;
  if ((s = check_layer_args(desc, weights, h, B, policy, residual, out)) != MOESPEC_OK) return s;
  void *ws = static_scratch();  // the first GPU-touching step: every argument error has been reported by now
  if (!ws) return MOESPEC_ERR_HIP;
  return layer_forward(desc, weights, h, M, B, policy, ext_shortlist, residual, out, nullptr, ws, (size_t)MOESPEC_STATIC_SCRATCH_BYTES,
                       hip_stream);
}

moespec_status moespec_rms_scale(const moespec_desc *desc, const void *h, int32_t M, void *x, void *hip_stream) {
  moespec_status s = check_desc(desc);
  if (s != MOESPEC_OK) return s;
  if (M < 1 || M > kMaxTokens || !h || !x || !aligned16(h) || !aligned16(x)) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(launch_rms_scale(*desc, h, M, x, static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_stack_forward(const moespec_desc *desc, const moespec_weights *layers, int32_t n_layers, void *h,
                                     int32_t M, int32_t B, int32_t policy, int32_t pre_norm, int32_t *budget_ids,
                                     int32_t *tok_ids, void *ws, size_t ws_bytes, void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if (!layers || n_layers < 1 || n_layers > 4096 || (pre_norm != 0 && pre_norm != 1)) return MOESPEC_ERR_INVALID_ARG;
  for (int32_t l = 0; l < n_layers; ++l)  // every layer is validated before the first launch
    if ((s = check_layer_args(desc, &layers[l], h, B, policy, h, h)) != MOESPEC_OK) return s;
  Workspace w = carve_workspace(*desc, M, ws);
  for (int32_t l = 0; l < n_layers; ++l) {
    const void *x = h;
    if (pre_norm) {
      // the first layer's input is scaled by a launch of its own; every later one by the combine of the layer before
      if (l == 0 && launch_rms_scale(*desc, h, M, w.xnorm, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return MOESPEC_ERR_HIP;
      x = w.xnorm;
    }
    moespec_taps t{};
    t.budget_ids = budget_ids ? budget_ids + (size_t)l * B : nullptr;
    t.tok_ids = tok_ids ? tok_ids + (size_t)l * M * desc->top_k : nullptr;
    // the combine reads residual[t, j] and writes out[t, j] in the same thread, after every kernel that reads the
    // layer input: updating the residual stream (and, for the next layer, the scaled input) in place is safe
    void *x_next = (pre_norm && l + 1 < n_layers) ? w.xnorm : nullptr;
    if ((s = layer_forward(desc, &layers[l], x, M, B, policy, nullptr, h, h, &t, ws, ws_bytes, hip_stream, nullptr,
                           x_next)) != MOESPEC_OK)
      return s;
  }
  return MOESPEC_OK;
}

moespec_status moespec_calibration_count(const moespec_desc *desc, const int32_t *topk_ids, int32_t M,
                                         int64_t *counts, void *hip_stream) {
  moespec_status s = check_desc(desc);
  if (s != MOESPEC_OK) return s;
  if (M < 1 || M > kMaxTokens || !topk_ids || !counts) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(launch_calibration_count(topk_ids, M, desc->top_k, desc->n_experts, counts,
                                           static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_static_shortlist(const moespec_desc *desc, const int64_t *counts, int32_t B,
                                        int32_t *shortlist, void *hip_stream) {
  moespec_status s = check_desc(desc);
  if (s != MOESPEC_OK) return s;
  if (B < 1 || B > desc->n_experts || !counts || !shortlist) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(launch_static_shortlist(counts, desc->n_experts, B, shortlist, static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_coverage_curve(const moespec_desc *desc, const double *scores, double *curve,
                                      void *hip_stream) {
  moespec_status s = check_desc(desc);
  if (s != MOESPEC_OK) return s;
  if (!scores || !curve) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(launch_coverage_curve(scores, desc->n_experts, curve, static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_reconstruction_error(const moespec_desc *desc, const void *out_budgeted, const void *out_full,
                                            int32_t M, double *err, void *ws, size_t ws_bytes, void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if (!out_budgeted || !out_full || !err) return MOESPEC_ERR_INVALID_ARG;
  Workspace w = carve_workspace(*desc, M, ws);
  // the per-token partial sums (2 M doubles) borrow the y buffer (M * k * d floats, d >= 4)
  return from_hip(launch_reconstruction_error(*desc, out_budgeted, out_full, M, reinterpret_cast<double *>(w.y), err,
                                              static_cast<hipStream_t>(hip_stream)));
}

moespec_status moespec_oracle_ranking(const moespec_desc *desc, const moespec_weights *weights, const void *h,
                                      int32_t M, int32_t B, int32_t *ranking, double *err, void *ws, size_t ws_bytes,
                                      void *hip_stream) {
  moespec_status s = check_common(desc, M, ws, ws_bytes);
  if (s != MOESPEC_OK) return s;
  if ((s = check_weights(weights, true, true)) != MOESPEC_OK) return s;
  if (B < 1 || B > desc->n_experts || !h || !aligned16(h) || !ranking || !err) return MOESPEC_ERR_INVALID_ARG;
  // the per-token k x k Gram blocks (doubles) borrow the act buffer once the down pass has read it
  const size_t es = desc->dtype == MOESPEC_BF16 ? 2 : 4;
  if ((size_t)desc->top_k * 8 > (size_t)desc->d_ff * es) return MOESPEC_ERR_UNSUPPORTED_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Workspace w = carve_workspace(*desc, M, ws);
  const int N = desc->n_experts;
  // natural routing (Eq. (2)): the budgeted path with B = N and truncation keeps every token's top-k
  const bool self_seg = expert_ffn_self_segmenting(*desc, M);
  hipError_t e = launch_route(*desc, *weights, h, M, w.probs, nullptr, nullptr, w.done, 1 + N, st);
  if (e != hipSuccess) return MOESPEC_ERR_HIP;
  e = launch_budget(*desc, w.probs, M, N, MOESPEC_TRUNCATE, nullptr, nullptr, w.budget_ids, w.tok_ids, w.tok_w,
                    w.seg_expert, w.seg_off, w.perm, nullptr, w.items, w.done, true, !self_seg, w.scores, st);
  if (e != hipSuccess) return MOESPEC_ERR_HIP;
  e = launch_expert_ffn(*desc, *weights, h, M, N, w.seg_expert, w.seg_off, w.perm, w.tok_ids, w.tok_w, nullptr,
                        nullptr, w.act, w.y, w.items, !self_seg, self_seg ? w.done + 1 : nullptr, w.budget_ids,
                        w.pub_items, w.pub_lists, st);
  if (e != hipSuccess) return MOESPEC_ERR_HIP;
  return from_hip(launch_oracle_ranking(*desc, w.y, down_splits(*desc, N), (size_t)M * desc->top_k * desc->d,
                                        w.tok_ids, w.tok_w, M, B, static_cast<double *>(w.act), w.gram, ranking, err,
                                        st));
}

moespec_status moespec_stream_read(const void *buf, size_t bytes, uint32_t *checksum, void *hip_stream) {
  if (!buf || !checksum || !aligned16(buf) || (reinterpret_cast<uintptr_t>(checksum) & 3u) != 0)
    return MOESPEC_ERR_INVALID_ARG;
  if (bytes < 16 || bytes % 16 != 0 || bytes >= ((size_t)1 << 40)) return MOESPEC_ERR_INVALID_ARG;
  return from_hip(launch_stream_read(buf, bytes, checksum, static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
