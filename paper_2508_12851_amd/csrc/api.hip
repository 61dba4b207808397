// C ABI of libprism: host-side validation, workspace carving and launch order.
#include "prism_internal.h"

namespace prism {

prism_status validate_desc(const prism_layer_desc* d, int32_t T, bool need_ffn_shapes) {
  PRISM_RETURN_IF(d == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(T < 0, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->hidden < 1 || d->n_experts < 1 || d->n_shared < 0, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->top_k < 1 || d->top_k > d->n_experts, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->bias_group_tokens < 0, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->gate_mode != PRISM_GATES_RENORMALIZED && d->gate_mode != PRISM_GATES_SOFTMAX_ALL,
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->weight_layout != PRISM_WEIGHTS_ROW_MAJOR && d->weight_layout != PRISM_WEIGHTS_TILED,
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->weight_layout == PRISM_WEIGHTS_TILED && d->dtype != PRISM_BF16, PRISM_ERR_UNSUPPORTED);
  PRISM_RETURN_IF(d->dtype != PRISM_F32 && d->dtype != PRISM_BF16, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(d->n_experts > PRISM_MAX_EXPERTS || d->top_k > PRISM_MAX_TOPK ||
                      d->n_shared > PRISM_MAX_SHARED,
                  PRISM_ERR_UNSUPPORTED);
  PRISM_RETURN_IF(d->hidden % 8 != 0, PRISM_ERR_UNSUPPORTED);
  const long long rows = (long long)T * d->top_k + (long long)T * d->n_shared;
  PRISM_RETURN_IF(rows >= (1LL << 30), PRISM_ERR_UNSUPPORTED);
  if (need_ffn_shapes) {
    PRISM_RETURN_IF(d->ffn < 1, PRISM_ERR_INVALID_ARG);
    if (d->dtype == PRISM_BF16)
      PRISM_RETURN_IF(d->hidden % 64 != 0 || d->ffn % 64 != 0, PRISM_ERR_UNSUPPORTED);
  }
  return PRISM_OK;
}

static prism_status check_workspace(const prism_layer_desc& d, int T, void* ws, size_t ws_bytes,
                                    Workspace* out) {
  PRISM_RETURN_IF(ws == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(((uintptr_t)ws & 255u) != 0, PRISM_ERR_INVALID_ARG);
  const Workspace probe = carve(d, T, nullptr);
  PRISM_RETURN_IF(ws_bytes < probe.total, PRISM_ERR_WORKSPACE_TOO_SMALL);
  *out = carve(d, T, ws);
  return PRISM_OK;
}

static prism_status check_weights(const prism_layer_desc& d, const prism_expert_weights* w) {
  PRISM_RETURN_IF(w == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(w->w_gate == nullptr || w->w_up == nullptr || w->w_down == nullptr,
                  PRISM_ERR_INVALID_ARG);
  if (d.n_shared > 0)
    PRISM_RETURN_IF(w->shared_w_gate == nullptr || w->shared_w_up == nullptr ||
                        w->shared_w_down == nullptr,
                    PRISM_ERR_INVALID_ARG);
  return PRISM_OK;
}

// ---------------------------------------------------------------------------
// Scratch memory of prism_moe_layer_static: a fixed device array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy at its own address; `scratch`
// itself is only a host-side handle of the symbol, the device address comes from
// hipGetSymbolAddress (once per device, with that device current) and is what the kernels get.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = PRISM_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static prism_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PRISM_ERR_LAUNCH;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    // two threads racing here ask for the same address; either store is fine
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return PRISM_ERR_LAUNCH;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return PRISM_OK;
}

}  // namespace prism

using namespace prism;

extern "C" {
#pragma GCC visibility push(default)

const char* prism_status_string(prism_status s) {
  switch (s) {
    case PRISM_OK: return "ok";
    case PRISM_ERR_INVALID_ARG: return "invalid argument";
    case PRISM_ERR_UNSUPPORTED: return "size or dtype outside the supported limits";
    case PRISM_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case PRISM_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}

prism_status prism_workspace_bytes(const prism_layer_desc* desc, int32_t max_tokens, size_t* bytes) {
  PRISM_RETURN_IF(bytes == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_TRY(validate_desc(desc, max_tokens, true));
  *bytes = carve(*desc, max_tokens, nullptr).total;
  return PRISM_OK;
}

prism_status prism_route(const prism_layer_desc* desc, const void* x, const void* w_router,
                         const float* router_bias, int32_t T, float* logits, int32_t* topk_idx,
                         float* topk_gate, int32_t* counts, int64_t* counts_accum, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, false));
  PRISM_RETURN_IF(counts == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0)
    PRISM_RETURN_IF(x == nullptr || w_router == nullptr || topk_idx == nullptr || topk_gate == nullptr,
                    PRISM_ERR_INVALID_ARG);
  return launch_route(*desc, x, w_router, router_bias, T, logits, topk_idx, topk_gate, counts,
                      counts_accum, (hipStream_t)stream);
}

prism_status prism_dispatch(const prism_layer_desc* desc, const int32_t* topk_idx,
                            const uint8_t* local_mask, int32_t T, int32_t* local_src,
                            int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                            int32_t* n_local_remote, int64_t* remote_bytes, void* workspace,
                            size_t workspace_bytes, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, false));
  PRISM_RETURN_IF(local_mask == nullptr || local_offsets == nullptr || remote_offsets == nullptr ||
                      n_local_remote == nullptr || remote_bytes == nullptr,
                  PRISM_ERR_INVALID_ARG);
  if (T > 0)
    PRISM_RETURN_IF(topk_idx == nullptr || local_src == nullptr || remote_src == nullptr,
                    PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, workspace, workspace_bytes, &ws));
  return launch_dispatch(*desc, topk_idx, local_mask, T, local_src, local_offsets, remote_src,
                         remote_offsets, n_local_remote, remote_bytes, nullptr, ws.block_hist,
                         nullptr, nullptr, (hipStream_t)stream);
}

prism_status prism_expert_ffn(const prism_layer_desc* desc, const void* x,
                              const prism_expert_weights* weights, const int32_t* local_src,
                              const int32_t* local_offsets, int32_t T, void* y, void* workspace,
                              size_t workspace_bytes, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, true));
  PRISM_TRY(check_weights(*desc, weights));
  PRISM_RETURN_IF(local_offsets == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0) PRISM_RETURN_IF(x == nullptr || local_src == nullptr || y == nullptr, PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, workspace, workspace_bytes, &ws));
  return launch_expert_ffn(*desc, x, *weights, local_src, local_offsets, T, y, ws.h, ws.tiles,
                           ws.part, ws.slice_part, (hipStream_t)stream, nullptr, nullptr);
}

prism_status prism_combine(const prism_layer_desc* desc, const void* y, const int32_t* local_src,
                           const int32_t* local_offsets, const float* topk_gate, int32_t T,
                           void* out, void* workspace, size_t workspace_bytes, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, true));
  PRISM_RETURN_IF(local_offsets == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0)
    PRISM_RETURN_IF(y == nullptr || local_src == nullptr || topk_gate == nullptr || out == nullptr,
                    PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, workspace, workspace_bytes, &ws));
  const hipStream_t st = (hipStream_t)stream;
  PRISM_TRY(launch_build_inverse(*desc, local_src, local_offsets, T, ws.inv, st));
  return launch_combine(*desc, y, ws.inv, topk_gate, T, out, st);
}

prism_status prism_pack_remote(const prism_layer_desc* desc, const void* x, const int32_t* remote_src,
                               const int32_t* remote_offsets, int32_t T, void* packed, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, false));
  PRISM_RETURN_IF(remote_offsets == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0) PRISM_RETURN_IF(x == nullptr || remote_src == nullptr || packed == nullptr, PRISM_ERR_INVALID_ARG);
  return launch_pack_rows(*desc, x, remote_src, remote_offsets, T, packed, (hipStream_t)stream);
}

prism_status prism_combine_remote(const prism_layer_desc* desc, const void* y_remote,
                                  const int32_t* remote_src, const int32_t* remote_offsets,
                                  const float* topk_gate, int32_t T, void* out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, false));
  PRISM_RETURN_IF(remote_offsets == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0)
    PRISM_RETURN_IF(y_remote == nullptr || remote_src == nullptr || topk_gate == nullptr || out == nullptr,
                    PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, workspace, workspace_bytes, &ws));
  const hipStream_t st = (hipStream_t)stream;
  PRISM_TRY(launch_build_inverse(*desc, remote_src, remote_offsets, T, ws.inv, st));
  return launch_combine(*desc, y_remote, ws.inv, topk_gate, T, out, st, nullptr, nullptr, true);
}

prism_status prism_pack_weights(const void* src, int32_t rows, int32_t cols, void* dst, void* stream) {
  PRISM_ENTER();
  PRISM_RETURN_IF(src == nullptr || dst == nullptr || rows < 1 || cols < 1, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF((((uintptr_t)src | (uintptr_t)dst) & 15u) != 0, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(rows % 16 != 0 || cols % 32 != 0, PRISM_ERR_UNSUPPORTED);
  PRISM_RETURN_IF((size_t)rows * cols * 2 >= 0xFFFF0000ull, PRISM_ERR_UNSUPPORTED);
  return launch_pack_weights(src, rows, cols, dst, (hipStream_t)stream);
}

prism_status prism_debug_check_weights(const prism_layer_desc* desc,
                                       const prism_expert_weights* weights,
                                       const uint8_t* local_mask, int32_t* bad_expert) {
  PRISM_TRY(validate_desc(desc, 0, false));
  PRISM_TRY(check_weights(*desc, weights));
  PRISM_RETURN_IF(local_mask == nullptr, PRISM_ERR_INVALID_ARG);
  const int E = desc->n_experts, S = desc->n_shared;
  uint8_t mask[PRISM_MAX_EXPERTS];
  const void* routed[3][PRISM_MAX_EXPERTS];
  const void* shared[3][PRISM_MAX_SHARED];
  const void* const* rt[3] = {weights->w_gate, weights->w_up, weights->w_down};
  const void* const* sh[3] = {weights->shared_w_gate, weights->shared_w_up, weights->shared_w_down};
  if (hipMemcpy(mask, local_mask, (size_t)E, hipMemcpyDeviceToHost) != hipSuccess) return PRISM_ERR_LAUNCH;
  for (int i = 0; i < 3; ++i) {
    if (hipMemcpy(routed[i], rt[i], (size_t)E * sizeof(void*), hipMemcpyDeviceToHost) != hipSuccess)
      return PRISM_ERR_LAUNCH;
    if (S > 0 && hipMemcpy(shared[i], sh[i], (size_t)S * sizeof(void*), hipMemcpyDeviceToHost) != hipSuccess)
      return PRISM_ERR_LAUNCH;
  }
  auto bad = [](const void* p) { return p == nullptr || ((uintptr_t)p & 15u) != 0; };
  for (int e = 0; e < E + S; ++e) {
    const bool hosted = e >= E || mask[e] != 0;
    if (!hosted) continue;
    for (int i = 0; i < 3; ++i)
      if (bad(e < E ? routed[i][e] : shared[i][e - E])) {
        if (bad_expert != nullptr) *bad_expert = e;
        return PRISM_ERR_INVALID_ARG;
      }
  }
  return PRISM_OK;
}

prism_status prism_moe_layer_traced(const prism_layer_desc* desc, const void* x,
                                    const void* w_router, const float* router_bias,
                                    const prism_expert_weights* weights,
                                    const uint8_t* local_mask, int32_t T, void* out,
                                    int32_t* topk_idx, float* topk_gate, int32_t* counts,
                                    int64_t* counts_accum, int32_t* remote_src,
                                    int32_t* remote_offsets, int32_t* n_local_remote,
                                    int64_t* remote_bytes, void* workspace, size_t workspace_bytes,
                                    void* stream, void* const* stage_events) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, true));
  PRISM_TRY(check_weights(*desc, weights));
  PRISM_RETURN_IF(local_mask == nullptr || counts == nullptr || remote_offsets == nullptr ||
                      n_local_remote == nullptr || remote_bytes == nullptr,
                  PRISM_ERR_INVALID_ARG);
  if (T > 0)
    PRISM_RETURN_IF(x == nullptr || w_router == nullptr || out == nullptr || topk_idx == nullptr ||
                        topk_gate == nullptr || remote_src == nullptr,
                    PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, workspace, workspace_bytes, &ws));
  const hipStream_t st = (hipStream_t)stream;
  void* const* ev = stage_events;
  const int32_t* n_splits = nullptr;   // set if the down projection is left as contraction slices
  if (decode_front_end_applies(*desc, T)) {
    PRISM_TRY(launch_decode_front_end(*desc, x, w_router, router_bias, local_mask, T, topk_idx,
                                      topk_gate, counts, counts_accum, ws.local_src,
                                      ws.local_offsets, remote_src, remote_offsets, n_local_remote,
                                      remote_bytes, ws.inv, ws.route_part, ws.tiles, st, ev));
    PRISM_TRY(launch_expert_ffn(*desc, x, *weights, ws.local_src, ws.local_offsets, T, ws.y, ws.h,
                                ws.tiles, ws.part, ws.slice_part, st, ev, &n_splits, true));
  } else {
    trace(ev, PRISM_STAGE_ROUTE, 0, st);
    // the activation counts come out of the dispatch histogram, not out of the router
    PRISM_TRY(launch_route(*desc, x, w_router, router_bias, T, nullptr, topk_idx, topk_gate, nullptr,
                           nullptr, st));
    trace(ev, PRISM_STAGE_ROUTE, 1, st);
    trace(ev, PRISM_STAGE_DISPATCH, 0, st);
    bool schedules_built = false;
    PRISM_TRY(launch_dispatch(*desc, topk_idx, local_mask, T, ws.local_src, ws.local_offsets,
                              remote_src, remote_offsets, n_local_remote, remote_bytes, ws.inv,
                              ws.block_hist, counts, counts_accum, st, ws.tiles, &schedules_built));
    trace(ev, PRISM_STAGE_DISPATCH, 1, st);
    PRISM_TRY(launch_expert_ffn(*desc, x, *weights, ws.local_src, ws.local_offsets, T, ws.y, ws.h,
                                ws.tiles, ws.part, ws.slice_part, st, ev, &n_splits, schedules_built));
  }
  trace(ev, PRISM_STAGE_COMBINE, 0, st);
  PRISM_TRY(launch_combine(*desc, ws.y, ws.inv, topk_gate, T, out, st, ws.part, n_splits));
  trace(ev, PRISM_STAGE_COMBINE, 1, st);
  return PRISM_OK;
}

prism_status prism_layer_permutation(const prism_layer_desc* desc, int32_t T, const void* workspace,
                                     size_t workspace_bytes, int32_t* local_src,
                                     int32_t* local_offsets, int32_t* inv, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, true));
  PRISM_RETURN_IF(local_offsets == nullptr, PRISM_ERR_INVALID_ARG);
  if (T > 0) PRISM_RETURN_IF(local_src == nullptr, PRISM_ERR_INVALID_ARG);
  Workspace ws;
  PRISM_TRY(check_workspace(*desc, T, const_cast<void*>(workspace), workspace_bytes, &ws));
  const hipStream_t st = (hipStream_t)stream;
  const size_t A = (size_t)T * desc->top_k;
  auto copy = [&](void* dst, const void* src, size_t bytes) {
    return bytes == 0 || hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess;
  };
  if (!copy(local_offsets, ws.local_offsets, (size_t)(desc->n_experts + 1) * 4) ||
      !copy(local_src, ws.local_src, A * 4) || (inv != nullptr && !copy(inv, ws.inv, A * 4)))
    return PRISM_ERR_LAUNCH;
  return PRISM_OK;
}

prism_status prism_moe_layer(const prism_layer_desc* desc, const void* x, const void* w_router,
                             const float* router_bias, const prism_expert_weights* weights,
                             const uint8_t* local_mask, int32_t T, void* out, int32_t* topk_idx,
                             float* topk_gate, int32_t* counts, int64_t* counts_accum,
                             int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, void* workspace,
                             size_t workspace_bytes, void* stream) {
  return prism_moe_layer_traced(desc, x, w_router, router_bias, weights, local_mask, T, out,
                                topk_idx, topk_gate, counts, counts_accum, remote_src,
                                remote_offsets, n_local_remote, remote_bytes, workspace,
                                workspace_bytes, stream, nullptr);
}

prism_status prism_moe_layer_static(const prism_layer_desc* desc, const void* x, const void* w_router,
                                    const float* router_bias, const prism_expert_weights* weights,
                                    const uint8_t* local_mask, int32_t T, void* out, int32_t* topk_idx,
                                    float* topk_gate, int32_t* counts, int64_t* counts_accum,
                                    int32_t* remote_src, int32_t* remote_offsets,
                                    int32_t* n_local_remote, int64_t* remote_bytes, void* stream) {
  PRISM_ENTER();
  PRISM_TRY(validate_desc(desc, T, true));
  // the same layout the caller's workspace would have; it has to fit the fixed array
  PRISM_RETURN_IF(carve(*desc, T, nullptr).total > kStaticScratchBytes, PRISM_ERR_WORKSPACE_TOO_SMALL);
  void* ws = nullptr;
  PRISM_TRY(static_scratch(&ws));
  return prism_moe_layer_traced(desc, x, w_router, router_bias, weights, local_mask, T, out, topk_idx,
                                topk_gate, counts, counts_accum, remote_src, remote_offsets,
                                n_local_remote, remote_bytes, ws, kStaticScratchBytes, stream, nullptr);
}

#pragma GCC visibility pop
}  // extern "C"
