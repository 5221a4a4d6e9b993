// C entry points of libmoe: host-side validation, workspace carving, launch.
// Validation touches no HIP API, so every error path is testable without a GPU.
#include "moe_internal.h"

namespace moe {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int act_bytes(int dt) { return dt == MOE_F32 ? 4 : 2; }

// Structural checks of the layer description (dtype support is checked apart).
static moe_status check_config(const moe_config* c) {
  if (!c) return MOE_ERR_INVALID_ARG;
  if (c->hidden <= 0 || c->hidden % 8) return MOE_ERR_INVALID_ARG;
  if (c->n_experts <= 0 || c->top_k < 1 || c->top_k > c->n_experts) return MOE_ERR_INVALID_ARG;
  if (c->score_fn != MOE_SCORE_SOFTMAX && c->score_fn != MOE_SCORE_SIGMOID)
    return MOE_ERR_INVALID_ARG;
  if (c->n_groups < 1 || c->n_experts % c->n_groups) return MOE_ERR_INVALID_ARG;
  if (c->n_groups > 1) {
    int gs = c->n_experts / c->n_groups;
    if (c->topk_groups < 1 || c->topk_groups > c->n_groups) return MOE_ERR_INVALID_ARG;
    if (c->group_score_n < 1 || c->group_score_n > gs) return MOE_ERR_INVALID_ARG;
    if (c->top_k > c->topk_groups * gs) return MOE_ERR_INVALID_ARG;
  }
  if (c->expert_lo < 0 || c->expert_hi > c->n_experts || c->expert_lo >= c->expert_hi)
    return MOE_ERR_INVALID_ARG;
  if (c->inter_local <= 0 || c->inter_local % 8) return MOE_ERR_INVALID_ARG;
  if (!(c->routed_scale == c->routed_scale)) return MOE_ERR_INVALID_ARG;  // NaN
  // dtypes
  if (c->act_dtype != MOE_F32 && c->act_dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  bool ok = (c->act_dtype == MOE_F32 && c->weight_dtype == MOE_F32) ||
            (c->act_dtype == MOE_BF16 &&
             (c->weight_dtype == MOE_BF16 || c->weight_dtype == MOE_FP8_E4M3_B128));
  if (!ok) return MOE_ERR_UNSUPPORTED;
  if (c->weight_dtype == MOE_FP8_E4M3_B128 && (c->inter_local % 128 || c->hidden % 128))
    return MOE_ERR_UNSUPPORTED;
  // kernel limits
  if (c->top_k > 32 || c->n_experts > 512 || c->n_groups > 64) return MOE_ERR_UNSUPPORTED;
  return MOE_OK;
}

// Sizing calls pass a null base: pieces are then null too (no arithmetic on a
// null pointer), only `bytes` is meaningful.
template <typename T>
static T* piece(void* ws, size_t off) {
  return ws ? reinterpret_cast<T*>(static_cast<char*>(ws) + off) : nullptr;
}

RouteWs carve_route(void* ws, int T, int E) {
  RouteWs r;
  size_t off = 0;
  r.counters = piece<int32_t>(ws, off);   off += kRouteCounterBytes;
  r.logits = piece<float>(ws, off);       off += align_up(size_t(T) * E * 4 * gate_split_cap(T, E));
  r.xnorm2 = piece<float>(ws, off);       off += align_up(size_t(T) * 4 * gate_split_cap(T, E));
  r.wnorm2 = piece<float>(ws, off);       off += align_up(size_t(E) * 4 * gate_split_cap(T, E));
  r.recheck = piece<int32_t>(ws, off);    off += align_up(size_t(T) * 4);
  r.recheck_low = piece<float>(ws, off);  off += align_up(size_t(T) * 4);
  r.bytes = off;
  return r;
}

DispatchWs carve_dispatch(void* ws, int T, int k, int E_loc) {
  DispatchWs d;
  size_t A = size_t(T) * k;
  d.n_blocks = int((A + kDispatchChunk - 1) / kDispatchChunk);   // sub-chunks of 64 assignments
  d.block_hist = static_cast<int32_t*>(ws);
  d.bytes = align_up(size_t(d.n_blocks) * E_loc * 4);
  return d;
}

FfnWs carve_ffn(void* ws, int rows_capacity, int n_experts, int I_loc, int abytes) {
  FfnWs f;
  f.max_tiles = rows_capacity / kMaxTileRows + n_experts + 1;
  size_t off = 0;
  f.tiles = piece<int32_t>(ws, off);  off += align_up(size_t(1 + 5 * f.max_tiles) * 4 + 12);
  f.tiles2 = piece<int32_t>(ws, off); off += align_up(size_t(1 + 5 * f.max_tiles) * 4 + 12);
  f.hmid = piece<char>(ws, off);      off += align_up(size_t(rows_capacity) * I_loc * abytes);
  f.tickets = piece<int32_t>(ws, off); off += align_up(size_t(2) * kFfnSplitSlots * 4);
  f.partial = piece<float>(ws, off);   off += align_up(size_t(kFfnSplitSlots) * kFfnPartBytes);
  f.bytes = off;
  return f;
}

}  // namespace moe

using namespace moe;

// ---- moe_dispatch_noalloc: the dispatch index scratch lives in the library ----
// The multi-kernel dispatch keeps one count per (local expert, sub-chunk of 64
// assignments) between its kernels.  For callers that cannot provide a workspace
// this fixed device array stands in for it; each GPU the library runs on holds
// its own copy at its own address until the process ends.
constexpr size_t kNoAllocScratchBytes = size_t(4) << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

// Device address of `scratch` on the current device, resolved once per device
// (the array's name is only a host-side handle for hipGetSymbolAddress; it is
// never passed to a kernel or a runtime call as an address).
static hipError_t noalloc_scratch(void** out) {
  static void* ptr_of_device[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr_of_device[dev] = p;
  }
  *out = ptr_of_device[dev];
  return hipSuccess;
}

extern "C" {

const char* moe_status_string(moe_status s) {
  switch (s) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED: return "unsupported dtype or shape";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_DEVICE: return "device launch failed";
  }
  return "unknown status";
}

size_t moe_workspace_bytes(const moe_config* cfg, int32_t T) {
  if (check_config(cfg) != MOE_OK || T < 0) return 0;
  if (T == 0) return 256;
  int k = cfg->top_k;
  size_t r = carve_route(nullptr, T, cfg->n_experts).bytes;
  size_t d = carve_dispatch(nullptr, T, k, cfg->expert_hi - cfg->expert_lo).bytes;
  // the FFN is called with at most T*k rows and at most n_experts experts
  size_t f = carve_ffn(nullptr, T * k, cfg->n_experts, cfg->inter_local,
                       act_bytes(cfg->act_dtype)).bytes;
  size_t m = r > d ? r : d;
  return m > f ? m : f;
}

moe_status moe_route(const moe_config* cfg, int32_t T, const void* x, const void* gate_w,
                     const float* logit_bias, const float* select_bias,
                     const float* logits_in, int32_t* topk_ids, float* topk_w, void* ws,
                     size_t ws_bytes, void* stream) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (T < 0) return MOE_ERR_INVALID_ARG;
  if (T == 0) return MOE_OK;
  if (size_t(T) * cfg->n_experts > (size_t(1) << 31) - 1) return MOE_ERR_UNSUPPORTED;
  if (!topk_ids || !topk_w || !ws) return MOE_ERR_INVALID_ARG;
  if (!logits_in && (!x || !gate_w)) return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {x, gate_w, logit_bias, select_bias, logits_in, topk_ids, topk_w, ws};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
  RouteWs r = carve_route(ws, T, cfg->n_experts);
  if (ws_bytes < r.bytes) return MOE_ERR_WORKSPACE;
  hipError_t e = launch_route(*cfg, T, x, gate_w, logit_bias, select_bias, logits_in, topk_ids,
                              topk_w, r, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

namespace {
// hidden-column sharding over a TP group: the shard must be whole 16-byte pieces
bool shard_ok(const moe_config* cfg, int32_t tp_rank, int32_t tp_size) {
  if (tp_size < 1 || tp_rank < 0 || tp_rank >= tp_size) return false;
  if (cfg->hidden % tp_size) return false;
  return (cfg->hidden / tp_size) % 8 == 0;
}

moe_status dispatch_impl(const moe_config* cfg, int32_t T, const void* x, const int32_t* topk_ids,
                         int32_t tp_rank, int32_t tp_size, int32_t* counts, int32_t* offsets,
                         int32_t* perm, int32_t* inv, void* xs, void* ws, size_t ws_bytes,
                         void* stream, int elem_bytes = 0) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (T < 0 || !shard_ok(cfg, tp_rank, tp_size)) return MOE_ERR_INVALID_ARG;
  if (T == 0) return MOE_OK;
  if (size_t(T) * cfg->top_k > (size_t(1) << 30)) return MOE_ERR_UNSUPPORTED;
  if (!x || !topk_ids || !counts || !offsets || !perm || !inv || !xs || !ws)
    return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {x, topk_ids, counts, offsets, perm, inv, xs, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) return MOE_ERR_INVALID_ARG;
  DispatchWs d = carve_dispatch(ws, T, cfg->top_k, cfg->expert_hi - cfg->expert_lo);
  if (ws_bytes < d.bytes) return MOE_ERR_WORKSPACE;
  hipError_t e = launch_dispatch(*cfg, T, x, topk_ids, counts, offsets, perm, inv, xs, tp_rank,
                                 tp_size, d, static_cast<hipStream_t>(stream), elem_bytes);
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}
}  // namespace

moe_status moe_dispatch(const moe_config* cfg, int32_t T, const void* x,
                        const int32_t* topk_ids, int32_t* counts, int32_t* offsets,
                        int32_t* perm, int32_t* inv, void* xs, void* ws, size_t ws_bytes,
                        void* stream) {
  return dispatch_impl(cfg, T, x, topk_ids, 0, 1, counts, offsets, perm, inv, xs, ws, ws_bytes,
                       stream);
}

size_t moe_dispatch_noalloc_max_bytes(void) { return kNoAllocScratchBytes; }

moe_status moe_dispatch_noalloc(const moe_config* cfg, int32_t T, const void* x,
                                const int32_t* topk_ids, int32_t* counts, int32_t* offsets,
                                int32_t* perm, int32_t* inv, void* xs, void* stream) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (T < 0) return MOE_ERR_INVALID_ARG;
  if (T == 0) return MOE_OK;
  if (size_t(T) * cfg->top_k > (size_t(1) << 30)) return MOE_ERR_UNSUPPORTED;
  // the size limit is checked before anything touches the device
  const size_t need = carve_dispatch(nullptr, T, cfg->top_k, cfg->expert_hi - cfg->expert_lo).bytes;
  if (need > kNoAllocScratchBytes) return MOE_ERR_WORKSPACE;
  void* ws = nullptr;
  if (noalloc_scratch(&ws) != hipSuccess) return MOE_ERR_DEVICE;
  return dispatch_impl(cfg, T, x, topk_ids, 0, 1, counts, offsets, perm, inv, xs, ws,
                       kNoAllocScratchBytes, stream);
}

moe_status moe_dispatch_shard(const moe_config* cfg, int32_t T, const void* x,
                              const int32_t* topk_ids, int32_t tp_rank, int32_t tp_size,
                              int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                              void* xs_shard, void* ws, size_t ws_bytes, void* stream) {
  return dispatch_impl(cfg, T, x, topk_ids, tp_rank, tp_size, counts, offsets, perm, inv, xs_shard,
                       ws, ws_bytes, stream);
}

moe_status moe_dispatch_fp8q(const moe_config* cfg, int32_t T, const void* xq,
                             const float* xq_scales, const int32_t* topk_ids, int32_t* counts,
                             int32_t* offsets, int32_t* perm, int32_t* inv, void* xs_q,
                             float* xs_scales, void* ws, size_t ws_bytes, void* stream) {
  if (!cfg) return MOE_ERR_INVALID_ARG;
  if (cfg->hidden % 128) return MOE_ERR_UNSUPPORTED;
  if (!xq_scales || !xs_scales || !aligned16(xq_scales) || !aligned16(xs_scales))
    return MOE_ERR_INVALID_ARG;
  moe_status st = dispatch_impl(cfg, T, xq, topk_ids, 0, 1, counts, offsets, perm, inv, xs_q, ws,
                                ws_bytes, stream, 1);
  if (st != MOE_OK || T == 0) return st;
  hipError_t e = launch_dispatch_scales(xq_scales, T, perm, offsets, cfg->expert_hi - cfg->expert_lo,
                                        cfg->top_k, cfg->hidden / 128, xs_scales, T * cfg->top_k,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

moe_status moe_expert_ffn(const moe_config* cfg, int32_t n_experts_here, const void* xs,
                          const int32_t* offsets, int32_t rows_capacity, const void* w_gate,
                          const void* w_up, const void* w_down, const float* s_gate,
                          const float* s_up, const float* s_down, void* ys, void* ws,
                          size_t ws_bytes, void* stream) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (n_experts_here < 1 || n_experts_here > cfg->n_experts || rows_capacity < 0)
    return MOE_ERR_INVALID_ARG;
  if (rows_capacity == 0) return MOE_OK;
  if (!xs || !offsets || !w_gate || !w_up || !w_down || !ys || !ws) return MOE_ERR_INVALID_ARG;
  bool fp8 = cfg->weight_dtype == MOE_FP8_E4M3_B128;
  if (fp8 && (!s_gate || !s_up || !s_down)) return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {xs, offsets, w_gate, w_up, w_down, s_gate, s_up, s_down, ys, ws};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
  FfnWs f = carve_ffn(ws, rows_capacity, n_experts_here, cfg->inter_local,
                      act_bytes(cfg->act_dtype));
  if (ws_bytes < f.bytes) return MOE_ERR_WORKSPACE;
  hipError_t e = launch_expert_ffn(*cfg, n_experts_here, xs, offsets, rows_capacity, w_gate,
                                   w_up, w_down, s_gate, s_up, s_down, ys, f,
                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

moe_status moe_combine(const moe_config* cfg, int32_t T, const void* ys, const int32_t* inv,
                       const float* topk_w, const void* shared_ys, float* out, void* stream) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (T < 0) return MOE_ERR_INVALID_ARG;
  if (T == 0) return MOE_OK;
  if (!ys || !inv || !topk_w || !out) return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {ys, inv, topk_w, shared_ys, out};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
  hipError_t e = launch_combine(*cfg, T, ys, inv, topk_w, shared_ys, out, cfg->hidden, 0,
                                static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

moe_status moe_combine_stage(const moe_config* cfg, int32_t T, const void* ys_block,
                             const int32_t* inv, const float* topk_w, int32_t tp_size,
                             int32_t accumulate, float* out_block, void* stream) {
  moe_status st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (T < 0 || !shard_ok(cfg, 0, tp_size) || (accumulate != 0 && accumulate != 1))
    return MOE_ERR_INVALID_ARG;
  if (T == 0) return MOE_OK;
  if (!ys_block || !inv || !topk_w || !out_block) return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {ys_block, inv, topk_w, out_block};
  for (const void* p : ptrs)
    if (!aligned16(p)) return MOE_ERR_INVALID_ARG;
  hipError_t e = launch_combine(*cfg, T, ys_block, inv, topk_w, nullptr, out_block,
                                cfg->hidden / tp_size, accumulate,
                                static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

}  // extern "C"
