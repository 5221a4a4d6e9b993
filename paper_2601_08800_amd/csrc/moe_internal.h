// Internal declarations shared by the translation units of libmoe.
// Host-side launch wrappers live next to their kernels; the C entry points in
// moe_api.cpp validate arguments and carve the workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;

// ---- workspace carving (all sizes in bytes, 256-byte aligned pieces) ------
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// route
constexpr int kRouteCounterBytes = 256;       // [0]=tokens re-scored in fp64
constexpr int kGateMaxSplit = 4;              // K splits of the gate GEMM when few tokens leave CUs idle
constexpr int kGateWgTarget = 512;            // workgroups the gate GEMM aims at: two per CU
constexpr int kGateTileM = 64, kGateTileN = 128;
// K splits the gate GEMM can use at most on a T x E grid of tiles (its workspace
// holds that many slabs).  Never below two: the exact two-kernel route keeps one
// double per (token, expert) in the same area.
inline int gate_split_cap(int T, int E) {
  const long blocks = long((T + kGateTileM - 1) / kGateTileM) * ((E + kGateTileN - 1) / kGateTileN);
  int n = 1;
  while (n < kGateMaxSplit && blocks * n * 2 <= kGateWgTarget) n *= 2;
  return n < 2 ? 2 : n;
}
#ifndef MOE_GATE_CHAIN
#define MOE_GATE_CHAIN 1
#endif
constexpr int kGateChainSteps = MOE_GATE_CHAIN;   // K-steps of 64 per fp32 accumulation chain
struct RouteWs {
  int32_t* counters;   // [64]
  float* logits;       // [gate_split_cap][T,E] fast logits (fp32), one slab per K split
  float* xnorm2;       // [gate_split_cap][T] sum of squares of the token row, per K split
  float* wnorm2;       // [gate_split_cap][E] sum of squares of the gate row, per K split
  int32_t* recheck;    // [T] token ids to re-score
  float* recheck_low;  // [T] per listed token: smallest lower bound of its picks (NaN: not known)
  size_t bytes;
};
RouteWs carve_route(void* ws, int T, int E);

// dispatch
constexpr int kDispatchChunk = 64;            // assignments per histogram column (one wavefront)
struct DispatchWs {
  int32_t* block_hist; // [E_loc, n_blocks] counts per expert and sub-chunk of 64
                       // assignments -> after the scan: start of the sub-chunk's
                       // run inside the expert's segment
  int n_blocks;
  size_t bytes;
};
DispatchWs carve_dispatch(void* ws, int T, int k, int E_loc);

// expert FFN
constexpr int kMaxTileRows = 32;              // smallest M tile any FFN kernel uses
constexpr int kFfnSplitSlots = 256;           // K-split parts in flight: one workgroup per CU at most
constexpr size_t kFfnPartBytes = size_t(512) * 128 * 4;   // fp32 accumulators of one workgroup
struct FfnWs {
  int32_t* tiles;      // [0]=number of M tiles, then 5-int tile records
  int32_t* tiles2;     // a second table of the same capacity (GEMM-2 with another tile height)
  void* hmid;          // [rows_capacity, I_loc] act dtype
  float* partial;      // fp32 partial sums of K-split tiles: kFfnSplitSlots workgroups' accumulators
  int32_t* tickets;    // [2 * kFfnSplitSlots] arrival counters of the split tiles (GEMM-1, GEMM-2)
  int max_tiles;
  size_t bytes;
};
FfnWs carve_ffn(void* ws, int rows_capacity, int n_experts, int I_loc, int act_bytes);

// ---- optional per-kernel event timing ---------------------------------------
void prof_mark(int kernel_id, hipStream_t s, bool begin);
extern bool g_prof_on;
// Launch `kernel` and, when profiling is on, bracket it with an event pair.
#define MOE_LAUNCH(id, kernel, grid, block, lds, stream, ...)            \
  do {                                                                   \
    if (::moe::g_prof_on) ::moe::prof_mark(id, stream, true);            \
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);   \
    if (::moe::g_prof_on) ::moe::prof_mark(id, stream, false);           \
  } while (0)

// A kernel that uses more than 64 KB of dynamic LDS must opt in, once per device.
// `done` is the call site's own record (one bit per device ordinal); a repeated
// call from a racing thread is harmless.
inline void lds_opt_in(const void* kernel, int bytes, uint64_t& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return;
  const uint64_t bit = uint64_t(1) << (dev & 63);
  if (done & bit) return;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess)
    done |= bit;
}

// ---- launchers (return hipGetLastError() of their launches) ---------------
hipError_t launch_route(const moe_config& c, int T, const void* x, const void* gate_w,
                        const float* logit_bias, const float* select_bias,
                        const float* logits_in, int32_t* ids, float* w, const RouteWs& ws,
                        hipStream_t s);

hipError_t launch_dispatch(const moe_config& c, int T, const void* x, const int32_t* ids,
                           int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                           void* xs, int tp_rank, int tp_size, const DispatchWs& ws,
                           hipStream_t s, int elem_bytes = 0);

hipError_t launch_dispatch_scales(const float* in, int in_pitch, const int32_t* perm,
                                  const int32_t* offsets, int E_loc, int k, int n_blocks, float* out,
                                  int out_pitch, hipStream_t s);

hipError_t launch_expert_ffn(const moe_config& c, int n_experts, const void* xs,
                             const int32_t* offsets, int rows_capacity, const void* w_gate,
                             const void* w_up, const void* w_down, const float* s_gate,
                             const float* s_up, const float* s_down, void* ys,
                             const FfnWs& ws, hipStream_t s);

hipError_t launch_combine(const moe_config& c, int T, const void* ys, const int32_t* inv,
                          const float* w, const void* shared_ys, float* out, int width,
                          int accumulate, hipStream_t s);

}  // namespace moe
