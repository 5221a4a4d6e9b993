// Sanitizer leg of the host-side argument validation: compiled together with
// csrc/moe_api.hip (host pass under -fsanitize=address,undefined) and run by
// tests/test_sanitizers.py.  The kernel launchers are replaced by stubs that
// record the call, so every entry point can be driven through its error paths
// and its accepting path without a GPU: validation and workspace carving touch
// no HIP API.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "moe_internal.h"

namespace moe {
bool g_prof_on = false;
void prof_mark(int, hipStream_t, bool) {}
static int g_launches = 0;
hipError_t launch_route(const moe_config&, int, const void*, const void*, const float*, const float*,
                        const float*, int32_t*, float*, const RouteWs&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_dispatch(const moe_config&, int, const void*, const int32_t*, int32_t*, int32_t*, int32_t*,
                           int32_t*, void*, int, int, const DispatchWs&, hipStream_t, int) { ++g_launches; return hipSuccess; }
hipError_t launch_dispatch_scales(const float*, int, const int32_t*, const int32_t*, int, int, int, float*, int,
                                  hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_expert_ffn(const moe_config&, int, const void*, const int32_t*, int, const void*, const void*,
                             const void*, const float*, const float*, const float*, void*, const FfnWs&,
                             hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_combine(const moe_config&, int, const void*, const int32_t*, const float*, const void*, float*,
                          int, int, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace moe

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); std::exit(3); } } while (0)

int main() {
  moe_config c{};
  c.hidden = 256; c.n_experts = 8; c.top_k = 2; c.score_fn = MOE_SCORE_SOFTMAX; c.renormalize = 1;
  c.routed_scale = 1.f; c.n_groups = 1; c.topk_groups = 1; c.group_score_n = 0; c.expert_lo = 0;
  c.expert_hi = 8; c.inter_local = 512; c.act_dtype = MOE_BF16; c.weight_dtype = MOE_BF16;
  const int T = 100;
  const size_t need = moe_workspace_bytes(&c, T);
  CHECK(need > 0 && moe_workspace_bytes(&c, -1) == 0 && moe_workspace_bytes(nullptr, T) == 0);
  // real host memory stands in for the device buffers: the stubs never touch it,
  // and a carve that ran past `need` bytes would be caught
  std::vector<char> ws(need + 16), buf(1 << 16);
  void* W = reinterpret_cast<void*>((reinterpret_cast<uintptr_t>(ws.data()) + 15) & ~uintptr_t(15));
  void* P = reinterpret_cast<void*>((reinterpret_cast<uintptr_t>(buf.data()) + 15) & ~uintptr_t(15));
  void* Q = static_cast<char*>(P) + 1;                    // misaligned
  int32_t* I = static_cast<int32_t*>(P);
  float* F = static_cast<float*>(P);

  CHECK(moe_route(&c, T, P, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_OK);
  CHECK(moe::g_launches == 1);
  CHECK(moe_route(&c, T, P, P, nullptr, nullptr, nullptr, I, F, W, 64, nullptr) == MOE_ERR_WORKSPACE);
  CHECK(moe_route(&c, T, nullptr, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_route(&c, T, Q, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_route(&c, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == MOE_OK);
  CHECK(moe_route(nullptr, T, P, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_dispatch(&c, T, P, I, I, I, I, I, P, W, need, nullptr) == MOE_OK);
  CHECK(moe_dispatch(&c, T, P, I, I, I, I, I, P, W, 0, nullptr) == MOE_ERR_WORKSPACE);
  CHECK(moe_dispatch_shard(&c, T, P, I, 3, 2, I, I, I, I, P, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_dispatch_shard(&c, T, P, I, 1, 2, I, I, I, I, P, W, need, nullptr) == MOE_OK);
  CHECK(moe_expert_ffn(&c, 8, P, I, T * 2, P, P, P, nullptr, nullptr, nullptr, P, W, need, nullptr) == MOE_OK);
  CHECK(moe_expert_ffn(&c, 9, P, I, T * 2, P, P, P, nullptr, nullptr, nullptr, P, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_expert_ffn(&c, 8, P, I, T * 2, P, P, P, nullptr, nullptr, nullptr, P, W, 64, nullptr) == MOE_ERR_WORKSPACE);
  CHECK(moe_combine(&c, T, P, I, F, nullptr, F, nullptr) == MOE_OK);
  CHECK(moe_combine(&c, T, P, I, F, Q, F, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_combine_stage(&c, T, P, I, F, 2, 0, F, nullptr) == MOE_OK);
  CHECK(moe_combine_stage(&c, T, P, I, F, 3, 0, F, nullptr) == MOE_ERR_INVALID_ARG);
  CHECK(moe_combine_stage(&c, T, P, I, F, 2, 2, F, nullptr) == MOE_ERR_INVALID_ARG);
  // the entry point without a workspace: its size limit and the argument checks come
  // before anything touches the device (65 536 tokens x top-2 over 8 experts fit, x top-8 over
  // 128 local experts of a 128-expert layer is exactly the limit, one chunk more is refused)
  CHECK(moe_dispatch_noalloc_max_bytes() == (size_t(4) << 20));
  {
    moe_config big = c; big.n_experts = 128; big.expert_hi = 128; big.top_k = 8;
    CHECK(moe_dispatch_noalloc(&big, 65536 + 8, P, I, I, I, I, I, P, nullptr) == MOE_ERR_WORKSPACE);
    CHECK(moe_dispatch_noalloc(&big, -1, P, I, I, I, I, I, P, nullptr) == MOE_ERR_INVALID_ARG);
    CHECK(moe_dispatch_noalloc(nullptr, 8, P, I, I, I, I, I, P, nullptr) == MOE_ERR_INVALID_ARG);
    CHECK(moe_dispatch_noalloc(&big, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == MOE_OK);
  }
  // every structural rule of the layer description
  moe_config b = c; b.hidden = 100; CHECK(moe_workspace_bytes(&b, T) == 0);
  b = c; b.top_k = 9; CHECK(moe_route(&b, T, P, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_ERR_INVALID_ARG);
  b = c; b.n_groups = 3; CHECK(moe_workspace_bytes(&b, T) == 0);
  b = c; b.n_groups = 4; b.topk_groups = 2; b.group_score_n = 3; CHECK(moe_workspace_bytes(&b, T) == 0);
  b = c; b.expert_lo = 5; b.expert_hi = 5; CHECK(moe_workspace_bytes(&b, T) == 0);
  b = c; b.weight_dtype = MOE_FP8_E4M3_B128; b.inter_local = 520;
  CHECK(moe_route(&b, T, P, P, nullptr, nullptr, nullptr, I, F, W, need, nullptr) == MOE_ERR_UNSUPPORTED);
  b = c; b.act_dtype = MOE_F32; CHECK(moe_workspace_bytes(&b, T) == 0);      // f32 activations need f32 weights
  b = c; b.n_experts = 600; b.expert_hi = 600; CHECK(moe_workspace_bytes(&b, T) == 0);
  // the largest layer the kernels admit: the carve must stay inside what workspace_bytes reports
  b = c; b.n_experts = 512; b.expert_hi = 512; b.top_k = 32; b.hidden = 7168; b.inter_local = 2048;
  const int Tb = 4096;
  const size_t nb = moe_workspace_bytes(&b, Tb);
  CHECK(nb > 0);
  CHECK(moe::carve_route(nullptr, Tb, 512).bytes <= nb);
  CHECK(moe::carve_dispatch(nullptr, Tb, 32, 512).bytes <= nb);
  CHECK(moe::carve_ffn(nullptr, Tb * 32, 512, 2048, 2).bytes <= nb);
  for (int s = 0; s <= 5; ++s) CHECK(moe_status_string(static_cast<moe_status>(s)) != nullptr);
  std::puts("api sanitizer leg: ok");
  return 0;
}
