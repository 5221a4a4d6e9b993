// Per-kernel event timing used by the benchmark (see moe_profile_* in moe.h).
#include <vector>

#include "moe_internal.h"

namespace moe {

bool g_prof_on = false;
uint32_t g_prof_mask = 0xffffffffu;

namespace {
struct Rec { int id; hipEvent_t a, b; };
std::vector<Rec> g_pool;
size_t g_used = 0;
bool g_open = false;   // a begin mark was taken and awaits its end mark
}  // namespace

void prof_mark(int kernel_id, hipStream_t s, bool begin) {
  if (!(g_prof_mask >> kernel_id & 1u)) return;
  if (begin) {
    if (g_used >= g_pool.size()) { g_open = false; return; }
    g_pool[g_used].id = kernel_id;
    // a record whose begin or end mark fails is dropped, not read later
    g_open = hipEventRecord(g_pool[g_used].a, s) == hipSuccess;
  } else if (g_open) {
    if (hipEventRecord(g_pool[g_used].b, s) == hipSuccess) ++g_used;
    g_open = false;
  }
}

}  // namespace moe

using namespace moe;

extern "C" {

moe_status moe_profile_enable(int32_t max_records) {
  if (max_records < 0) return MOE_ERR_INVALID_ARG;
  g_prof_on = false;
  for (auto& r : g_pool) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_pool.clear();
  g_used = 0;
  g_open = false;
  if (max_records == 0) return MOE_OK;
  g_pool.reserve(max_records);
  for (int32_t i = 0; i < max_records; ++i) {
    Rec r;
    r.id = 0;
    if (hipEventCreate(&r.a) != hipSuccess) break;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); break; }
    g_pool.push_back(r);       // the pool only ever holds pairs that exist
  }
  if (g_pool.size() != size_t(max_records)) {
    for (auto& r : g_pool) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_pool.clear();
    return MOE_ERR_DEVICE;
  }
  g_prof_on = true;
  return MOE_OK;
}

moe_status moe_profile_filter(uint32_t mask) {
  g_prof_mask = mask;
  return MOE_OK;
}

moe_status moe_profile_read(double* total_ms, int32_t* launches) {
  if (!total_ms || !launches) return MOE_ERR_INVALID_ARG;
  for (int i = 0; i < MOE_K_COUNT; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  for (size_t i = 0; i < g_used; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(g_pool[i].b) != hipSuccess) return MOE_ERR_DEVICE;
    if (hipEventElapsedTime(&ms, g_pool[i].a, g_pool[i].b) != hipSuccess) return MOE_ERR_DEVICE;
    total_ms[g_pool[i].id] += ms;
    launches[g_pool[i].id] += 1;
  }
  g_used = 0;
  return MOE_OK;
}

const char* moe_kernel_name(int32_t id) {
  static const char* names[MOE_K_COUNT] = {
      "gate_norms", "gate_gemm", "select", "rescore", "dispatch_hist", "dispatch_scan",
      "dispatch_scatter", "dispatch_gather", "ffn_tiles", "ffn_gemm1", "ffn_gemm2", "combine"};
  return (id >= 0 && id < MOE_K_COUNT) ? names[id] : "unknown";
}

}  // extern "C"
