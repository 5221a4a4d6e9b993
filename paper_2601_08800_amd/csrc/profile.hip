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

// ---- calibration: the matrix units with nothing else going on ---------------
// Every wavefront runs `iters` rounds of eight independent
// v_mfma_f32_32x32x16_bf16 on register operands (128 accumulator registers, two
// wavefronts per SIMD: the shape of the tall-tile GEMM's inner loop without its
// loads, LDS reads and barriers).  Operands are non-trivial bit patterns so that
// the data path toggles as it does on real inputs.  Nothing is stored unless
// `sink` is given.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void mfma_probe_kernel(int iters, float* sink) {
  const uint32_t h = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
  // bf16 values of magnitude 0.5 .. 1 with hashed signs and mantissas
  const uint32_t pat = 0x3f003f00u | (h & 0x807f807fu);
  uint4 ua = make_uint4(pat, pat ^ 0x80000040u, pat ^ 0x00408000u, pat ^ 0x80108010u);
  uint4 ub = make_uint4(pat ^ 0x00208020u, pat ^ 0x80400000u, pat ^ 0x00008008u, pat ^ 0x80048004u);
  probe_f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
  for (int it = 0; it < iters; ++it) {
    const probe_bf16x8 a = __builtin_bit_cast(probe_bf16x8, ua), b = __builtin_bit_cast(probe_bf16x8, ub);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    ua.x ^= 0x80008000u;          // keep the sums from drifting: alternate the sign of one pair
  }
  if (sink) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) s += acc[j][q];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
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

moe_status moe_probe_mfma_rate(int32_t workgroups, int32_t iters, void* stream, double* tflops) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || !tflops) return MOE_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return MOE_ERR_DEVICE;
  if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return MOE_ERR_DEVICE;}
  float ms = 0.f;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(512), 0, s, iters / 8 + 1, (float*)nullptr);  // warm-up
  bool ok = hipEventRecord(a, s) == hipSuccess;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(512), 0, s, iters, (float*)nullptr);
  ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(b, s) == hipSuccess &&
       hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (!ok || ms <= 0.f) return MOE_ERR_DEVICE;
  // 8 wavefronts x iters x 8 instructions x 32*32*16*2 flops
  *tflops = double(workgroups) * 8.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
  return MOE_OK;
}

const char* moe_kernel_name(int32_t id) {
  static const char* names[MOE_K_COUNT] = {
      "gate_norms", "gate_gemm", "select", "rescore", "dispatch_hist", "dispatch_scan",
      "dispatch_scatter", "dispatch_gather", "ffn_tiles", "ffn_gemm1", "ffn_gemm2", "combine"};
  return (id >= 0 && id < MOE_K_COUNT) ? names[id] : "unknown";
}

}  // extern "C"
