// Combine: return the expert outputs along the original route, weighted by the
// top-k weights, into the fp32 partial sum awaiting the intra-node all-reduce
// (Sec. II "Combine"; the accumulation step of Alg. 1: the rows a stage returns
// are scaled by their top-k weights and added to the running result).
//
// Gather-by-token: one wavefront owns a token, walks the row in 16-byte pieces
// and adds the token's local expert rows in ascending j, so there are no
// atomics and the result does not depend on scheduling.  Bandwidth-bound:
// reads A_loc*H (+T*H shared) activations, writes T*H fp32.
#include "moe_internal.h"

namespace moe {

namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// streaming (non-temporal) 16-byte accesses: data that is touched once
__device__ __forceinline__ uint4 nt_load16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(void* p, uint4 v) {
  u32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, static_cast<u32x4_t*>(p));
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ void fma8(float (&acc)[8], float w, const uint4& v) {
  acc[0] = fmaf(w, bf16_lo(v.x), acc[0]);
  acc[1] = fmaf(w, bf16_hi(v.x), acc[1]);
  acc[2] = fmaf(w, bf16_lo(v.y), acc[2]);
  acc[3] = fmaf(w, bf16_hi(v.y), acc[3]);
  acc[4] = fmaf(w, bf16_lo(v.z), acc[4]);
  acc[5] = fmaf(w, bf16_hi(v.z), acc[5]);
  acc[6] = fmaf(w, bf16_lo(v.w), acc[6]);
  acc[7] = fmaf(w, bf16_hi(v.w), acc[7]);
}

// bf16 rows: a piece is 8 elements (16 B in, 32 B out).
__global__ __launch_bounds__(256) void combine_bf16_kernel(
    const uint4* __restrict__ ys, const int32_t* __restrict__ inv, const float* __restrict__ w,
    const uint4* __restrict__ shared_ys, float4* __restrict__ out, int T, int k, int row8,
    int accumulate) {
  const int lane = threadIdx.x & 63;
  constexpr int P = 4;                          // pieces per lane in flight
  // a wavefront owns one segment of 64*P pieces of one token's row: wide rows are
  // shared out over several wavefronts, each with one round of loads and stores
  const int nseg = (row8 + 64 * P - 1) / (64 * P);
  const int gw = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int t = gw / nseg;
  if (t >= T) return;
  int pos = -1;
  float wt = 0.f;
  if (lane < k) {
    pos = inv[size_t(t) * k + lane];
    wt = w[size_t(t) * k + lane];
  }
  const uint64_t have = __ballot(pos >= 0);
  // every lane of the wavefront runs the body (the shuffles below need all of them)
  {
    const int cb = (gw - t * nseg) * 64 * P;
    const int c0 = cb + lane;
    float acc[P][8];
#pragma unroll
    for (int i = 0; i < P; ++i)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[i][q] = 0.f;
    uint64_t m = have;
    while (m) {                               // ascending j
      const int j = __ffsll((unsigned long long)m) - 1;
      m &= m - 1;
      const int p = __shfl(pos, j);
      const float wj = __shfl(wt, j);
      const uint4* row = ys + size_t(p) * row8;
      uint4 v[P];
#pragma unroll
      for (int i = 0; i < P; ++i)
        if (c0 + 64 * i < row8) v[i] = nt_load16(row + c0 + 64 * i);
#pragma unroll
      for (int i = 0; i < P; ++i)
        if (c0 + 64 * i < row8) fma8(acc[i], wj, v[i]);
    }
    if (shared_ys) {
      const uint4* row = shared_ys + size_t(t) * row8;
      uint4 v[P];
#pragma unroll
      for (int i = 0; i < P; ++i)
        if (c0 + 64 * i < row8) v[i] = nt_load16(row + c0 + 64 * i);
#pragma unroll
      for (int i = 0; i < P; ++i)
        if (c0 + 64 * i < row8) fma8(acc[i], 1.0f, v[i]);
    }
#pragma unroll
    for (int i = 0; i < P; ++i) {
      const int c = c0 + 64 * i;
      if (c < row8) {
        float4* o = out + (size_t(t) * row8 + c) * 2;
        if (accumulate) {                     // Y <- Y + (weighted sum of this stage)
          const float4 o0 = o[0], o1 = o[1];
          acc[i][0] += o0.x; acc[i][1] += o0.y; acc[i][2] += o0.z; acc[i][3] += o0.w;
          acc[i][4] += o1.x; acc[i][5] += o1.y; acc[i][6] += o1.z; acc[i][7] += o1.w;
        }
        nt_store16(o, make_uint4(__float_as_uint(acc[i][0]), __float_as_uint(acc[i][1]),
                                 __float_as_uint(acc[i][2]), __float_as_uint(acc[i][3])));
        nt_store16(o + 1, make_uint4(__float_as_uint(acc[i][4]), __float_as_uint(acc[i][5]),
                                     __float_as_uint(acc[i][6]), __float_as_uint(acc[i][7])));
      }
    }
  }
}

// fp32 rows: a piece is 4 elements.
__global__ __launch_bounds__(256) void combine_f32_kernel(
    const float4* __restrict__ ys, const int32_t* __restrict__ inv, const float* __restrict__ w,
    const float4* __restrict__ shared_ys, float4* __restrict__ out, int T, int k, int row4,
    int accumulate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= T) return;
  int pos = -1;
  float wt = 0.f;
  if (lane < k) {
    pos = inv[size_t(t) * k + lane];
    wt = w[size_t(t) * k + lane];
  }
  const uint64_t have = __ballot(pos >= 0);
  // the loop bounds are the same in every lane (the shuffles below need all of them)
  for (int cb = 0; cb < row4; cb += 64) {
    const int c = cb + lane;
    const bool in = c < row4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    uint64_t m = have;
    while (m) {
      const int j = __ffsll((unsigned long long)m) - 1;
      m &= m - 1;
      const int p = __shfl(pos, j);
      const float wj = __shfl(wt, j);
      if (in) {
        const float4 v = ys[size_t(p) * row4 + c];
        acc.x = fmaf(wj, v.x, acc.x);
        acc.y = fmaf(wj, v.y, acc.y);
        acc.z = fmaf(wj, v.z, acc.z);
        acc.w = fmaf(wj, v.w, acc.w);
      }
    }
    if (!in) continue;
    if (shared_ys) {
      const float4 v = shared_ys[size_t(t) * row4 + c];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (accumulate) {
      const float4 o = out[size_t(t) * row4 + c];
      acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
    }
    out[size_t(t) * row4 + c] = acc;
  }
}

}  // namespace

// `width` = elements per row of ys / shared_ys / out (the hidden size, or one
// hidden-column block of it).
hipError_t launch_combine(const moe_config& c, int T, const void* ys, const int32_t* inv,
                          const float* w, const void* shared_ys, float* out, int width,
                          int accumulate, hipStream_t s) {
  const dim3 block(256);
  dim3 grid((T + 3) / 4);
  if (c.act_dtype == MOE_BF16) {
    const size_t nseg = (size_t(width / 8) + 255) / 256;      // wavefronts per token row
    grid = dim3(unsigned((size_t(T) * nseg + 3) / 4));
    MOE_LAUNCH(MOE_K_COMBINE, combine_bf16_kernel, grid, block, 0, s, static_cast<const uint4*>(ys), inv,
                       w, static_cast<const uint4*>(shared_ys), reinterpret_cast<float4*>(out), T,
                       c.top_k, width / 8, accumulate);
  } else {
    MOE_LAUNCH(MOE_K_COMBINE, combine_f32_kernel, grid, block, 0, s, static_cast<const float4*>(ys), inv,
                       w, static_cast<const float4*>(shared_ys), reinterpret_cast<float4*>(out), T,
                       c.top_k, width / 4, accumulate);
  }
  return hipGetLastError();
}

}  // namespace moe
