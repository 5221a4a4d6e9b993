// Dispatch: build the expert-contiguous send buffer (Sec. II "EP"; Alg. 2).
//
// A stable counting sort of the local assignments by expert, with no atomics
// anywhere (so the permutation is unique and repeatable):
//   1. hist    one wavefront per chunk of assignments counts, per local
//              expert, the chunk's assignments (wave ballots, no atomics)
//   2. scan    per expert an exclusive scan over chunks, then an exclusive
//              scan over experts -> counts, offsets, per-chunk start positions
//   3. scatter the same ballots give every assignment its rank inside its
//              chunk -> perm, inv
//   4. gather  one wavefront per token reads the row ONCE (16 B per lane,
//              coalesced) and writes it to each of its local positions
#include "moe_internal.h"

namespace moe {

namespace {

constexpr int kMaxLocalExperts = 512;

__device__ __forceinline__ uint64_t lanemask_lt() {
  return (uint64_t(1) << (threadIdx.x & 63)) - 1;
}

// One wavefront per chunk. MODE 0: histogram. MODE 1: scatter.
template <int MODE>
__global__ __launch_bounds__(64) void dispatch_index_kernel(
    const int32_t* __restrict__ ids, int A, int e_lo, int E_loc, int32_t* __restrict__ block_hist,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv) {
  __shared__ int32_t cnt[kMaxLocalExperts];
  const int lane = threadIdx.x;
  const int b = blockIdx.x;
  int32_t* mine = block_hist + size_t(b) * E_loc;
  for (int e = lane; e < E_loc; e += 64) cnt[e] = (MODE == 0) ? 0 : mine[e];
  __syncthreads();
  const int base = b * kDispatchChunk;
  for (int it = 0; it < kDispatchChunk / 64; ++it) {
    const int a = base + it * 64 + lane;
    int e = -1;
    if (a < A) e = ids[a] - e_lo;
    const bool local = (e >= 0) && (e < E_loc);
    if (MODE == 1 && a < A && !local) inv[a] = -1;
    uint64_t todo = __ballot(local);
    // visit the distinct experts present in this group of 64 assignments
    while (todo) {
      const int leader = __ffsll((unsigned long long)todo) - 1;
      const int e0 = __shfl(e, leader);
      const uint64_t m = __ballot(local && e == e0);
      const int start = cnt[e0];          // same value in every lane
      if (MODE == 1 && local && e == e0) {
        const int pos = start + __popcll(m & lanemask_lt());
        perm[pos] = a;
        inv[a] = pos;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      if (lane == leader) cnt[e0] = start + __popcll(m);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      todo &= ~m;
    }
  }
  if (MODE == 0) {
    __syncthreads();
    for (int e = lane; e < E_loc; e += 64) mine[e] = cnt[e];
  }
}

// Single block. block_hist[b][e] (counts) -> start position of chunk b's first
// assignment of expert e; counts[e]; offsets = exclusive scan of counts.
__global__ __launch_bounds__(256) void dispatch_scan_kernel(int32_t* __restrict__ block_hist,
                                                           int n_blocks, int E_loc,
                                                           int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets) {
  __shared__ int32_t tot[kMaxLocalExperts + 1];
  for (int e = threadIdx.x; e < E_loc; e += blockDim.x) {
    int run = 0;
    for (int b = 0; b < n_blocks; ++b) {
      int c = block_hist[size_t(b) * E_loc + e];
      block_hist[size_t(b) * E_loc + e] = run;
      run += c;
    }
    tot[e] = run;
    counts[e] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int e = 0; e < E_loc; ++e) {
      int c = tot[e];
      tot[e] = run;
      offsets[e] = run;
      run += c;
    }
    offsets[E_loc] = run;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_blocks * E_loc; i += blockDim.x) block_hist[i] += tot[i % E_loc];
}

// One wavefront per token: read the row once, write it to every local position.
// `row16` = row length in 16-byte pieces.
template <int PIECES>
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const uint4* __restrict__ x,
                                                             const int32_t* __restrict__ inv,
                                                             uint4* __restrict__ xs, int T, int k,
                                                             int row16) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= T) return;
  int pos = -1;
  if (lane < k) pos = inv[size_t(t) * k + lane];      // k <= 32
  const uint64_t have = __ballot(pos >= 0);
  if (!have) return;
  const uint4* src = x + size_t(t) * row16;
  for (int c0 = 0; c0 < row16; c0 += 64 * PIECES) {
    uint4 v[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int c = c0 + i * 64 + lane;
      if (c < row16) v[i] = src[c];
    }
    uint64_t m = have;
    while (m) {
      const int j = __ffsll((unsigned long long)m) - 1;
      m &= m - 1;
      const int p = __shfl(pos, j);
      uint4* dst = xs + size_t(p) * row16;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        const int c = c0 + i * 64 + lane;
        if (c < row16) dst[c] = v[i];
      }
    }
  }
}

}  // namespace

hipError_t launch_dispatch(const moe_config& c, int T, const void* x, const int32_t* ids,
                           int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                           void* xs, const DispatchWs& ws, hipStream_t s) {
  const int k = c.top_k;
  const int A = T * k;
  const int E_loc = c.expert_hi - c.expert_lo;
  MOE_LAUNCH(MOE_K_DISPATCH_HIST, dispatch_index_kernel<0>, dim3(ws.n_blocks), dim3(64), 0, s, ids, A,
                     c.expert_lo, E_loc, ws.block_hist, perm, inv);
  MOE_LAUNCH(MOE_K_DISPATCH_SCAN, dispatch_scan_kernel, dim3(1), dim3(256), 0, s, ws.block_hist, ws.n_blocks,
                     E_loc, counts, offsets);
  MOE_LAUNCH(MOE_K_DISPATCH_SCATTER, dispatch_index_kernel<1>, dim3(ws.n_blocks), dim3(64), 0, s, ids, A,
                     c.expert_lo, E_loc, ws.block_hist, perm, inv);
  const int row16 = c.hidden * (c.act_dtype == MOE_F32 ? 4 : 2) / 16;
  MOE_LAUNCH(MOE_K_DISPATCH_GATHER, dispatch_gather_kernel<8>, dim3((T + 3) / 4), dim3(256), 0, s,
                     static_cast<const uint4*>(x), inv, static_cast<uint4*>(xs), T, k, row16);
  return hipGetLastError();
}

}  // namespace moe
