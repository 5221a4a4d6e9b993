// Dispatch: build the expert-contiguous send buffer (Sec. II "EP"; Alg. 2).
//
// A stable counting sort of the local assignments by expert, with no atomics
// anywhere (so the permutation is unique and repeatable):
//   1. hist    per sub-chunk of 256 consecutive assignments and per local
//              expert, count by comparison (a thread per pair, no atomics)
//   2. scan    per expert an exclusive scan over sub-chunks, then an exclusive
//              scan over experts -> counts, offsets, per-pair start positions
//   3. scatter every (sub-chunk, expert) pair walks its 256 ids in order and
//              writes perm / inv from its start position
//   4. gather  one wavefront per token reads the row ONCE (16 B per lane,
//              coalesced) and writes it to each of its local positions
#include "moe_internal.h"

namespace moe {

namespace {

constexpr int kMaxLocalExperts = 512;

constexpr int kSub = 256;                         // assignments per histogram row
constexpr int kSubsPerBlock = kDispatchChunk / kSub;

// hist[sub][e] = number of assignments of sub-chunk `sub` (256 consecutive
// flat assignments) that go to local expert e.  A workgroup stages 1024 ids in
// LDS; each thread owns (sub-chunk, expert) pairs and counts by comparison, so
// no atomics are needed.  MODE 1 walks the same pairs again, now with the
// start position of each pair known, and writes perm / inv in order.
template <int MODE>
__global__ __launch_bounds__(256) void dispatch_index_kernel(
    const int32_t* __restrict__ ids, int A, int e_lo, int E_loc, int32_t* __restrict__ hist,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv) {
  __shared__ int32_t sid[kDispatchChunk];
  const int base = blockIdx.x * kDispatchChunk;
  for (int i = threadIdx.x; i < kDispatchChunk; i += 256) {
    const int a = base + i;
    int e = -1;
    if (a < A) {
      e = ids[a] - e_lo;
      if (e < 0 || e >= E_loc) {
        e = -1;
        if (MODE == 1) inv[a] = -1;
      }
    }
    sid[i] = e;
  }
  __syncthreads();
  for (int pair = threadIdx.x; pair < kSubsPerBlock * E_loc; pair += 256) {
    const int sub = pair / E_loc, e = pair - sub * E_loc;
    const int32_t* row = sid + sub * kSub;
    const size_t h = (size_t(blockIdx.x) * kSubsPerBlock + sub) * E_loc + e;
    if (MODE == 0) {
      int n = 0;
#pragma unroll 8
      for (int i = 0; i < kSub; ++i) n += (row[i] == e);
      hist[h] = n;
    } else {
      int pos = hist[h];
      const int a0 = base + sub * kSub;
      for (int i = 0; i < kSub; ++i) {
        if (row[i] == e) {
          perm[pos] = a0 + i;
          inv[a0 + i] = pos;
          ++pos;
        }
      }
    }
  }
}

// Single block.  hist[sub][e] (counts) -> start position of sub-chunk `sub`'s
// first assignment of expert e; counts[e]; offsets = exclusive scan of counts.
// Thread (e, seg) sums a contiguous segment of sub-chunks, the segment totals
// are scanned in LDS, then each thread rewrites its segment as running starts.
__global__ __launch_bounds__(256) void dispatch_scan_kernel(int32_t* __restrict__ hist, int n_sub,
                                                           int E_loc, int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets) {
  __shared__ int32_t seg_tot[256];
  __shared__ int32_t tot[kMaxLocalExperts + 1];
  const int segs = E_loc >= 256 ? 1 : 256 / E_loc;
  const int per = (n_sub + segs - 1) / segs;
  for (int e0 = 0; e0 < E_loc; e0 += 256) {
    const int e = e0 + int(threadIdx.x) % (E_loc < 256 ? E_loc : 256);
    const int seg = int(threadIdx.x) / (E_loc < 256 ? E_loc : 256);
    const bool on = seg < segs && e < E_loc;
    const int s0 = seg * per, s1 = (s0 + per < n_sub) ? s0 + per : n_sub;
    int sum = 0;
    if (on)
      for (int sb = s0; sb < s1; ++sb) sum += hist[size_t(sb) * E_loc + e];
    seg_tot[threadIdx.x] = on ? sum : 0;
    __syncthreads();
    int before = 0;
    if (on) {
      const int stride = E_loc < 256 ? E_loc : 256;
      for (int q = 0; q < seg; ++q) before += seg_tot[q * stride + (e - e0)];
      int all = before;
      for (int q = seg; q < segs; ++q) all += seg_tot[q * stride + (e - e0)];
      if (seg == 0) { tot[e] = all; counts[e] = all; }
      int run = before;
      for (int sb = s0; sb < s1; ++sb) {
        const int c = hist[size_t(sb) * E_loc + e];
        hist[size_t(sb) * E_loc + e] = run;
        run += c;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    int run = 0;
    for (int e = 0; e < E_loc; ++e) {
      const int c = tot[e];
      tot[e] = run;
      offsets[e] = run;
      run += c;
    }
    offsets[E_loc] = run;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_sub * E_loc; i += blockDim.x) hist[i] += tot[i % E_loc];
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
  MOE_LAUNCH(MOE_K_DISPATCH_HIST, dispatch_index_kernel<0>, dim3(ws.n_blocks), dim3(256), 0, s, ids, A,
                     c.expert_lo, E_loc, ws.block_hist, perm, inv);
  MOE_LAUNCH(MOE_K_DISPATCH_SCAN, dispatch_scan_kernel, dim3(1), dim3(256), 0, s, ws.block_hist, ws.n_blocks * kSubsPerBlock,
                     E_loc, counts, offsets);
  MOE_LAUNCH(MOE_K_DISPATCH_SCATTER, dispatch_index_kernel<1>, dim3(ws.n_blocks), dim3(256), 0, s, ids, A,
                     c.expert_lo, E_loc, ws.block_hist, perm, inv);
  const int row16 = c.hidden * (c.act_dtype == MOE_F32 ? 4 : 2) / 16;
  MOE_LAUNCH(MOE_K_DISPATCH_GATHER, dispatch_gather_kernel<8>, dim3((T + 3) / 4), dim3(256), 0, s,
                     static_cast<const uint4*>(x), inv, static_cast<uint4*>(xs), T, k, row16);
  return hipGetLastError();
}

}  // namespace moe
