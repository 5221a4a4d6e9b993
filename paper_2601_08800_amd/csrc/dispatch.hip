// Dispatch: build the expert-contiguous send buffer (Sec. II "EP"; Alg. 2).
//
// A stable counting sort of the local assignments by expert, with no atomics
// anywhere (so the permutation is unique and repeatable):
//   1. count   one wavefront per sub-chunk of 64 consecutive assignments counts
//              them per local expert with ballots (one per bit of the expert
//              index, no atomics) and notes every
//              assignment's rank among its expert's assignments of the sub-chunk
//   2. scan    per expert (a workgroup of four wavefronts each) an exclusive scan over the
//              sub-chunks -> counts; offsets = exclusive scan over experts,
//              rebuilt in LDS by every scatter workgroup
//   3. place   position = offsets[e] + start of the sub-chunk's run + rank
//   4. gather  one wavefront per token reads the row ONCE (16 B per lane,
//              coalesced) and writes it to each of its local positions
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

constexpr int kSub = 64;   // assignments per histogram column: one wavefront

__device__ __forceinline__ uint64_t lanemask_lt() {
  return (uint64_t(1) << (threadIdx.x & 63)) - 1;
}

// Lanes of the wavefront that hold the same local expert as this lane: one
// ballot per bit of the expert index (at most 9), each narrowing the set to the
// lanes that agree with this lane on that bit.  Meaningful where e >= 0.
__device__ __forceinline__ uint64_t same_expert_lanes(int e, int E_loc) {
  uint64_t same = __ballot(e >= 0);
  const int nbits = E_loc > 1 ? 32 - __clz(E_loc - 1) : 0;
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (e >> b) & 1;
    const uint64_t m = __ballot(bit);
    same &= bit ? m : ~m;
  }
  return same;
}

// One wavefront per sub-chunk of 64 consecutive flat assignments.  The lanes
// that go to the same local expert find each other with ballots, which yields,
// without atomics, the count per expert
// and the rank of every assignment among its expert's assignments of the
// sub-chunk.  Counts go to hist[E_loc][n_sub] (built in a wavefront-private LDS
// row, so absent experts get their zero), ranks are parked in inv[].
__global__ __launch_bounds__(256) void dispatch_count_kernel(
    const int32_t* __restrict__ ids, int A, int e_lo, int E_loc, int n_sub,
    int32_t* __restrict__ hist, int32_t* __restrict__ inv) {
  __shared__ int32_t cnt[4][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = blockIdx.x * 4 + wave;
  if (sub >= n_sub) return;
  const int a = sub * kSub + lane;
  int e = -1;
  if (a < A) {
    e = ids[a] - e_lo;
    if (e < 0 || e >= E_loc) e = -1;
  }
  int32_t* row = cnt[wave];                    // same-wavefront LDS accesses execute in order
  for (int x = lane; x < E_loc; x += 64) row[x] = 0;
  const uint64_t same = same_expert_lanes(e, E_loc);
  int rank = -1;
  if (e >= 0) {
    rank = __popcll(same & lanemask_lt());
    if (rank == 0) row[e] = __popcll(same);    // the lowest lane of each expert present
  }
  if (a < A) inv[a] = rank;                    // -1: expert not local
  for (int x = lane; x < E_loc; x += 64) hist[size_t(x) * n_sub + sub] = row[x];
}

// Position of every local assignment: offsets[e] + start of its sub-chunk's run
// inside the expert's segment + its rank (left in inv[] by the count kernel).
// Every workgroup rebuilds offsets = exclusive scan of counts in LDS (E_loc <=
// 512 values, one wavefront); workgroup 0 also stores them.
__global__ __launch_bounds__(256) void dispatch_place_kernel(
    const int32_t* __restrict__ ids, int A, int e_lo, int E_loc, int n_sub,
    const int32_t* __restrict__ hist, const int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets_out, int32_t* __restrict__ perm, int32_t* __restrict__ inv) {
  __shared__ int32_t offsets[513];
  if (threadIdx.x < 64) {
    const int l = threadIdx.x;
    const int per = (E_loc + 63) / 64;
    const int x0 = l * per, x1 = (x0 + per < E_loc) ? x0 + per : E_loc;
    int sum = 0;
    for (int x = x0; x < x1; ++x) sum += counts[x];
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(incl, off);
      if (l >= off) incl += o;
    }
    int run = incl - sum;
    for (int x = x0; x < x1; ++x) {
      offsets[x] = run;
      if (blockIdx.x == 0) offsets_out[x] = run;
      run += counts[x];
    }
    if (l == 63) {
      offsets[E_loc] = incl;
      if (blockIdx.x == 0) offsets_out[E_loc] = incl;
    }
  }
  __syncthreads();
  const int a = blockIdx.x * 256 + threadIdx.x;
  if (a >= A) return;
  const int rank = inv[a];
  if (rank < 0) return;                        // inv[a] stays -1
  const int e = ids[a] - e_lo;
  const int pos = offsets[e] + hist[size_t(e) * n_sub + a / kSub] + rank;
  perm[pos] = a;
  inv[a] = pos;
}

// One workgroup of four wavefronts per local expert: exclusive scan of the
// expert's row of counts (thread i owns a contiguous run of sub-chunks; a scan over
// the lanes of each wavefront, then over the four wavefront totals), counts[e] =
// the row's total.  Integer sums: the result does not depend on the split.
__global__ __launch_bounds__(256) void dispatch_scan_kernel(int32_t* __restrict__ hist, int n_sub,
                                                           int32_t* __restrict__ counts) {
  __shared__ int32_t wave_total[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, e = blockIdx.x;
  int32_t* row = hist + size_t(e) * n_sub;
  const int per = (n_sub + 255) / 256;
  const int s0 = min(n_sub, tid * per), s1 = min(n_sub, s0 + per);
  int sum = 0;
  for (int sb = s0; sb < s1; ++sb) sum += row[sb];
  int incl = sum;                               // inclusive scan over the lanes of the wavefront
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int run = incl - sum;
  for (int w = 0; w < wave; ++w) run += wave_total[w];
  for (int sb = s0; sb < s1; ++sb) {
    const int c = row[sb];
    row[sb] = run;
    run += c;
  }
  if (tid == 255) counts[e] = run;
}

// One wavefront per token: read the row once, write it to every local position.
// Lengths in 16-byte pieces: `src16` = pitch of a token row, `col16` = first
// piece of the copied column window, `row16` = width of the window = pitch of
// the destination rows (the whole row: col16 = 0, row16 = src16).
template <int PIECES>
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const uint4* __restrict__ x,
                                                             const int32_t* __restrict__ inv,
                                                             uint4* __restrict__ xs, int T, int k,
                                                             int src16, int col16, int row16) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= T) return;
  int pos = -1;
  if (lane < k) pos = inv[size_t(t) * k + lane];      // k <= 32
  const uint64_t have = __ballot(pos >= 0);
  if (!have) return;
  const uint4* src = x + size_t(t) * src16 + col16;
  for (int c0 = 0; c0 < row16; c0 += 64 * PIECES) {
    uint4 v[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int c = c0 + i * 64 + lane;
      if (c < row16) v[i] = nt_load16(src + c);
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
        if (c < row16) nt_store16(dst + c, v[i]);
      }
    }
  }
}

// Few assignments (A <= kSmallA): the whole dispatch in one launch.  Every
// workgroup rebuilds the same index in its own LDS (count per sub-chunk, scan
// per expert, scan over experts, place: the steps and the order of the kernels
// above, so the permutation is the same), workgroup 0 stores it, and each
// workgroup then copies the rows of its four tokens.  The redundant index work
// is a few microseconds on otherwise idle CUs and replaces three launches.
// LDS: hist[n_sub][E_loc] | slot[n_sub*64] | cnt[E_loc] | offs[E_loc+1].
constexpr int kSmallA = 4096;
constexpr size_t kSmallLds = 60 * 1024;
inline size_t small_lds_bytes(int E_loc, int n_sub) {
  return (size_t(n_sub) * E_loc + size_t(n_sub) * kSub + 2 * size_t(E_loc) + 1) * sizeof(int32_t);
}

template <int PIECES>
__global__ __launch_bounds__(256) void dispatch_small_kernel(
    const int32_t* __restrict__ ids, int A, int e_lo, int E_loc, int n_sub,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets_out, int32_t* __restrict__ perm,
    int32_t* __restrict__ inv, const uint4* __restrict__ x, uint4* __restrict__ xs, int T, int k,
    int src16, int col16, int row16) {
  extern __shared__ int32_t lds[];
  int32_t* const hist = lds;                         // [n_sub][E_loc]
  int32_t* const slot = hist + n_sub * E_loc;        // [n_sub*64]: (e << 6 | rank), then position
  int32_t* const cnt = slot + n_sub * kSub;          // [E_loc]
  int32_t* const offs = cnt + E_loc;                 // [E_loc + 1]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool first = blockIdx.x == 0;
  for (int i = tid; i < n_sub * E_loc; i += 256) hist[i] = 0;
  __syncthreads();
  // 1. count: ballots find the lanes of a sub-chunk that share an expert
  for (int sub = wave; sub < n_sub; sub += 4) {
    const int a = sub * kSub + lane;
    int e = -1;
    if (a < A) {
      e = ids[a] - e_lo;
      if (e < 0 || e >= E_loc) e = -1;
    }
    const uint64_t same = same_expert_lanes(e, E_loc);
    int rank = 0;
    if (e >= 0) {
      rank = __popcll(same & lanemask_lt());
      if (rank == 0) hist[sub * E_loc + e] = __popcll(same);
    }
    slot[a] = e >= 0 ? (e << 6 | rank) : -1;
  }
  __syncthreads();
  // 2. scan over the sub-chunks, one thread per expert
  for (int e = tid; e < E_loc; e += 256) {
    int run = 0;
    for (int sb = 0; sb < n_sub; ++sb) {
      const int c = hist[sb * E_loc + e];
      hist[sb * E_loc + e] = run;
      run += c;
    }
    cnt[e] = run;
    if (first) counts[e] = run;
  }
  __syncthreads();
  // 3. offsets = exclusive scan of the counts (one wavefront)
  if (wave == 0) {
    const int per = (E_loc + 63) / 64;
    const int x0 = lane * per, x1 = (x0 + per < E_loc) ? x0 + per : E_loc;
    int sum = 0;
    for (int i = x0; i < x1; ++i) sum += cnt[i];
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    int run = incl - sum;
    for (int i = x0; i < x1; ++i) {
      offs[i] = run;
      if (first) offsets_out[i] = run;
      run += cnt[i];
    }
    if (lane == 63) {
      offs[E_loc] = incl;
      if (first) offsets_out[E_loc] = incl;
    }
  }
  __syncthreads();
  // 4. place
  for (int a = tid; a < A; a += 256) {
    const int sl = slot[a];
    int pos = -1;
    if (sl >= 0) {
      const int e = sl >> 6;
      pos = offs[e] + hist[(a / kSub) * E_loc + e] + (sl & 63);
      if (first) perm[pos] = a;
    }
    slot[a] = pos;
    if (first) inv[a] = pos;
  }
  __syncthreads();
  // 5. copy the rows of this workgroup's tokens (one wavefront per token)
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  int pos = -1;
  if (lane < k) pos = slot[t * k + lane];
  const uint64_t have = __ballot(pos >= 0);
  if (!have) return;
  const uint4* src = x + size_t(t) * src16 + col16;
  for (int c0 = 0; c0 < row16; c0 += 64 * PIECES) {
    uint4 v[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int c = c0 + i * 64 + lane;
      if (c < row16) v[i] = nt_load16(src + c);
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
        if (c < row16) nt_store16(dst + c, v[i]);
      }
    }
  }
}

// Per-row block scales follow their rows: out[kb][pos] = in[kb][token of pos] for
// the valid positions (both arrays are block-major: one row of the array per
// 128-column block).
__global__ __launch_bounds__(256) void dispatch_scales_kernel(
    const float* __restrict__ in, int in_pitch, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ offsets, int E_loc, int k, int n_blocks, float* __restrict__ out,
    int out_pitch) {
  const int pos = blockIdx.x * 256 + threadIdx.x;
  if (pos >= offsets[E_loc] || pos >= out_pitch) return;
  const int t = perm[pos] / k;
  for (int kb = 0; kb < n_blocks; ++kb) out[size_t(kb) * out_pitch + pos] = in[size_t(kb) * in_pitch + t];
}

}  // namespace

hipError_t launch_dispatch_scales(const float* in, int in_pitch, const int32_t* perm,
                                  const int32_t* offsets, int E_loc, int k, int n_blocks, float* out,
                                  int out_pitch, hipStream_t s) {
  MOE_LAUNCH(MOE_K_DISPATCH_GATHER, dispatch_scales_kernel, dim3((out_pitch + 255) / 256), dim3(256), 0, s,
             in, in_pitch, perm, offsets, E_loc, k, n_blocks, out, out_pitch);
  return hipGetLastError();
}

hipError_t launch_dispatch(const moe_config& c, int T, const void* x, const int32_t* ids,
                           int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                           void* xs, int tp_rank, int tp_size, const DispatchWs& ws,
                           hipStream_t s, int elem_bytes) {
  const int k = c.top_k;
  const int A = T * k;
  const int E_loc = c.expert_hi - c.expert_lo;
  const int n_sub = (A + kSub - 1) / kSub;
  // column window of TP rank tp_rank of tp_size (the whole row for 0 of 1);
  // elem_bytes overrides the element size of the rows (1: quantised codes)
  if (elem_bytes == 0) elem_bytes = c.act_dtype == MOE_F32 ? 4 : 2;
  const int src16 = c.hidden * elem_bytes / 16;
  const int row16 = src16 / tp_size;
  if (A <= kSmallA && small_lds_bytes(E_loc, n_sub) <= kSmallLds) {
    MOE_LAUNCH(MOE_K_DISPATCH_GATHER, dispatch_small_kernel<8>, dim3((T + 3) / 4), dim3(256),
               small_lds_bytes(E_loc, n_sub), s, ids, A, c.expert_lo, E_loc, n_sub, counts, offsets,
               perm, inv, static_cast<const uint4*>(x), static_cast<uint4*>(xs), T, k, src16,
               tp_rank * row16, row16);
    return hipGetLastError();
  }
  const dim3 grid_idx((n_sub + 3) / 4), block_idx(256);
  MOE_LAUNCH(MOE_K_DISPATCH_HIST, dispatch_count_kernel, grid_idx, block_idx, 0, s, ids, A,
             c.expert_lo, E_loc, n_sub, ws.block_hist, inv);
  MOE_LAUNCH(MOE_K_DISPATCH_SCAN, dispatch_scan_kernel, dim3(E_loc), dim3(256), 0, s, ws.block_hist,
             n_sub, counts);
  MOE_LAUNCH(MOE_K_DISPATCH_SCATTER, dispatch_place_kernel, dim3((A + 255) / 256), block_idx, 0, s,
             ids, A, c.expert_lo, E_loc, n_sub, ws.block_hist, counts, offsets, perm, inv);
  MOE_LAUNCH(MOE_K_DISPATCH_GATHER, dispatch_gather_kernel<8>, dim3((T + 3) / 4), dim3(256), 0, s,
             static_cast<const uint4*>(x), inv, static_cast<uint4*>(xs), T, k, src16,
             tp_rank * row16, row16);
  return hipGetLastError();
}

}  // namespace moe
