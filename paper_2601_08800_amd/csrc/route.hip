// Route: gate scoring and top-k selection (Sec. III-B-2: each token goes to
// its top-k activated experts; Alg. 2: the expert map is computed from the
// local hidden states).
//
// The selected ids must be those of exact arithmetic on the stored inputs,
// whatever the summation order.  Three stages make that cheap:
//   1. gate GEMM   bf16 MFMA 32x32x16, fp32 accumulation in short chains that
//                  are flushed into fp64 sums; also the squared row norms
//   2. select      one wavefront per token: keys, group limit, top-k by
//                  shuffle arg-max, and an interval test: every comparison
//                  the selection relied on must hold for ANY keys within the
//                  error bound of stage 1; tokens that fail are listed
//   3. re-score    one workgroup per listed token: the experts whose key
//                  interval reaches the selection get an fp64 dot product and
//                  the selection is redone in fp64
// Decode-sized batches (T*E*H up to 2^28) skip all three: one kernel computes
// every logit in fp64 and selects on fp64 keys.
// Error model of stage 1 for a chain of n bf16 products (exact in fp32) added
// in fp32: every addition is off by at most one ulp of the running sum, so
// |error| <= 2n * 2^-24 * sum|x_h w_h| <= 2n * 2^-24 * |x|_2 |w|_2.
#include <limits.h>

#include "moe_internal.h"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kUlp = 5.9604645e-8f;   // 2^-24

// ------------------------------------------------------------------ helpers
// Pairwise lane exchange, step s pairs disjoint groups of 2^s lanes: steps 0..3
// are DPP moves inside a row of 16 lanes (quad permutes, then the half-row and
// row mirrors: after the quads are uniform a mirror pairs each lane with a lane
// of the other group), steps 4 and 5 cross rows through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}

template <int STEP>
__device__ __forceinline__ int lane_xchg32(int v) {
  if (STEP == 0) return dpp_mov<0xB1>(v);        // quad_perm [1,0,3,2]
  if (STEP == 1) return dpp_mov<0x4E>(v);        // quad_perm [2,3,0,1]
  if (STEP == 2) return dpp_mov<0x141>(v);       // row_half_mirror
  if (STEP == 3) return dpp_mov<0x140>(v);       // row_mirror
  return __shfl_xor(v, STEP == 4 ? 16 : 32);
}

template <int STEP>
__device__ __forceinline__ int lane_xchg(int v) { return lane_xchg32<STEP>(v); }
template <int STEP>
__device__ __forceinline__ float lane_xchg(float v) {
  return __builtin_bit_cast(float, lane_xchg32<STEP>(__builtin_bit_cast(int, v)));
}
template <int STEP>
__device__ __forceinline__ double lane_xchg(double v) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)lane_xchg32<STEP>((int)(uint32_t)u);
  const uint32_t hi = (uint32_t)lane_xchg32<STEP>((int)(uint32_t)(u >> 32));
  return __builtin_bit_cast(double, (uint64_t(hi) << 32) | lo);
}

#define MOE_ALL_STEPS(F) F(0) F(1) F(2) F(3) F(4) F(5)

// Value of lane `l` (the same l in every lane) as a scalar broadcast: no LDS crossbar.
__device__ __forceinline__ int read_lane(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float read_lane(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ double read_lane(double v, int l) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, l);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), l);
  return __builtin_bit_cast(double, (uint64_t(hi) << 32) | lo);
}

__device__ __forceinline__ int lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Sum over the wave in a fixed order, the same in every lane: a butterfly inside
// each row of 16 lanes, then (row0 + row1) + (row2 + row3) from the row results
// read as scalars.
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#define STEP_(S) v += lane_xchg<S>(v);
  STEP_(0) STEP_(1) STEP_(2) STEP_(3)
#undef STEP_
  const T r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
  return (r0 + r1) + (r2 + r3);
}

// Largest value over the wave, the same in every lane: the four DPP steps make
// each row of 16 lanes uniform, the four row results are then read as scalars.
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#define STEP_(S) { const T o = lane_xchg<S>(v); v = o > v ? o : v; }
  STEP_(0) STEP_(1) STEP_(2) STEP_(3)
#undef STEP_
  const T r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
  const T a = r1 > r0 ? r1 : r0, b = r3 > r2 ? r3 : r2;
  return b > a ? b : a;
}

__device__ __forceinline__ int wave_min(int v) {
#define STEP_(S) { const int o = lane_xchg<S>(v); v = o < v ? o : v; }
  MOE_ALL_STEPS(STEP_)
#undef STEP_
  return v;
}

// Largest value over the wave, ties to the lowest index; idx == INT_MAX marks
// "no candidate".  Result is the same in every lane.  The maximum is a plain
// wave_max; the lanes that hold it answer a ballot, and the usual single winner's
// index is read from its lane (a minimum over the tied lanes otherwise).
template <typename T>
__device__ __forceinline__ void wave_argmax(T& v, int& idx) {
  const bool cand = idx != INT_MAX;
  const T vv = cand ? v : (T)-INFINITY;
  const T m = wave_max(vv);
  const uint64_t tie = __ballot(cand && vv == m);
  int win = INT_MAX;
  if (tie != 0) {
    if ((tie & (tie - 1)) == 0) win = read_lane(idx, __ffsll((unsigned long long)tie) - 1);
    else win = wave_min((tie >> lane_id() & 1) ? idx : INT_MAX);
  }
  v = tie != 0 ? m : (T)0;
  idx = win;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) {
  return __uint_as_float(hi16 << 16);
}

// Sum of squares of the eight bf16 values of a 16-byte piece, added to acc (fp32).
__device__ __forceinline__ float piece_sumsq(const uint4& a, float acc) {
  const uint32_t v[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float lo = bf16_bits_to_f32(v[q] & 0xffffu), hi = bf16_bits_to_f32(v[q] >> 16);
    acc = fmaf(lo, lo, acc);
    acc = fmaf(hi, hi, acc);
  }
  return acc;
}

// fp64 dot product of two 16-byte pieces (8 bf16 or 4 fp32), added to acc.
template <bool BF16>
__device__ __forceinline__ double piece_dot64(const uint4& a, const uint4& b, double acc) {
  const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (BF16) {
      acc = fma((double)bf16_bits_to_f32(av[i] & 0xffffu), (double)bf16_bits_to_f32(bv[i] & 0xffffu), acc);
      acc = fma((double)bf16_bits_to_f32(av[i] >> 16), (double)bf16_bits_to_f32(bv[i] >> 16), acc);
    } else {
      acc = fma((double)__uint_as_float(av[i]), (double)__uint_as_float(bv[i]), acc);
    }
  }
  return acc;
}

// fp64 dot product of one token row with one gate row, one wavefront, fixed
// order (lane-strided partial sums, then a butterfly): exact products, fp64 sums.
template <bool BF16>
__device__ __forceinline__ double wave_dot64(const void* xrow, const void* wrow, int H, int lane) {
  double acc = 0.0;
  if (BF16) {
    const uint4* xa = static_cast<const uint4*>(xrow);
    const uint4* wa = static_cast<const uint4*>(wrow);
#pragma unroll 4
    for (int c = lane; c < H / 8; c += 64) {
      const uint4 a = xa[c], b = wa[c];
      const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc = fma((double)bf16_bits_to_f32(av[i] & 0xffffu), (double)bf16_bits_to_f32(bv[i] & 0xffffu), acc);
        acc = fma((double)bf16_bits_to_f32(av[i] >> 16), (double)bf16_bits_to_f32(bv[i] >> 16), acc);
      }
    }
  } else {
    const float4* xa = static_cast<const float4*>(xrow);
    const float4* wa = static_cast<const float4*>(wrow);
#pragma unroll 4
    for (int c = lane; c < H / 4; c += 64) {
      const float4 a = xa[c], b = wa[c];
      acc = fma((double)a.x, (double)b.x, acc);
      acc = fma((double)a.y, (double)b.y, acc);
      acc = fma((double)a.z, (double)b.z, acc);
      acc = fma((double)a.w, (double)b.w, acc);
    }
  }
  return wave_sum(acc);
}

// ------------------------------------------------- stage 0: gate row norms
// One wavefront per gate row: wnorm2[e] = sum_h w[e,h]^2.  Also clears the
// re-score counter (a fill kernel rather than a memset, so the call can be
// captured in a graph).
template <bool BF16>
__global__ __launch_bounds__(256) void gate_wnorm_kernel(const void* __restrict__ gate_w, int E,
                                                        int H, float* __restrict__ wnorm2,
                                                        int32_t* __restrict__ counters) {
  if (blockIdx.x == 0 && threadIdx.x < 64) counters[threadIdx.x] = 0;
  if (!gate_w) return;
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (e >= E) return;
  const size_t rb = size_t(e) * H * (BF16 ? 2 : 4);
  const char* row = static_cast<const char*>(gate_w) + rb;
  const double s = wave_dot64<BF16>(row, row, H, lane);
  if (lane == 0) wnorm2[e] = (float)(s * (1.0 + 1e-6));
}

// ------------------------ stage 1 (fp32 inputs, many tokens): fp64 VALU gate
// One workgroup per token; each wavefront takes every 4th expert.  Exact
// products, fp64 sums: the logits are good to the fp32 store.
template <bool BF16>
__global__ __launch_bounds__(256) void gate_f64_kernel(const void* __restrict__ x,
                                                      const void* __restrict__ gate_w, int T,
                                                      int H, int E, float* __restrict__ logits,
                                                      float* __restrict__ xnorm2) {
  const int t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t eb = BF16 ? 2 : 4;
  const char* xr = static_cast<const char*>(x) + size_t(t) * H * eb;
  for (int e = wave; e < E; e += 4) {
    const double z = wave_dot64<BF16>(xr, static_cast<const char*>(gate_w) + size_t(e) * H * eb, H, lane);
    if (lane == 0) logits[size_t(t) * E + e] = (float)z;
  }
  if (wave == 0) {
    const double s = wave_dot64<BF16>(xr, xr, H, lane);
    if (lane == 0) xnorm2[t] = (float)(s * (1.0 + 1e-6));
  }
}

// ------------------------------------------ stage 1 (bf16): MFMA gate GEMM
// Register-staged variant, used when H is not a multiple of 64 (it zero-fills
// the K tail); otherwise gate_dma_kernel below runs the same tile.
// Block tile 64 tokens x 128 experts, K step 64, 8 wavefronts as 2 (M) x 4 (N),
// each one 32x32 MFMA tile (16 fp32 accumulators flushed into 16 fp64 sums every
// K step): the flush is as much VALU work as the MFMAs are matrix work, so many
// light wavefronts per SIMD (three workgroups fit a CU) overlap the two and the
// register-staged loads better than four wavefronts with two tiles each did.
// LDS tiles are [row][8 pieces of 16 B] with the piece index XOR-ed by (row/2)&7
// so that the 16 lanes the LDS serves per cycle fall on 16 different 16-byte
// columns.
// K of the gate GEMM is split until about this many workgroups run (2 per CU)
constexpr int GBM = kGateTileM, GBN = kGateTileN, GBK = 64;

__device__ __forceinline__ int swz(int row, int piece) {
  return row * 8 + (piece ^ ((row >> 1) & 7));
}

template <int CHAIN_STEPS>
__global__ __launch_bounds__(512) void gate_mfma_kernel(const uint16_t* __restrict__ x,
                                                        const uint16_t* __restrict__ gate_w, int T,
                                                        int H, int E, float* __restrict__ logits,
                                                        float* __restrict__ xnorm2,
                                                        float* __restrict__ wnorm2,
                                                        int32_t* __restrict__ counters) {
  __shared__ uint4 As[2][GBM * 8];
  __shared__ uint4 Bs[2][GBN * 8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int m0 = blockIdx.x * GBM, n0 = blockIdx.y * GBN;
  const int all_steps = (H + GBK - 1) / GBK;
  const int per_split = (all_steps + gridDim.z - 1) / gridDim.z;
  const int ks0 = blockIdx.z * per_split;
  const int ksteps = (ks0 + per_split < all_steps ? ks0 + per_split : all_steps) - ks0;
  logits += size_t(blockIdx.z) * T * E;
  xnorm2 += size_t(blockIdx.z) * T;
  wnorm2 += size_t(blockIdx.z) * E;
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid < 64) counters[tid] = 0;

  // global -> register staging: A 1 piece / thread, B 2 pieces / thread
  const int lrow = tid >> 3, lpiece = tid & 7;        // lrow 0..63
  uint4 ra, rb[2];
  float xsq = 0.f, wsq[2] = {0.f, 0.f};
  auto gload = [&](int ks) {
    const int kcol = (ks0 + ks) * GBK + lpiece * 8;
    const bool kin = kcol < H;
    int r = m0 + lrow;
    r = r < T ? r : T - 1;
    ra = kin ? *reinterpret_cast<const uint4*>(x + size_t(r) * H + kcol) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int n = n0 + lrow + 64 * i;
      n = n < E ? n : E - 1;
      rb[i] = kin ? *reinterpret_cast<const uint4*>(gate_w + size_t(n) * H + kcol) : make_uint4(0, 0, 0, 0);
    }
  };
  auto lstore = [&](int buf) {
    As[buf][swz(lrow, lpiece)] = ra;
    const uint32_t v[4] = {ra.x, ra.y, ra.z, ra.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float lo = bf16_bits_to_f32(v[q] & 0xffffu), hi = bf16_bits_to_f32(v[q] >> 16);
      xsq = fmaf(lo, lo, xsq);
      xsq = fmaf(hi, hi, xsq);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) Bs[buf][swz(lrow + 64 * i, lpiece)] = rb[i];
    if (blockIdx.x == 0) {                            // the first token tile also sums the gate rows' squares
#pragma unroll
      for (int i = 0; i < 2; ++i) wsq[i] = piece_sumsq(rb[i], wsq[i]);
    }
  };

  f32x16 acc;
  double dsum[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { acc[i] = 0.f; dsum[i] = 0.0; }

  gload(0);
  lstore(0);
  __syncthreads();
  for (int ks = 0; ks < ksteps; ++ks) {
    const int buf = ks & 1;
    if (ks + 1 < ksteps) gload(ks + 1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int piece = kk * 2 + (lane >> 5);
      const uint4 av = As[buf][swz(wm * 32 + (lane & 31), piece)];
      const uint4 bv = Bs[buf][swz(wn * 32 + (lane & 31), piece)];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                    __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
    }
    if ((ks + 1) % CHAIN_STEPS == 0 || ks + 1 == ksteps) {
#pragma unroll
      for (int i = 0; i < 16; ++i) { dsum[i] += (double)acc[i]; acc[i] = 0.f; }
    }
    if (ks + 1 < ksteps) lstore(buf ^ 1);
    __syncthreads();
  }

  // D layout of the 32x32 MFMA: lane l, register i -> row (i/4)*8 + (l/32)*4 + i%4, col l%32
  const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    if (row < T && col < E) logits[size_t(row) * E + col] = (float)dsum[i];
  }
  // squared row norms: the 8 threads with equal lrow hold one row's pieces
  if (blockIdx.y == 0) {
    float s = xsq;
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 4);
    const int r = m0 + lrow;
    if (lpiece == 0 && r < T) xnorm2[r] = s * 1.001f;
  }
  if (blockIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float s = wsq[i];
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      const int n = n0 + lrow + 64 * i;
      if (lpiece == 0 && n < E) wnorm2[n] = s * 1.001f;
    }
  }
}

// The gate GEMM with the operands brought global -> LDS directly
// (`global_load_lds_dwordx4`, no staging registers) into a ring of NS stages:
// one barrier per K step and an explicit vmcnt wait that leaves the younger
// stages in flight.  Tile BM tokens x 128 experts, eight wavefronts as BM/32 (M)
// x 256/BM (N), one or two 32x32 MFMA tiles each.  Needs H to be a multiple of 64
// (a DMA cannot zero-fill a K tail).  LDS slot s of a stage holds (row s/8, piece
// (s%8) ^ (row/2)&7): the lane that owns the slot fetches that piece, which is
// the swz() layout the fragment reads expect.
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

template <int BM, int NS, int CHAIN_STEPS>
__device__ __forceinline__ void gate_dma_body(const uint16_t* __restrict__ x,
                                              const uint16_t* __restrict__ gate_w, int T, int H,
                                              int E, float* __restrict__ logits,
                                              float* __restrict__ xnorm2,
                                              float* __restrict__ wnorm2,
                                              int32_t* __restrict__ counters, uint4* smem) {
  constexpr int MW = BM / 32;                // wavefronts along M
  constexpr int NT = (GBN / 32) * MW / 8;    // MFMA tiles (32 experts each) per wavefront
  constexpr int NA = BM / 64;                // A load instructions per thread and step
  constexpr int NLOAD = NA + 2;              // load instructions per thread and step
  uint4* const As = smem;                    // [NS][BM * 8]
  uint4* const Bs = smem + NS * BM * 8;      // [NS][GBN * 8]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % MW, wn = wave / MW;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * GBN;
  const int all_steps = H / GBK;
  const int per_split = (all_steps + gridDim.z - 1) / gridDim.z;
  const int ks0 = blockIdx.z * per_split;
  const int ksteps = (ks0 + per_split < all_steps ? ks0 + per_split : all_steps) - ks0;
  logits += size_t(blockIdx.z) * T * E;
  xnorm2 += size_t(blockIdx.z) * T;
  wnorm2 += size_t(blockIdx.z) * E;
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid < 64) counters[tid] = 0;

  // this thread's slots: tid + 512 i of the A stage (i < NA) and of the B stage (i < 2);
  // rows lrow + 64 i, and (lrow + 64 i) / 2 & 7 does not depend on i
  const int lrow = tid >> 3;
  const int gpiece = (tid & 7) ^ ((lrow >> 1) & 7);
  const uint16_t* asrc[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int r = m0 + lrow + 64 * i;
    asrc[i] = x + size_t(r < T ? r : T - 1) * H + gpiece * 8;
  }
  const uint16_t* bsrc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int n = n0 + lrow + 64 * i;
    bsrc[i] = gate_w + size_t(n < E ? n : E - 1) * H + gpiece * 8;
  }
  auto issue = [&](int ks) {
    const int kcol = (ks0 + ks) * GBK;
    const int st = ks % NS;
#pragma unroll
    for (int i = 0; i < NA; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(asrc[i] + kcol),
                                       (lptr_t)(As + st * BM * 8 + (i * 8 + wave) * 64), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(bsrc[i] + kcol),
                                       (lptr_t)(Bs + st * GBN * 8 + (i * 8 + wave) * 64), 16, 0, 0);
  };

  f32x16 acc[NT];
  double dsum[NT][16];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[j][i] = 0.f; dsum[j][i] = 0.0; }
  float xsq[NA], wsq[2] = {0.f, 0.f};
#pragma unroll
  for (int i = 0; i < NA; ++i) xsq[i] = 0.f;

#pragma unroll
  for (int d = 0; d < NS - 1; ++d)
    if (d < ksteps) issue(d);
  for (int ks = 0; ks < ksteps; ++ks) {
    // step ks must have landed; the NS-2 younger steps may stay in flight
    if (ks + NS - 2 < ksteps) wait_vmcnt<NLOAD * (NS - 2)>(); else wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // every wavefront is done with step ks-1: refill its stage
    if (ks + NS - 1 < ksteps) issue(ks + NS - 1);
    const uint4* const Ast = As + (ks % NS) * BM * 8;
    const uint4* const Bst = Bs + (ks % NS) * GBN * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int piece = kk * 2 + (lane >> 5);
      const uint4 av = Ast[swz(wm * 32 + (lane & 31), piece)];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const uint4 bv = Bst[swz((wn * NT + j) * 32 + (lane & 31), piece)];
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                         __builtin_bit_cast(bf16x8, bv), acc[j], 0, 0, 0);
      }
    }
    if (blockIdx.y == 0) {                        // squared row norms from this thread's own pieces
#pragma unroll
      for (int i = 0; i < NA; ++i) xsq[i] = piece_sumsq(Ast[tid + 512 * i], xsq[i]);
    }
    if (blockIdx.x == 0) {                        // the first token tile also sums the gate rows' squares
#pragma unroll
      for (int i = 0; i < 2; ++i) wsq[i] = piece_sumsq(Bst[tid + 512 * i], wsq[i]);
    }
    if ((ks + 1) % CHAIN_STEPS == 0 || ks + 1 == ksteps) {
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dsum[j][i] += (double)acc[j][i]; acc[j][i] = 0.f; }
    }
  }

  // D layout of the 32x32 MFMA: lane l, register i -> row (i/4)*8 + (l/32)*4 + i%4, col l%32
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int col = n0 + (wn * NT + j) * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      if (row < T && col < E) logits[size_t(row) * E + col] = (float)dsum[j][i];
    }
  }
  if (blockIdx.y == 0) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      float s = xsq[i];
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      const int r = m0 + lrow + 64 * i;
      if ((tid & 7) == 0 && r < T) xnorm2[r] = s * 1.001f;
    }
  }
  if (blockIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float s = wsq[i];
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      const int n = n0 + lrow + 64 * i;
      if ((tid & 7) == 0 && n < E) wnorm2[n] = s * 1.001f;
    }
  }
}

template <int BM, int NS, int CHAIN_STEPS>
__global__ __launch_bounds__(512) void gate_dma_kernel(const uint16_t* __restrict__ x,
                                                       const uint16_t* __restrict__ gate_w, int T,
                                                       int H, int E, float* __restrict__ logits,
                                                       float* __restrict__ xnorm2,
                                                       float* __restrict__ wnorm2,
                                                       int32_t* __restrict__ counters) {
  extern __shared__ uint4 gate_smem[];
  // The ring is handed on as a generic pointer: with the LDS array named in the
  // loop the compiler puts a vmcnt(0) in front of every LDS read that follows a
  // DMA in program order, which would drain the ring; the waits and the barrier
  // in the body order the DMA writes and the reads explicitly.
  gate_dma_body<BM, NS, CHAIN_STEPS>(x, gate_w, T, H, E, logits, xnorm2, wnorm2, counters, gate_smem);
}

// ----------------------------------------------------------- stage 2: select
struct SelCfg {
  int E, k, score_fn, renormalize, G, Kg, gn;
  float scale;
  float chain_err;   // 2n * 2^-24 of the gate accumulation (0 when logits are given)
  int have_norms;
  int nsplit;        // K splits of the gate GEMM: logits and row norms are sums of this many slabs
  int wsplit;        // slabs of the gate rows' sums of squares (stride E)
  int T;             // tokens: slab strides are T*E (logits) and T (row norms)
};

// Norm of token t's row from the per-split sums of squares.
__device__ __forceinline__ float token_norm(const SelCfg& c, const float* __restrict__ xnorm2, int t) {
  if (!c.have_norms) return 0.f;
  float s = xnorm2[t];
  for (int i = 1; i < c.nsplit; ++i) s += xnorm2[t + size_t(i) * c.T];
  return sqrtf(s);
}

// Norm of gate row e from the per-split sums of squares.
__device__ __forceinline__ float gate_norm(const SelCfg& c, const float* __restrict__ wnorm2, int e) {
  float s = wnorm2[e];
  for (int i = 1; i < c.wsplit; ++i) s += wnorm2[e + i * c.E];
  return sqrtf(s);
}

// Fast key of one expert from its stage-1 logit z (the slabs already added up):
// key, the bound eps on |key - exact key|, and the value sc the weight is made of.
// wn = norm of the gate row (unused without norms).
__device__ __forceinline__ void fast_key_one(const SelCfg& c, float z, float xn, float wn,
                                             const float* __restrict__ logit_bias,
                                             const float* __restrict__ select_bias, int e,
                                             float& key, float& eps, float& sc) {
  float ez = 0.f;
  if (c.have_norms) ez = c.chain_err * xn * wn * 1.001f + 2.f * kUlp * fabsf(z);
  if (logit_bias) {
    z += logit_bias[e];
    ez += kUlp * fabsf(z);
  }
  if (c.score_fn == MOE_SCORE_SOFTMAX) {
    key = z; eps = ez; sc = z;
  } else {
    const float s = 1.0f / (1.0f + expf(-z));
    const float sb = select_bias ? select_bias[e] : 0.f;
    key = s + sb;
    sc = s;
    // |sigmoid(z+d)-sigmoid(z)| <= s(1-s)|d| + d^2/16 ; fp32 evaluation of
    // the sigmoid and of the bias add is good to a few ulp of 1+|sb|
    eps = ez * (s * (1.f - s) + ez + 16.f * kUlp) + 16.f * kUlp * (1.f + fabsf(sb));
  }
}

// Per-lane view of one token's experts: expert e = slot*64 + lane.
template <typename FT, int EPL>
struct Keys {
  FT key[EPL];   // selection key
  FT eps[EPL];   // bound on |key - exact key|
  FT sc[EPL];    // value the weight is made of: logit (softmax) or sigmoid score
};

template <typename FT>
struct Groups {
  uint64_t kept;    // bit g: group g survives the group limit
  bool certain;     // the cut between kept and dropped groups holds for any keys within eps
  uint32_t need;    // bit per slot: the expert may be one of its group's group_score_n largest
  uint64_t open;    // bit g: whether group g is kept depends on exact scores
};

template <typename FT>
struct Picks {
  int id;        // lane j < k: j-th pick
  FT sc;         // its logit / score
  FT low;        // smallest lower bound of a picked key
  bool certain;  // every comparison held with the error intervals apart
};

// Fast keys of token t from the stage-1 logits.
template <int EPL>
__device__ __forceinline__ void fast_keys(const SelCfg& c, const float* __restrict__ logits_row,
                                          const float* __restrict__ logit_bias,
                                          const float* __restrict__ select_bias, float xn,
                                          const float* __restrict__ wnorm2, int lane,
                                          Keys<float, EPL>& K) {
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = i * 64 + lane;
    float key = -INFINITY, eps = 0.f, sc = 0.f;
    if (e < c.E) {
      float z = logits_row[e];
      for (int sp = 1; sp < c.nsplit; ++sp) z += logits_row[e + size_t(sp) * c.T * c.E];
      const float wn = c.have_norms ? gate_norm(c, wnorm2, e) : 0.f;
      fast_key_one(c, z, xn, wn, logit_bias, select_bias, e, key, eps, sc);
    }
    K.key[i] = key; K.eps[i] = eps; K.sc[i] = sc;
  }
}

// Group limit: keep the Kg groups with the largest sum of their gn largest
// keys; ties go to the lowest group.  Lane g ends up holding group g's score.
template <typename FT, int EPL>
__device__ __forceinline__ void group_stage(const SelCfg& c, const Keys<FT, EPL>& K, int lane,
                                            Groups<FT>& Gp) {
  const int gs = c.E / c.G;
  FT gsum = 0, gerr = 0;          // lane g: score of group g and the bound on its error
  uint32_t need = 0;
  if (64 % gs == 0 && c.gn <= 2 && c.E % 64 == 0) {
    // groups are aligned runs of gs lanes inside a slot: butterfly (max1, max2,
    // max eps, min lower bound of the two largest) over each run, all groups at once
    const int per_slot = 64 / gs;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if (i * 64 >= c.E) break;
      FT m1 = K.key[i], m2 = -INFINITY, me = K.eps[i];
      FT l1 = K.key[i] - K.eps[i], l2 = -INFINITY;      // two largest lower bounds
#define STEP_(S)                                                                   \
  if ((1 << S) < gs) {                                                             \
    const FT o1 = lane_xchg<S>(m1), o2 = lane_xchg<S>(m2), oe = lane_xchg<S>(me);  \
    const FT p1 = lane_xchg<S>(l1), p2 = lane_xchg<S>(l2);                         \
    const FT lo = m1 < o1 ? m1 : o1, hi2 = m2 > o2 ? m2 : o2;                      \
    m1 = m1 > o1 ? m1 : o1;                                                        \
    m2 = lo > hi2 ? lo : hi2;                                                      \
    me = me > oe ? me : oe;                                                        \
    const FT ql = l1 < p1 ? l1 : p1, qh = l2 > p2 ? l2 : p2;                       \
    l1 = l1 > p1 ? l1 : p1;                                                        \
    l2 = ql > qh ? ql : qh;                                                        \
  }
      MOE_ALL_STEPS(STEP_)
#undef STEP_
      const FT sum = c.gn == 2 ? m1 + m2 : m1;
      const FT nth_low = c.gn == 2 ? l2 : l1;            // <= the gn-th largest exact key
      if (K.key[i] + K.eps[i] >= nth_low) need |= 1u << i;
      // lane g fetches its group's values from the first lane of the run
      const int g0 = i * per_slot;
      const int src = (lane >= g0 && lane < g0 + per_slot) ? (lane - g0) * gs : 0;
      const FT s_ = __shfl(sum, src), e_ = __shfl(me, src);
      if (lane >= g0 && lane < g0 + per_slot) { gsum = s_; gerr = e_ * (FT)c.gn; }
    }
  } else {
    for (int g = 0; g < c.G; ++g) {
      uint32_t taken = 0;
      FT sum = 0, me = 0, nth_low = INFINITY;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        const int e = i * 64 + lane;
        if (e < c.E && e / gs == g) me = K.eps[i] > me ? K.eps[i] : me;
      }
      me = wave_max(me);
      for (int r = 0; r < c.gn; ++r) {
        FT v = 0; int idx = INT_MAX;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const int e = i * 64 + lane;
          if (e < c.E && e / gs == g && !(taken >> i & 1) && (idx == INT_MAX || K.key[i] > v)) {
            v = K.key[i]; idx = e;
          }
        }
        wave_argmax(v, idx);
        sum += v;
        nth_low = v - me;       // keys come in descending order; me bounds every eps
        if ((idx & 63) == lane) taken |= 1u << (idx >> 6);
      }
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        const int e = i * 64 + lane;
        if (e < c.E && e / gs == g && K.key[i] + K.eps[i] >= nth_low) need |= 1u << i;
      }
      if (lane == g) { gsum = sum; gerr = me * (FT)c.gn; }
    }
  }
  uint64_t kept = 0;
  FT low = INFINITY;
  for (int r = 0; r < c.Kg; ++r) {
    FT v = gsum; int idx = (lane < c.G && !(kept >> lane & 1)) ? lane : INT_MAX;
    wave_argmax(v, idx);
    kept |= uint64_t(1) << idx;
    const FT lo = read_lane(gsum - gerr, idx & 63);
    low = lo < low ? lo : low;
  }
  FT hi = (lane < c.G && !(kept >> lane & 1)) ? gsum + gerr : -INFINITY;
  hi = wave_max(hi);
  Gp.kept = kept;
  Gp.certain = (c.Kg >= c.G) || (low > hi);
  Gp.need = need;
  // A kept group whose lower bound clears every dropped group's upper bound stays
  // kept whatever the exact keys are (only kept groups can outrank it), and a
  // dropped group whose upper bound is below every kept group's lower bound stays
  // dropped; the cut is open only among the others.
  bool open = false;
  if (lane < c.G) open = (kept >> lane & 1) ? !(gsum - gerr > hi) : !(gsum + gerr < low);
  Gp.open = __ballot(open);
}

// Eligibility bits per slot: valid expert whose group is kept.
template <int EPL>
__device__ __forceinline__ uint32_t eligible_mask(const SelCfg& c, uint64_t kept, int lane) {
  uint32_t elig = 0;
  const int gs = c.E / c.G;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = i * 64 + lane;
    if (e < c.E && (c.G <= 1 || (kept >> (e / gs) & 1))) elig |= 1u << i;
  }
  return elig;
}

// Top-k among the eligible experts, k successive arg-max reductions; ties go to
// the lowest expert index.
template <typename FT, int EPL>
__device__ __forceinline__ void topk_stage(const SelCfg& c, const Keys<FT, EPL>& K, uint32_t elig,
                                           int lane, Picks<FT>& P) {
  uint32_t taken = 0;
  FT prev_lo = INFINITY, low = INFINITY;
  P.id = -1; P.sc = 0; P.certain = true;
  for (int j = 0; j < c.k; ++j) {
    FT v = 0; int idx = INT_MAX;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if ((elig >> i & 1) && !(taken >> i & 1) && (idx == INT_MAX || K.key[i] > v)) {
        v = K.key[i]; idx = i * 64 + lane;
      }
    }
    wave_argmax(v, idx);
    const int owner = idx & 63, slot = idx >> 6;
    FT oe = 0, os = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (i == slot) { oe = K.eps[i]; os = K.sc[i]; }
    oe = read_lane(oe, owner);
    os = read_lane(os, owner);
    if (lane == owner) taken |= 1u << slot;
    if (lane == j) { P.id = idx; P.sc = os; }
    if (!(prev_lo > v + oe) && j > 0) P.certain = false;
    prev_lo = v - oe;
    low = prev_lo < low ? prev_lo : low;
  }
  FT hi = -INFINITY;
  bool any = false;
#pragma unroll
  for (int i = 0; i < EPL; ++i)
    if ((elig >> i & 1) && !(taken >> i & 1)) {
      const FT h = K.key[i] + K.eps[i];
      hi = (!any || h > hi) ? h : hi;
      any = true;
    }
  const bool some = __ballot(any) != 0;
  hi = wave_max(any ? hi : (FT)-INFINITY);
  if (some && !(prev_lo > hi)) P.certain = false;
  P.low = low;
}

// Weights of the picked experts; lane j < k returns w[t,j].
template <typename FT, int EPL>
__device__ __forceinline__ FT pick_weight(const SelCfg& c, const Keys<FT, EPL>& K,
                                          const Picks<FT>& P, int lane) {
  const bool mine = lane < c.k;
  FT num, den;
  if (c.score_fn == MOE_SCORE_SOFTMAX) {
    if (c.renormalize) {
      const FT m = wave_max(mine ? P.sc : (FT)-INFINITY);
      num = mine ? (FT)exp((FT)(P.sc - m)) : (FT)0;
      den = wave_sum(num);
    } else {
      FT m = -INFINITY;
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if (i * 64 + lane < c.E) m = K.sc[i] > m ? K.sc[i] : m;
      m = wave_max(m);
      FT s = 0;
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if (i * 64 + lane < c.E) s += (FT)exp((FT)(K.sc[i] - m));
      den = wave_sum(s);
      num = mine ? (FT)exp((FT)(P.sc - m)) : (FT)0;
    }
  } else {
    num = mine ? P.sc : (FT)0;
    den = c.renormalize ? wave_sum(num) : (FT)1;
  }
  return num / den * (FT)c.scale;
}

template <int EPL>
__global__ __launch_bounds__(256) void route_select_kernel(
    SelCfg c, int T, const float* __restrict__ logits, const float* __restrict__ logit_bias,
    const float* __restrict__ select_bias, const float* __restrict__ xnorm2,
    const float* __restrict__ wnorm2, int32_t* __restrict__ ids, float* __restrict__ w,
    int32_t* __restrict__ counters, int32_t* __restrict__ recheck,
    float* __restrict__ recheck_low) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  Keys<float, EPL> K;
  const float xn = token_norm(c, xnorm2, t);
  fast_keys<EPL>(c, logits + size_t(t) * c.E, logit_bias, select_bias, xn, wnorm2, lane, K);
  Groups<float> Gp;
  Gp.kept = 0; Gp.certain = true; Gp.need = 0; Gp.open = 0;
  if (c.G > 1) group_stage<float, EPL>(c, K, lane, Gp);
  Picks<float> P;
  topk_stage<float, EPL>(c, K, eligible_mask<EPL>(c, Gp.kept, lane), lane, P);
  if (P.certain && Gp.certain) {
    const float wt = pick_weight<float, EPL>(c, K, P, lane);
    if (lane < c.k) {
      ids[size_t(t) * c.k + lane] = P.id;
      w[size_t(t) * c.k + lane] = wt;
    }
  } else if (lane == 0) {
    // order of the list is irrelevant: every listed token is re-scored on its own
    const int slot = atomicAdd(&counters[0], 1);
    recheck[slot] = t;
    // with the groups settled, the re-scoring starts from the picks found here
    recheck_low[slot] = Gp.certain ? P.low : __builtin_nanf("");
  }
}

// --------------------------------------------------------- stage 3: re-score
// One wavefront per listed token (four independent tokens per workgroup, no
// workgroup barrier).  Phase 1 (only when the group cut is in doubt): the
// experts that may be among their group's largest get exact keys and the groups
// are chosen in fp64.  Phase 2: with the groups fixed, the experts whose key
// interval reaches the picks get exact keys and the top-k is taken in fp64.
// Experts outside those sets keep their fast keys: by construction they cannot
// change either decision.  A wavefront's candidate list and exact logits live
// in its own slice of LDS; LDS operations of one wavefront execute in order.
// COOP (short lists: few tokens in the batch): one token per workgroup.  The four
// wavefronts run the same selection steps on the same data (so their control
// flow is identical and the barriers below are reached by all of them) and share
// out each exact dot product, a quarter of the token row each: the chain of
// dependent load rounds, which is all this kernel's time, is four times shorter.
template <int EPL, bool BF16, bool COOP>
__global__ __launch_bounds__(256, 2) void route_recheck_kernel(
    SelCfg c, int H, const void* __restrict__ x, const void* __restrict__ gate_w,
    const float* __restrict__ logits_in, const float* __restrict__ logits,
    const float* __restrict__ logit_bias, const float* __restrict__ select_bias,
    const float* __restrict__ xnorm2, const float* __restrict__ wnorm2, int32_t* __restrict__ ids,
    float* __restrict__ w, const int32_t* __restrict__ counters,
    const int32_t* __restrict__ recheck, const float* __restrict__ recheck_low) {
  __shared__ int xlist_all[4][EPL * 64];
  __shared__ double zx_all[4][EPL * 64];
  __shared__ float2 rint_all[4][EPL * 64];     // key intervals of the listed experts
  __shared__ double part_all[COOP ? 4 : 1][4]; // COOP: partial dot products of the wavefronts (up to 4 experts)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int* const xlist = xlist_all[wave];
  double* const zx = zx_all[wave];
  float2* const rint = rint_all[wave];
  const int n_list = counters[0];
  const size_t eb = BF16 ? 2 : 4;

  // exact logits of the experts in xlist[0..n) -> zx[e].  The wavefront walks the
  // token row once per batch of CB experts, lane-strided 16-byte pieces, four
  // pieces per lane and expert in flight; the lane sums are combined by a fixed
  // butterfly.
  // CB experts per walk over the token row.  6 and 8 measured slower (register
  // pressure); a second instance of this code with CB = 2 for the usual short list
  // (two picks whose order is in doubt) made the kernel slower as a whole
  // (re-score 46 -> 64 us on the 256-expert gate at 16384 tokens).
  constexpr int CB = 4;
  auto exact_logits = [&](int t, int n) {
    if (logits_in) {
      for (int q = lane; q < n; q += 64) {
        const int e = xlist[q];
        double z = (double)logits_in[size_t(t) * c.E + e];
        if (logit_bias) z += (double)logit_bias[e];
        zx[e] = z;
      }
      return;
    }
    const char* xrow = static_cast<const char*>(x) + size_t(t) * H * eb;
    const int n16 = int(H * eb / 16);
    for (int q0 = 0; q0 < n; q0 += CB) {
      double acc[CB];
      const char* wrow[CB];
      int ex[CB];
#pragma unroll
      for (int i = 0; i < CB; ++i) {
        acc[i] = 0.0;
        ex[i] = xlist[q0 + i < n ? q0 + i : n - 1];
        wrow[i] = static_cast<const char*>(gate_w) + size_t(ex[i]) * H * eb;
      }
      // U pieces per lane and expert in flight (the tail pieces are clamped to the
      // last one and masked out of the sum)
      constexpr int U = 4;
      // COOP: wavefront w walks the pieces w*64*U .. of every run of 4*64*U
      for (int p0 = COOP ? wave * 64 * U : 0; p0 < n16; p0 += (COOP ? 4 : 1) * 64 * U) {
        uint4 a[U], b[CB][U];
        bool in[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          int p = p0 + u * 64 + lane;
          in[u] = p < n16;
          p = in[u] ? p : n16 - 1;
          a[u] = *reinterpret_cast<const uint4*>(xrow + size_t(p) * 16);
#pragma unroll
          for (int i = 0; i < CB; ++i) b[i][u] = *reinterpret_cast<const uint4*>(wrow[i] + size_t(p) * 16);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int i = 0; i < CB; ++i) {
            const double d = piece_dot64<BF16>(a[u], b[i][u], 0.0);
            acc[i] += in[u] ? d : 0.0;
          }
      }
      if constexpr (COOP) {
        // the four partial sums of each expert, added in wavefront order by everyone
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          const double zp = wave_sum(acc[i]);
          if (lane == 0) part_all[wave][i] = zp;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          double z = ((part_all[0][i] + part_all[1][i]) + part_all[2][i]) + part_all[3][i];
          if (q0 + i < n && lane == 0) {
            if (logit_bias) z += (double)logit_bias[ex[i]];
            zx[ex[i]] = z;
          }
        }
        __syncthreads();                    // before the next batch overwrites the partial sums
      } else {
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          double z = wave_sum(acc[i]);
          if (q0 + i < n && lane == 0) {
            if (logit_bias) z += (double)logit_bias[ex[i]];
            zx[ex[i]] = z;
          }
        }
      }
    }
  };
  // list the experts flagged in `want`; returns how many
  auto make_list = [&](uint32_t want) {
    int n = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const bool in = want >> i & 1;
      const uint64_t m = __ballot(in);
      if (in) xlist[n + __popcll(m & ((uint64_t(1) << lane) - 1))] = i * 64 + lane;
      n += __popcll(m);
    }
    return n;
  };

  for (int li = COOP ? int(blockIdx.x) : int(blockIdx.x) * 4 + wave; li < n_list;
       li += COOP ? int(gridDim.x) : int(gridDim.x) * 4) {
    const int t = recheck[li];
    Keys<float, EPL> K;
    Keys<double, EPL> D;
    Groups<float> Gf;
    Gf.kept = 0; Gf.certain = true; Gf.need = 0; Gf.open = 0;
    uint32_t exact = 0;          // slots of this lane that hold exact keys
    auto adopt = [&](uint32_t want) {   // pull exact logits into D
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        if (!(want >> i & 1)) continue;
        const int e = i * 64 + lane;
        const double z = zx[e];
        if (c.score_fn == MOE_SCORE_SOFTMAX) {
          D.key[i] = z; D.sc[i] = z;
        } else {
          const double sg = 1.0 / (1.0 + exp(-z));
          D.sc[i] = sg;
          D.key[i] = sg + (select_bias ? (double)select_bias[e] : 0.0);
        }
      }
      exact |= want;
    };
    const float xn = token_norm(c, xnorm2, t);
    fast_keys<EPL>(c, logits + size_t(t) * c.E, logit_bias, select_bias, xn, wnorm2, lane, K);
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      D.key[i] = (double)K.key[i]; D.sc[i] = (double)K.sc[i]; D.eps[i] = 0.0;
    }
    if (c.G > 1) group_stage<float, EPL>(c, K, lane, Gf);
    uint64_t kept = Gf.kept;
    if (c.G > 1 && !Gf.certain) {       // phase 1: settle the groups in fp64
      // exact keys only where they can matter: the possible largest members of the
      // groups on whose scores the cut still depends.  The other groups keep their
      // fast scores, which the intervals already order against every open group.
      uint32_t want1 = 0;
      const int gs = c.E / c.G;
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if ((Gf.need >> i & 1) && (Gf.open >> ((i * 64 + lane) / gs) & 1)) want1 |= 1u << i;
      const int n = make_list(want1);
      exact_logits(t, n);
      adopt(want1);
      Groups<double> Gd;
      group_stage<double, EPL>(c, D, lane, Gd);
      kept = Gd.kept;
    }
    // phase 2: candidates of the top-k.  The smallest lower bound of the fast picks
    // comes from the selection pass unless the groups had to be settled here.
    const uint32_t elig = eligible_mask<EPL>(c, kept, lane);
    Picks<float> P;
    P.low = recheck_low[li];
    if (!(P.low == P.low)) topk_stage<float, EPL>(c, K, elig, lane, P);
    // Only experts whose upper bound reaches the smallest lower bound of a pick can
    // be among the picks.  Of those, an expert whose interval is apart from every
    // other's is ordered against all of them by its fast key already; the ones whose
    // intervals meet another's get exact keys.
    uint32_t region = 0;
    float lo[EPL], hi[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      lo[i] = K.key[i] - K.eps[i];
      hi[i] = K.key[i] + K.eps[i];
      if ((elig >> i & 1) && hi[i] >= P.low) region |= 1u << i;
    }
    int nr = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const bool in = region >> i & 1;
      const uint64_t m = __ballot(in);
      if (in) {
        const int pos = nr + __popcll(m & ((uint64_t(1) << lane) - 1));
        xlist[pos] = i * 64 + lane;
        rint[pos] = make_float2(lo[i], hi[i]);
      }
      nr += __popcll(m);
    }
    uint32_t want = 0;
    for (int q = 0; q < nr; ++q) {
      const int m = xlist[q];
      const float2 iv = rint[q];
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if ((region >> i & 1) && i * 64 + lane != m && lo[i] <= iv.y && iv.x <= hi[i]) want |= 1u << i;
    }
    want &= ~exact;
    const int n = make_list(want);
    exact_logits(t, n);
    adopt(want);
    Picks<double> Q;
    topk_stage<double, EPL>(c, D, elig, lane, Q);
    const double wt = pick_weight<double, EPL>(c, D, Q, lane);
    if (lane < c.k && (!COOP || wave == 0)) {
      ids[size_t(t) * c.k + lane] = Q.id;
      w[size_t(t) * c.k + lane] = (float)wt;
    }
  }
}

// -------------------- few tokens: gate, scores and top-k of a token in one pass
// One workgroup of sixteen wavefronts per token.  The wavefronts share out the experts and
// compute every logit exactly (fp64 sums of exact products, CB experts per walk
// over the token row); the first wavefront then builds fp64 keys for all experts
// and takes the group limit, the top-k and the weights in fp64.  No fast pass,
// no error intervals and nothing to re-score: at decode sizes the T*E*H fused
// multiply-adds cost less than the launches they replace.
template <int EPL, bool BF16>
__global__ __launch_bounds__(1024) void route_exact_kernel(
    SelCfg c, int H, const void* __restrict__ x, const void* __restrict__ gate_w,
    const float* __restrict__ logit_bias, const float* __restrict__ select_bias,
    int32_t* __restrict__ ids, float* __restrict__ w, int32_t* __restrict__ counters) {
  __shared__ double zx[EPL * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x;
  if (t == 0 && threadIdx.x < 64) counters[threadIdx.x] = 0;   // nothing is re-scored
  const size_t eb = BF16 ? 2 : 4;
  const char* xrow = static_cast<const char*>(x) + size_t(t) * H * eb;
  const int n16 = int(H * eb / 16);
  const int per = (c.E + 15) / 16;
  const int e_begin = min(c.E, wave * per), e_end = min(c.E, e_begin + per);
  constexpr int CB = 4, U = 4;   // experts per walk, pieces per lane and row in flight (8: spills)
  for (int e0 = e_begin; e0 < e_end; e0 += CB) {
    double acc[CB];
    const char* wrow[CB];
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      acc[i] = 0.0;
      wrow[i] = static_cast<const char*>(gate_w) + size_t(min(e0 + i, e_end - 1)) * H * eb;
    }
    for (int p0 = 0; p0 < n16; p0 += 64 * U) {
      uint4 a[U], b[CB][U];
      bool in[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int p = p0 + u * 64 + lane;
        in[u] = p < n16;
        p = in[u] ? p : n16 - 1;
        a[u] = *reinterpret_cast<const uint4*>(xrow + size_t(p) * 16);
#pragma unroll
        for (int i = 0; i < CB; ++i) b[i][u] = *reinterpret_cast<const uint4*>(wrow[i] + size_t(p) * 16);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          const double d = piece_dot64<BF16>(a[u], b[i][u], 0.0);
          acc[i] += in[u] ? d : 0.0;
        }
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      double z = wave_sum(acc[i]);
      if (e0 + i < e_end && lane == 0) {
        if (logit_bias) z += (double)logit_bias[e0 + i];
        zx[e0 + i] = z;
      }
    }
  }
  __syncthreads();
  if (wave != 0) return;
  Keys<double, EPL> D;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = i * 64 + lane;
    D.key[i] = -INFINITY; D.sc[i] = 0.0; D.eps[i] = 0.0;
    if (e < c.E) {
      const double z = zx[e];
      if (c.score_fn == MOE_SCORE_SOFTMAX) {
        D.key[i] = z; D.sc[i] = z;
      } else {
        const double sg = 1.0 / (1.0 + exp(-z));
        D.sc[i] = sg;
        D.key[i] = sg + (select_bias ? (double)select_bias[e] : 0.0);
      }
    }
  }
  uint64_t kept = 0;
  if (c.G > 1) {
    Groups<double> Gd;
    group_stage<double, EPL>(c, D, lane, Gd);
    kept = Gd.kept;
  }
  const uint32_t elig = eligible_mask<EPL>(c, kept, lane);
  Picks<double> Q;
  topk_stage<double, EPL>(c, D, elig, lane, Q);
  const double wt = pick_weight<double, EPL>(c, D, Q, lane);
  if (lane < c.k) {
    ids[size_t(t) * c.k + lane] = Q.id;
    w[size_t(t) * c.k + lane] = (float)wt;
  }
}

// ---------- few tokens, long gate rows: exact logits and selection as two kernels
// When a token's E*H multiply-adds are many (256 experts x hidden 7168), one
// workgroup per token is a chain of sixteen dependent load rounds per wavefront.
// Here a workgroup of four wavefronts takes sixteen experts of one token (a
// wavefront: four gate rows, eight 16-byte pieces per lane and row in flight), so
// a token is shared out over E/16 workgroups and the fp64 logits go to the
// workspace; a second kernel, one wavefront per token, selects on the fp64 keys.
template <bool BF16>
__global__ __launch_bounds__(256) void gate_exact_kernel(
    int H, int E, const void* __restrict__ x, const void* __restrict__ gate_w,
    const float* __restrict__ logit_bias, double* __restrict__ zx, int32_t* __restrict__ counters) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.y;
  if (blockIdx.x == 0 && t == 0 && threadIdx.x < 64) counters[threadIdx.x] = 0;   // nothing is re-scored
  constexpr int CB = 4, U = 8;
  const int e0 = (blockIdx.x * 4 + wave) * CB;
  if (e0 >= E) return;
  const size_t eb = BF16 ? 2 : 4;
  const char* xrow = static_cast<const char*>(x) + size_t(t) * H * eb;
  const int n16 = int(H * eb / 16);
  double acc[CB];
  const char* wrow[CB];
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    acc[i] = 0.0;
    wrow[i] = static_cast<const char*>(gate_w) + size_t(min(e0 + i, E - 1)) * H * eb;
  }
  for (int p0 = 0; p0 < n16; p0 += 64 * U) {
    uint4 a[U], b[CB][U];
    bool in[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int p = p0 + u * 64 + lane;
      in[u] = p < n16;
      p = in[u] ? p : n16 - 1;
      a[u] = *reinterpret_cast<const uint4*>(xrow + size_t(p) * 16);
#pragma unroll
      for (int i = 0; i < CB; ++i) b[i][u] = *reinterpret_cast<const uint4*>(wrow[i] + size_t(p) * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < CB; ++i) {
        const double d = piece_dot64<BF16>(a[u], b[i][u], 0.0);
        acc[i] += in[u] ? d : 0.0;
      }
  }
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    double z = wave_sum(acc[i]);
    if (e0 + i < E && lane == 0) {
      if (logit_bias) z += (double)logit_bias[e0 + i];
      zx[size_t(t) * E + e0 + i] = z;
    }
  }
}

template <int EPL>
__global__ __launch_bounds__(256) void select_exact_kernel(
    SelCfg c, int T, const double* __restrict__ zx, const float* __restrict__ select_bias,
    int32_t* __restrict__ ids, float* __restrict__ w) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  Keys<double, EPL> D;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = i * 64 + lane;
    D.key[i] = -INFINITY; D.sc[i] = 0.0; D.eps[i] = 0.0;
    if (e < c.E) {
      const double z = zx[size_t(t) * c.E + e];
      if (c.score_fn == MOE_SCORE_SOFTMAX) {
        D.key[i] = z; D.sc[i] = z;
      } else {
        const double sg = 1.0 / (1.0 + exp(-z));
        D.sc[i] = sg;
        D.key[i] = sg + (select_bias ? (double)select_bias[e] : 0.0);
      }
    }
  }
  uint64_t kept = 0;
  if (c.G > 1) {
    Groups<double> Gd;
    group_stage<double, EPL>(c, D, lane, Gd);
    kept = Gd.kept;
  }
  const uint32_t elig = eligible_mask<EPL>(c, kept, lane);
  Picks<double> Q;
  topk_stage<double, EPL>(c, D, elig, lane, Q);
  const double wt = pick_weight<double, EPL>(c, D, Q, lane);
  if (lane < c.k) {
    ids[size_t(t) * c.k + lane] = Q.id;
    w[size_t(t) * c.k + lane] = (float)wt;
  }
}

template <int EPL>
void launch_route_exact2(const SelCfg& sc, const moe_config& c, int T, const void* x,
                         const void* gate_w, const float* logit_bias, const float* select_bias,
                         int32_t* ids, float* w, const RouteWs& ws, hipStream_t s) {
  // the logits area holds at least two floats per (token, expert): room for one double
  double* zx = reinterpret_cast<double*>(ws.logits);
  const dim3 grid((c.n_experts + 15) / 16, T);
  if (c.act_dtype == MOE_BF16)
    MOE_LAUNCH(MOE_K_GATE_GEMM, gate_exact_kernel<true>, grid, dim3(256), 0, s, c.hidden, c.n_experts, x,
               gate_w, logit_bias, zx, ws.counters);
  else
    MOE_LAUNCH(MOE_K_GATE_GEMM, gate_exact_kernel<false>, grid, dim3(256), 0, s, c.hidden, c.n_experts, x,
               gate_w, logit_bias, zx, ws.counters);
  MOE_LAUNCH(MOE_K_SELECT, select_exact_kernel<EPL>, dim3((T + 3) / 4), dim3(256), 0, s, sc, T, zx,
             select_bias, ids, w);
}

template <int EPL>
void launch_route_exact(const SelCfg& sc, const moe_config& c, int T, const void* x,
                        const void* gate_w, const float* logit_bias, const float* select_bias,
                        int32_t* ids, float* w, const RouteWs& ws, hipStream_t s) {
  if (c.act_dtype == MOE_BF16)
    MOE_LAUNCH(MOE_K_GATE_GEMM, (route_exact_kernel<EPL, true>), dim3(T), dim3(1024), 0, s, sc,
               c.hidden, x, gate_w, logit_bias, select_bias, ids, w, ws.counters);
  else
    MOE_LAUNCH(MOE_K_GATE_GEMM, (route_exact_kernel<EPL, false>), dim3(T), dim3(1024), 0, s, sc,
               c.hidden, x, gate_w, logit_bias, select_bias, ids, w, ws.counters);
}

template <int EPL>
void launch_select_and_recheck(const SelCfg& sc, const moe_config& c, int T, const void* x,
                               const void* gate_w, const float* logit_bias,
                               const float* select_bias, const float* logits_in,
                               const float* logits, int32_t* ids, float* w, const RouteWs& ws,
                               hipStream_t s) {
  MOE_LAUNCH(MOE_K_SELECT, route_select_kernel<EPL>, dim3((T + 3) / 4), dim3(256), 0, s, sc, T, logits,
             logit_bias, select_bias, ws.xnorm2, ws.wnorm2, ids, w, ws.counters, ws.recheck,
             ws.recheck_low);
  // short batches have short lists: a workgroup per listed token, its wavefronts
  // sharing each dot product; otherwise four tokens per workgroup at a time
  const bool coop = T <= 1024 && !logits_in;
  const int grid = coop ? T : (T < 4096 ? (T + 3) / 4 : 1024);
#define MOE_RECHECK(BF, CO)                                                                       \
  MOE_LAUNCH(MOE_K_RESCORE, (route_recheck_kernel<EPL, BF, CO>), dim3(grid), dim3(256), 0, s, sc, \
             c.hidden, x, gate_w, logits_in, logits, logit_bias, select_bias, ws.xnorm2,          \
             ws.wnorm2, ids, w, ws.counters, ws.recheck, ws.recheck_low)
  if (c.act_dtype == MOE_BF16) {
    if (coop) MOE_RECHECK(true, true); else MOE_RECHECK(true, false);
  } else {
    if (coop) MOE_RECHECK(false, true); else MOE_RECHECK(false, false);
  }
#undef MOE_RECHECK
}

}  // namespace

hipError_t launch_route(const moe_config& c, int T, const void* x, const void* gate_w,
                        const float* logit_bias, const float* select_bias,
                        const float* logits_in, int32_t* ids, float* w, const RouteWs& ws,
                        hipStream_t s) {
  const int E = c.n_experts, H = c.hidden;
  const bool bf16 = c.act_dtype == MOE_BF16;
  const float* logits = logits_in;
  SelCfg sc;
  sc.E = E; sc.k = c.top_k; sc.score_fn = c.score_fn; sc.renormalize = c.renormalize;
  sc.G = c.n_groups; sc.Kg = c.topk_groups; sc.gn = c.group_score_n; sc.scale = c.routed_scale;
  sc.chain_err = 0.f; sc.have_norms = 0; sc.nsplit = 1; sc.wsplit = 1; sc.T = T;
  const int epl = (E + 63) / 64;
  // decode-sized batches: the exact gate costs T*E*H fp64 fused multiply-adds,
  // about 0.24 us per 2^20 of them, in one kernel for the whole stage (a workgroup
  // per token: not for long batches of tiny layers).  The bf16 pipeline of four
  // kernels takes 45-50 us at these sizes (measured on the 128-expert layer, hidden
  // 2048: 51 us exact against 46 us tiled at 768 tokens), which puts the crossover
  // near 5 * 2^25; the fp32 pipeline starts with an fp64 VALU gate of its own and is
  // never faster below 2^28.
  const size_t small_limit = bf16 ? size_t(5) << 25 : size_t(1) << 28;
  const bool small = size_t(T) * E * H <= small_limit && T <= 4096;
  // long gate rows and few tokens: the same arithmetic as two kernels.  Measured on
  // 256 experts x hidden 7168: 37 / 53 / 81 us at 16 / 64 / 128 tokens, where one
  // workgroup per token takes 84 us and the bf16 pipeline 92 us; the fp64 work grows
  // with the token count (135 us at 256), so the switch back sits at 2^28.
  const bool long_rows = size_t(E) * H > (size_t(1) << 19) && T <= 4096 &&
                         size_t(T) * E * H <= (size_t(1) << 28);
  if (!logits_in && long_rows) {
    if (epl <= 1) launch_route_exact2<1>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else if (epl <= 2) launch_route_exact2<2>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else if (epl <= 4) launch_route_exact2<4>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else launch_route_exact2<8>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    return hipGetLastError();
  }
  if (!logits_in && small) {
    if (epl <= 1) launch_route_exact<1>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else if (epl <= 2) launch_route_exact<2>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else if (epl <= 4) launch_route_exact<4>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    else launch_route_exact<8>(sc, c, T, x, gate_w, logit_bias, select_bias, ids, w, ws, s);
    return hipGetLastError();
  }
  // The bf16 gate GEMM sums the gate rows' squares and clears the counter itself
  // (its first token tile); the fp32 gate and the given-logits path use this kernel.
  if (logits_in || !bf16) {
    const void* gw_for_norm = logits_in ? nullptr : gate_w;
    if (bf16)
      MOE_LAUNCH(MOE_K_GATE_NORMS, gate_wnorm_kernel<true>, dim3((E + 3) / 4), dim3(256), 0, s, gw_for_norm,
                 E, H, ws.wnorm2, ws.counters);
    else
      MOE_LAUNCH(MOE_K_GATE_NORMS, gate_wnorm_kernel<false>, dim3((E + 3) / 4), dim3(256), 0, s, gw_for_norm,
                 E, H, ws.wnorm2, ws.counters);
  }
  if (!logits_in) {
    logits = ws.logits;
    sc.have_norms = 1;
    if (bf16) {
      // few tiles: split K so that about two workgroups per CU run (one workgroup is
      // one wavefront per SIMD, which hides no latency); each split keeps at least 8
      // K steps
      const int blocks = ((T + GBM - 1) / GBM) * ((E + GBN - 1) / GBN);
      const int ksteps = (H + GBK - 1) / GBK;
      int nsplit = 1;
      const int cap = gate_split_cap(T, E);
      while (nsplit < cap && blocks * nsplit * 2 <= kGateWgTarget && ksteps / (nsplit * 2) >= 8) nsplit *= 2;
      const dim3 grid((T + GBM - 1) / GBM, (E + GBN - 1) / GBN, nsplit);
      if (H % GBK == 0) {
        // two stages (48 KB): three workgroups share a CU, which measured faster than
        // deeper rings with fewer workgroups, and than 128-token tiles
        constexpr int NS = 2;
        constexpr int lds = NS * (GBM + GBN) * 8 * 16;
        MOE_LAUNCH(MOE_K_GATE_GEMM, (gate_dma_kernel<GBM, NS, kGateChainSteps>), grid, dim3(512), lds, s,
                   static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(gate_w), T, H, E,
                   ws.logits, ws.xnorm2, ws.wnorm2, ws.counters);
      } else {
        MOE_LAUNCH(MOE_K_GATE_GEMM, gate_mfma_kernel<kGateChainSteps>, grid, dim3(512), 0, s,
                   static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(gate_w), T, H, E,
                   ws.logits, ws.xnorm2, ws.wnorm2, ws.counters);
      }
      sc.nsplit = nsplit;
      sc.wsplit = nsplit;
      // chains of kGateChainSteps*64 products; +2 for the flush and the store.  The
      // partial dot products of the splits obey sum_s |x_s||w_s| <= |x||w|, so the
      // chain term is unchanged; summing the slabs in fp32 adds one ulp of that
      // product per addition and per slab store
      sc.chain_err = (2.f * kGateChainSteps * GBK + 2.f + 2.f * (nsplit - 1)) * kUlp;
    } else {
      MOE_LAUNCH(MOE_K_GATE_GEMM, gate_f64_kernel<false>, dim3(T), dim3(256), 0, s, x, gate_w, T,
                 H, E, ws.logits, ws.xnorm2);
      // fp64 sums: the only error is the fp32 store, covered by the 2 ulp term
      sc.chain_err = 1e-12f;
    }
  }
  if (epl <= 1)
    launch_select_and_recheck<1>(sc, c, T, x, gate_w, logit_bias, select_bias, logits_in, logits, ids, w, ws, s);
  else if (epl <= 2)
    launch_select_and_recheck<2>(sc, c, T, x, gate_w, logit_bias, select_bias, logits_in, logits, ids, w, ws, s);
  else if (epl <= 4)
    launch_select_and_recheck<4>(sc, c, T, x, gate_w, logit_bias, select_bias, logits_in, logits, ids, w, ws, s);
  else
    launch_select_and_recheck<8>(sc, c, T, x, gate_w, logit_bias, select_bias, logits_in, logits, ids, w, ws, s);
  return hipGetLastError();
}

}  // namespace moe
