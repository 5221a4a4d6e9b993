// Grouped expert MLP (Sec. II: every expert is an independent MLP; under TP
// its projections are sliced and the partial results summed afterwards).
//
//   GEMM-1  hmid[r,:] = silu(xs[r,:] Wgate_e^T) .* (xs[r,:] Wup_e^T)   r in expert e's rows
//   GEMM-2  ys[r,:]   = hmid[r,:] Wdown_e^T
//
// Both are "TN" GEMMs (activations [rows,K] and weights [N,K], K contiguous)
// over ragged row groups whose bounds live on the device.  A one-block
// prologue turns `offsets` into a table of M tiles (expert, first row, end
// row); the GEMM grid is sized for the worst case and workgroups past the
// table's length exit at once, so there is no host round trip.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation, K step 64.  GEMM-1
// loads a gate tile and the matching up tile so that one lane holds g and u of
// the same element and the SwiGLU is applied in registers.  Three kernels, by
// rows per expert: ffn_gemm8w_kernel (prefill: up to 256 rows x 256 weight rows
// per workgroup, operands global -> LDS directly, LDS rings; GEMM-2 of short groups
// of many experts: up to 128 rows x 512 weight rows), ffn_skinny_kernel
// (decode and fp8 weights: weight streaming, K split across wavefronts, no LDS
// staging) and the register-staged ffn_gemm_kernel for the shapes in between.
// fp8 weights: the weight-streaming kernel widens the e4m3 codes to bf16 in
// registers (exact) and multiplies the fp32 partial sum of each 128-deep K block
// by the 128x128 block scale; the tall-tile kernel keeps the codes in its LDS
// ring and rounds code * scale to bf16 on the way to the matrix unit.
#include <type_traits>

#include "moe_internal.h"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;

__device__ __forceinline__ int swz(int row, int piece) { return row * 8 + (piece ^ (row & 7)); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);   // round to nearest even
}

// silu(g) * u with the hardware exp2 and reciprocal (1 ulp each): the result is
// rounded to bf16 right after
__device__ __forceinline__ float silu_mul_fast(float g, float u) {
  const float t = __builtin_amdgcn_exp2f(g * -1.44269504088896341f);
  return g * u * __builtin_amdgcn_rcpf(1.0f + t);
}

__device__ __forceinline__ float silu_mul(float g, float u) {
  return g / (1.0f + __expf(-g)) * u;
}

// ------------------------------------------------------------- tile table
// tiles[0] = number of M tiles; then per tile a record (expert, first row, end
// row, index of the expert's first tile, number of tiles of the expert).
constexpr int kTileRec = 5;
// K-split of leftover tiles (see ffn_gemm8w_kernel): at most this many tiles are
// split, into at most kSplitMax parts of at least kSplitMinSteps K steps, and all
// parts together are at most one workgroup per CU.
constexpr int kCUs = 256;
constexpr int kSplitTickets = 256;
constexpr int kSplitMax = 4;
constexpr int kSplitMinSteps = 24;
constexpr int kPartFloats = 512 * 128;        // fp32 accumulators of one workgroup
static_assert(kSplitTickets == kFfnSplitSlots && kCUs <= kFfnSplitSlots, "workspace holds one slot per part");
static_assert(size_t(kPartFloats) * 4 == kFfnPartBytes, "partial-sum slot size");
#ifndef MOE_SPREAD_SLOTS
#define MOE_SPREAD_SLOTS 2
#endif
#ifndef MOE_RING_EXTRA_A
#define MOE_RING_EXTRA_A 2
#endif
// `balance`: an expert's rows are cut into ceil(M/bm) tiles of equal height
// (rounded up to 32 rows) instead of full tiles plus a short tail.
__global__ __launch_bounds__(256) void ffn_tiles_kernel(const int32_t* __restrict__ offsets,
                                                       int n_experts, int bm, int rows_capacity,
                                                       int32_t* __restrict__ tiles, int max_tiles,
                                                       int balance, int bm_second,
                                                       int32_t* __restrict__ tiles_second,
                                                       int32_t* __restrict__ tickets) {
  __shared__ int32_t start[513];
  __shared__ int32_t off[513];
  // arrival counters of the K-split tiles of the two GEMM launches that follow
  if (blockIdx.x == 0 && tickets)
    for (int i = threadIdx.x; i < 2 * kSplitTickets; i += blockDim.x) tickets[i] = 0;
  // a second workgroup, when launched, builds a second table with its own tile height
  if (blockIdx.x == 1) {
    bm = bm_second;
    tiles = tiles_second;
  }
  for (int e = threadIdx.x; e <= n_experts; e += blockDim.x) {
    int o = offsets[e];
    o = o < 0 ? 0 : o;
    off[e] = o > rows_capacity ? rows_capacity : o;
  }
  __syncthreads();
  if (threadIdx.x < 64) {                 // one wavefront scans the tile counts
    const int lane = threadIdx.x;
    const int per = (n_experts + 63) / 64;
    const int e0 = lane * per, e1 = (e0 + per < n_experts) ? e0 + per : n_experts;
    int sum = 0;
    for (int e = e0; e < e1; ++e) {
      const int m = off[e + 1] - off[e];
      sum += m > 0 ? (m + bm - 1) / bm : 0;
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    int run = incl - sum;
    for (int e = e0; e < e1; ++e) {
      const int m = off[e + 1] - off[e];
      start[e] = run;
      run += m > 0 ? (m + bm - 1) / bm : 0;
    }
    if (lane == 63) {
      start[n_experts] = incl;
      tiles[0] = incl < max_tiles ? incl : max_tiles;
    }
  }
  __syncthreads();
  // one thread per tile: its expert is the last one whose first tile is <= t
  const int n_tiles = start[n_experts] < max_tiles ? start[n_experts] : max_tiles;
  for (int t = threadIdx.x; t < n_tiles; t += blockDim.x) {
    int e = 0, e_hi = n_experts;
    while (e_hi - e > 1) {
      const int mid = (e + e_hi) >> 1;
      if (start[mid] <= t) e = mid; else e_hi = mid;
    }
    const int lo = off[e], hi = off[e + 1];
    int step = bm;
    if (balance) {
      const int nt = (hi - lo + bm - 1) / bm;
      step = (((hi - lo + nt - 1) / nt) + 31) / 32 * 32;
    }
    const int r = lo + (t - start[e]) * step;
    tiles[1 + kTileRec * t] = e;
    tiles[2 + kTileRec * t] = r;
    tiles[3 + kTileRec * t] = (r + step < hi) ? r + step : hi;
    tiles[4 + kTileRec * t] = start[e];
    tiles[5 + kTileRec * t] = (hi - lo + step - 1) / step;
  }
}

// ------------------------------------------------------------ MFMA GEMM
// C[rows, N] = A[rows, K] * B_e[N, K]^T over the M tiles of the table.
// DUAL: B0 = gate, B1 = up, C = silu(A B0^T) .* (A B1^T).
// Register-staged variant for bf16 shapes whose K is not a multiple of 64 (it
// zero-fills the K tail).
template <int BM, int BN, int WM, int WN, bool DUAL>
__global__ __launch_bounds__(256) void ffn_gemm_kernel(
    const uint16_t* __restrict__ A, const void* __restrict__ B0, const void* __restrict__ B1,
    uint16_t* __restrict__ C, int N, int K, const int32_t* __restrict__ tiles) {
  constexpr int BROWS = DUAL ? 2 * BN : BN;
  constexpr int WGN = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int NACC = DUAL ? 2 : 1;
  static_assert((BM / WM) * WGN == 4, "four wavefronts");
  constexpr int A_PER = BM * 8 / 256;
  constexpr int B_PER = BROWS * 8 / 256;

  // dynamic LDS: A double buffer, then B double buffer
  extern __shared__ uint4 smem[];
  uint4 (*As)[BM * 8] = reinterpret_cast<uint4 (*)[BM * 8]>(smem);
  uint4 (*Bs)[BROWS * 8] = reinterpret_cast<uint4 (*)[BROWS * 8]>(smem + 2 * BM * 8);

  const int n_ntiles = (N + BN - 1) / BN;
  const int mtile = blockIdx.x / n_ntiles, ntile = blockIdx.x % n_ntiles;
  if (mtile >= tiles[0]) return;
  const int e = tiles[1 + kTileRec * mtile], row0 = tiles[2 + kTileRec * mtile],
            row1 = tiles[3 + kTileRec * mtile];
  const int n0 = ntile * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int ksteps = (K + BK - 1) / BK;
  const size_t wbytes = 2;
  const char* Be0 = static_cast<const char*>(B0) + size_t(e) * N * K * wbytes;
  const char* Be1 = DUAL ? static_cast<const char*>(B1) + size_t(e) * N * K * wbytes : nullptr;

  uint4 ra[A_PER], rb[B_PER];
  auto gload = [&](int ks) {
    {
      const int lrow = tid >> 3, piece = tid & 7;
      const int kcol = ks * BK + piece * 8;
#pragma unroll
      for (int i = 0; i < A_PER; ++i) {
        int r = row0 + lrow + 32 * i;
        r = r < row1 ? r : row1 - 1;
        ra[i] = kcol < K ? *reinterpret_cast<const uint4*>(A + size_t(r) * K + kcol)
                         : make_uint4(0, 0, 0, 0);
      }
    }
    {
      const int lrow = tid >> 3, piece = tid & 7;
      const int kcol = ks * BK + piece * 8;
#pragma unroll
      for (int i = 0; i < B_PER; ++i) {
        const int lr = lrow + 32 * i;
        const char* base = (DUAL && lr >= BN) ? Be1 : Be0;
        int n = n0 + ((DUAL && lr >= BN) ? lr - BN : lr);
        n = n < N ? n : N - 1;
        rb[i] = kcol < K ? *reinterpret_cast<const uint4*>(base + (size_t(n) * K + kcol) * 2)
                         : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto lstore = [&](int buf) {
    {
      const int lrow = tid >> 3, piece = tid & 7;
#pragma unroll
      for (int i = 0; i < A_PER; ++i) As[buf][swz(lrow + 32 * i, piece)] = ra[i];
    }
    {
      const int lrow = tid >> 3, piece = tid & 7;
#pragma unroll
      for (int i = 0; i < B_PER; ++i) Bs[buf][swz(lrow + 32 * i, piece)] = rb[i];
    }
  };

  f32x16 acc[NACC][TM][TN];
#pragma unroll
  for (int a = 0; a < NACC; ++a)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[a][i][j][q] = 0.f;

  gload(0);
  lstore(0);
  __syncthreads();
  for (int ks = 0; ks < ksteps; ++ks) {
    const int buf = ks & 1;
    if (ks + 1 < ksteps) gload(ks + 1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int piece = kk * 2 + (lane >> 5);
      bf16x8 af[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = __builtin_bit_cast(bf16x8, As[buf][swz(wm * WM + i * 32 + (lane & 31), piece)]);
#pragma unroll
      for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const bf16x8 bf = __builtin_bit_cast(
              bf16x8, Bs[buf][swz(a * BN + wn * WN + j * 32 + (lane & 31), piece)]);
#pragma unroll
          for (int i = 0; i < TM; ++i)
            acc[a][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf, acc[a][i][j], 0, 0, 0);
        }
    }
    if (ks + 1 < ksteps) lstore(buf ^ 1);
    __syncthreads();
  }

  // D layout: lane l, register q -> row (q/4)*8 + (l/32)*4 + q%4, col l%32
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int row = row0 + wm * WM + i * 32 + (q >> 2) * 8 + (lane >> 5) * 4 + (q & 3);
        float v;
        if (DUAL) v = silu_mul(acc[0][i][j][q], acc[NACC - 1][i][j][q]);
        else v = acc[0][i][j][q];
        if (row < row1 && col < N) C[size_t(row) * N + col] = f32_to_bf16_bits(v);
      }
    }
}

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// ---------------------------------------- MFMA GEMM, 256x256 tile, 8 wavefronts
// Prefill-sized groups.  Block tile 256 rows x 256 weight rows (DUAL: 128 gate +
// the matching 128 up rows), 512 threads: wavefront (wm, wn) = (w/4, w%4) computes
// rows wm*128..+128 and the 64 weight rows of column block wn (DUAL: 32 gate + 32
// up), i.e. four 32-row blocks x two 32-column blocks = 128 accumulator registers.
// Operands go global -> LDS directly (`buffer_load_dwordx4 ... lds`, 16 B per
// lane, no register staging; a buffer descriptor per operand with the K step as
// scalar offset, which measured 1-4 % faster than 64-bit per-lane addresses and
// zero-fills rows past the tile's end); the
// per-lane offset is permuted so that the linear LDS write of a
// wavefront lands in the XOR-swizzled layout the MFMA operand reads expect
// (piece ^ (row/2)&7: the 16 lanes the LDS serves per cycle hit 16 different
// 16-byte columns).  Operand fragments are read one K sub-step ahead of the
// MFMAs that consume them.  Workgroup ids are remapped so that each XCD (own L2)
// walks a contiguous run of tiles, M tiles of one expert first: neighbours
// share the expert's weight panel and the activation panel.  Wavefronts w and
// w+4 (the two row halves) share a SIMD: while one of them waits (LDS latency, a
// load instruction being accepted, the barrier) the other keeps the matrix unit
// busy; on full tiles they do so in turns (see the two forms of the K loop).
// The operand pointers are __restrict__ on purpose: the compiler then knows that
// the LDS reads do not alias what the loads-to-LDS write (it cannot see their LDS
// side) and leaves the waiting for loads to the explicit vmcnt waits; without that
// it waits for every load in flight in front of each LDS read, which serialises
// the loop.  K step 64
// (128-byte rows: whole cache lines per row and load instruction); weights and
// activations have LDS rings of their own (see Ring).
// NBW = valid 32-row blocks of this wavefront's 128 rows (0..4).
// NB = valid 32-row blocks of the tile (1..8), WM = which half of the rows this
// wavefront computes; both compile-time so the K loop has no branches.  A weight
// stage holds 256 rows of 128 B, an activation stage NB*32 rows.  As many whole
// (activation + weight) stages as fit in the CU's 160 KB of LDS, at most four,
// give the depth of the weight ring; what is left takes up to two further
// activation stages (256-row tile: 2 weight + 3 activation stages = 160 KB;
// 160-row tile: 3 + 3; short tiles up to 4 + 6).  With the rotated K loop below
// the loads of a step must land three quarters of a step after the previous
// step's barrier, and the extra activation stage is worth 9 % on the 256-row
// tile.
// K step per stage: 64, i.e. 128-byte LDS rows, so that every load instruction
// moves whole cache lines.  (A K step of 32 would allow four stages for the tall
// tiles too, but its 64-byte row pieces halve the efficiency of the load path:
// measured 8 % slower on the 256-row tiles.)
// Eight e4m3 codes -> eight bf16 values of code * scale (exact widening to fp32,
// one fp32 multiply, round to nearest even).
__device__ __forceinline__ uint4 widen_scaled(uint2 c, float sc) {
  const f32x2 p0 = __builtin_amdgcn_cvt_pk_f32_fp8(c.x, false), p1 = __builtin_amdgcn_cvt_pk_f32_fp8(c.x, true);
  const f32x2 p2 = __builtin_amdgcn_cvt_pk_f32_fp8(c.y, false), p3 = __builtin_amdgcn_cvt_pk_f32_fp8(c.y, true);
  uint4 r;
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r.x) : "v"(p0[0] * sc), "v"(p0[1] * sc));
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r.y) : "v"(p1[0] * sc), "v"(p1[1] * sc));
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r.z) : "v"(p2[0] * sc), "v"(p2[1] * sc));
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r.w) : "v"(p3[0] * sc), "v"(p3[1] * sc));
  return r;
}

// One part of a K-split tile: `parts` workgroups share the tile's K range, part
// `slot - slot0` of them is this one; parts == 1: the whole K range, no partial sums.
struct SplitJob {
  int parts, slot, slot0;
  float* partial;          // [kCUs][kPartFloats]
  int32_t* ticket;         // arrival counter of the tile
};

// F8: the weight tile holds e4m3 codes (64-byte rows: four pieces), widened to
// bf16 on the way from LDS to the matrix unit.
// BR: weight rows of a stage (256, or 512 for the wide tiles of short row groups).
template <int NB, bool F8 = false, int BR = 256> struct Ring {
  static constexpr int kBK = 64;
  static constexpr int kPPR = kBK / 8;                              // 16-byte pieces per activation row
  static constexpr int kPPRB = F8 ? kBK / 16 : kBK / 8;             // ... per weight row
  static constexpr int kARows = NB * 32;
  static constexpr int kASlots = kARows * kPPR;                     // 16-byte slots of an A stage
  static constexpr int kBSlots = BR * kPPRB;                        // ... of a B stage
  static constexpr int kLds = 160 * 1024;
  static constexpr int kFit = kLds / ((kASlots + kBSlots) * 16);
  static constexpr int kSB = kFit > 4 ? 4 : kFit;                   // weight stages
  // LDS left over after kSB whole stages takes further activation stages
  static constexpr int kMore = (kLds - kSB * (kASlots + kBSlots) * 16) / (kASlots * 16);
  static constexpr int kSA = kSB + (kMore > MOE_RING_EXTRA_A ? MOE_RING_EXTRA_A : kMore);
};

// F8: Be0 / Be1 point at e4m3 codes, Se0 / Se1 at the expert's block scales of
// the 128-row block this wavefront's weight rows lie in ([K/128] values).  The
// scaled weight code * scale is rounded to bf16 before the MFMA (the exact
// per-block scale would need a second set of accumulators).
template <bool DUAL, int NB, int WM, bool F8, int BR = 256>
__device__ __forceinline__ void gemm8w_body(const uint16_t* __restrict__ A,
                                            const char* __restrict__ Be0,
                                            const char* __restrict__ Be1,
                                            const float* __restrict__ Se0,
                                            const float* __restrict__ Se1,
                                            uint16_t* __restrict__ C, int N, int K, int row0,
                                            int row1, int n0, uint4* smem, int wave, int kbeg,
                                            int klen, const SplitJob& job) {
  static_assert(BR == 256 || (BR == 512 && WM == 0 && NB <= 4), "wide tiles: all wavefronts on one row half");
  constexpr int NBW = NB - WM * 4 < 0 ? 0 : (NB - WM * 4 > 4 ? 4 : NB - WM * 4);
  constexpr int HALF = BR / 2;                       // DUAL: gate rows | up rows of a stage
  constexpr int SA = Ring<NB, F8, BR>::kSA, SB = Ring<NB, F8, BR>::kSB;
  constexpr int KS = Ring<NB, F8, BR>::kBK;          // K step
  constexpr int PPR = Ring<NB, F8, BR>::kPPR;        // pieces per activation row in LDS
  constexpr int PPRB = Ring<NB, F8, BR>::kPPRB;      // pieces per weight row in LDS
  constexpr int RPI = 64 / PPR;                      // rows filled by one load instruction
  constexpr int RPIB = 64 / PPRB;
  constexpr int WB = F8 ? 1 : 2;                     // bytes per weight element
  constexpr int AS = Ring<NB, F8, BR>::kASlots;      // slots of an A stage
  constexpr int BS = Ring<NB, F8, BR>::kBSlots;      // slots of a B stage
  uint4* const ringA = smem;
  uint4* const ringB = smem + SA * AS;
  const int lane = threadIdx.x & 63;
  const int wn = BR == 512 ? wave : wave & 3;        // column block of this wavefront
  const int ksteps = klen / KS;                      // this workgroup's K window starts at kbeg

  // LDS row r keeps its piece p at slot p ^ f(r): f = (r/2)&7 for 128-byte rows,
  // (r/4)&3 for 64-byte rows; both keep the 16 lanes the LDS serves per cycle
  // on 16 different 16-byte columns.
  auto slot = [&](int row, int piece) {
    return row * PPR + (piece ^ (PPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3));
  };
  auto slot_b = [&](int row, int piece) {
    return row * PPRB + (piece ^ (PPRB == 8 ? (row >> 1) & 7 : (row >> 2) & 3));
  };
  // loads: a wavefront instruction fills 64 consecutive slots = RPI rows.  Row
  // group rg = q*8 + wave; lane l -> row l/PPR, and it fetches the piece that
  // belongs in slot l%PPR of that row: (l%PPR) ^ ((rg*4 + l/16) & (PPR-1)).
  // A row groups exist for rg < NB*32/RPI.
  constexpr int AGROUPS = NB * 32 / RPI;
  constexpr int NAQ = AGROUPS / 8;                   // full rounds of 8 wavefronts
  constexpr int AREM = AGROUPS % 8;                  // wavefronts 0..AREM-1 load one more
  constexpr int NBQ = BR / RPIB / 8;                 // weight row groups per wavefront
  const int lrow = lane / PPR;
  // Operands through buffer descriptors: a wave-uniform base per operand (this
  // tile's first row / first weight row, at the K window's start), a 32-bit byte
  // offset per lane, and the K step as a scalar offset.  Rows past the tile's end
  // (or past the last weight row) are out of the descriptor's range and load zeros.
  const int arows = row1 - row0;
  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(A + size_t(row0) * K + kbeg), 0,
      int((size_t(arows - 1) * K + klen) * 2), 0x00020000);
  const int brows = (N - n0) < HALF * (DUAL ? 1 : 2) ? (N - n0) : HALF * (DUAL ? 1 : 2);
  const __amdgpu_buffer_rsrc_t rsrcB0 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(Be0 + (size_t(n0) * K + kbeg) * WB), 0,
      int((size_t(brows - 1) * K + klen) * WB), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB1 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>((DUAL ? Be1 : Be0) + (size_t(n0) * K + kbeg) * WB), 0,
      int((size_t(brows - 1) * K + klen) * WB), 0x00020000);
  int aoff[NAQ + 1], boff[NBQ];
#pragma unroll
  for (int q = 0; q < NAQ + 1; ++q) {
    const int rg = q * 8 + wave;
    const int piece = (lane % PPR) ^ ((rg * 4 + (lane >> 4)) & (PPR - 1));
    aoff[q] = ((rg * RPI + lrow) * K + piece * 8) * 2;
  }
#pragma unroll
  for (int q = 0; q < NBQ; ++q) {
    const int rg = q * 8 + wave;
    const int piece = (lane % PPRB) ^ ((rg * 4 + (lane >> 4)) & (PPRB - 1));
    const int br = rg * RPIB + lane / PPRB;
    const int bl = (DUAL && br >= HALF) ? br - HALF : br;     // row inside its matrix' tile
    boff[q] = bl * K * WB + piece * 16;
  }
  // weight row groups q: rows q*8*RPIB .. of the stage; the upper half is the up matrix
  auto b_is_up = [](int q) { return DUAL && q * 8 * RPIB >= HALF; };
#define MOE_LOAD_A(q, kcol, dst) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lptr_t)(dst), 16, aoff[q], (kcol) * 2, 0, 0)
#define MOE_LOAD_B(q, kcolb, dst)                                                                  \
  do {                                                                                             \
    if (b_is_up(q)) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB1, (lptr_t)(dst), 16, boff[q], (kcolb), 0, 0); \
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB0, (lptr_t)(dst), 16, boff[q], (kcolb), 0, 0);            \
  } while (0)
  const bool extra = AREM > 0 && wave < AREM;        // this wavefront loads one more A row group
  auto issue_a = [&](int ks) {
    const int kcol = ks * KS;
    uint4* st = ringA + (ks % SA) * AS;
#pragma unroll
    for (int q = 0; q < NAQ; ++q) MOE_LOAD_A(q, kcol, st + (q * 8 + wave) * 64);
    if (extra) MOE_LOAD_A(NAQ, kcol, st + (NAQ * 8 + wave) * 64);
  };
  auto issue_b = [&](int ks) {
    const int kcol = ks * KS * WB;
    uint4* st = ringB + (ks % SB) * BS;
#pragma unroll
    for (int q = 0; q < NBQ; ++q) MOE_LOAD_B(q, kcol, st + (q * 8 + wave) * 64);
  };
  // Issue group of step g (after its barrier): weights of step g+SB-1, then
  // activations of step g+SA-1 (SA >= SB).  Loads return in order, so at the
  // barrier of step ks everything younger than the weights of step ks may stay in
  // flight: the activation part of group ks-SB+1 (when SA > SB) and the SB-2 whole
  // groups after it.  Near the end of K, where groups shrink, wait for all.
  constexpr int YA = SA > SB ? 1 : 0;
  constexpr int YG = SB - 2;
  auto wait_step = [&](bool steady) {
    if (!steady) wait_vmcnt<0>();
    else if (extra) wait_vmcnt<YA * (NAQ + 1) + YG * (NAQ + 1 + NBQ)>();
    else wait_vmcnt<YA * NAQ + YG * (NAQ + NBQ)>();
  };

  constexpr int NA = NBW > 0 ? NBW : 1;
  f32x16 acc[NA][2];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  const int arow = WM * 128;
  const int brow0 = DUAL ? wn * 32 : wn * 64;
  const int brow1 = DUAL ? HALF + wn * 32 : wn * 64 + 32;
  constexpr int NKK = KS / 16;                       // MFMA sub-steps per K step

#pragma unroll
  for (int g = 1 - SA; g < 0; ++g) {
    if (g + SB - 1 >= 0 && g + SB - 1 < ksteps) issue_b(g + SB - 1);
    if (g + SA - 1 < ksteps) issue_a(g + SA - 1);
  }
  // One load instruction of a step's issue group: ops 0..NBQ-1 are the weight row
  // groups, NBQ..NBQ+NAQ-1 the activation row groups (weights first: see above).
  constexpr int NOPS = NBQ + NAQ;
  auto issue_op = [&](int op, uint4* stb, uint4* sta, int kcb, int kca) {
    if (op < NBQ) MOE_LOAD_B(op, kcb * WB, stb + (op * 8 + wave) * 64);
    else if (op < NOPS) MOE_LOAD_A(op - NBQ, kca, sta + ((op - NBQ) * 8 + wave) * 64);
  };
  // Two forms of the K loop.  Full 256-row tiles of bf16 weights alternate the two
  // wavefronts of a SIMD between memory and MFMA phases (measured 4-6 % faster on
  // the long-K GEMM-1, 1 % on GEMM-2).  Shorter tiles, where row half 1 has fewer
  // MFMAs than row half 0 and the phases would not balance (160-row tiles: 5 %
  // slower), and e4m3 weights, whose widening makes the memory phase the longer one
  // (7-9 % slower), keep all wavefronts in one phase with loads, LDS reads and MFMAs
  // interleaved.
  constexpr bool kAlternate = !F8 && NB == 8;
  if constexpr (kAlternate) {
  // The two wavefronts of a SIMD (w and w+4, the two row halves) take turns: a
  // step has four phases, each closed by a barrier, and a wavefront alternates
  // between a memory phase (issue half of its loads, read the operand fragments of
  // two K sub-steps) and an MFMA phase (the 4 x NBW MFMAs on those fragments); row
  // half 1 runs one phase behind row half 0, so that at any time one wavefront of a
  // SIMD feeds the matrix unit while the other one's loads and LDS reads are
  // accepted:
  //   phase   row half 0                      row half 1
  //   4j      loads B(j+SB-1), read (j, 0-1)   MFMAs (j-1, 2-3)
  //   4j+1    MFMAs (j, 0-1)                   loads B(j+SB-1), read (j, 0-1)
  //   4j+2    loads A(j+SA-1), read (j, 2-3)   MFMAs (j, 0-1)
  //   4j+3    MFMAs (j, 2-3)                   loads A(j+SA-1), read (j, 2-3)
  // Step j+1 must have landed when phase 4j+3 ends: every wavefront waits for its
  // own loads of that step before that barrier.  A stage is refilled only after
  // the barrier that follows its last read (B(j-1)'s stage in phase 4j or later,
  // A(j-1)'s in phase 4j+2 or later).  That is why all fragments of a half step are
  // read in the memory phase: a read left for the MFMA phase of row half 1 (phase
  // 4j+4 for sub-step 3 of step j) would meet row half 0's refill of the same
  // weight stage; such a variant measured 1 % faster and gave outputs that changed
  // from run to run on the 16 384-token step.
  uint4 fa[2][NA], fb[2][2];
  auto read_half = [&](int ks, int h) {
    if constexpr (NBW > 0) {
      const uint4* Ab = ringA + (ks % SA) * AS;
      const uint4* Bb = ringB + (ks % SB) * BS;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int piece = (h * 2 + sub) * 2 + (lane >> 5);
        fb[sub][0] = Bb[slot_b(brow0 + (lane & 31), piece)];
        fb[sub][1] = Bb[slot_b(brow1 + (lane & 31), piece)];
#pragma unroll
        for (int i = 0; i < NBW; ++i) fa[sub][i] = Ab[slot(arow + i * 32 + (lane & 31), piece)];
      }
    }
  };
  auto mma_half = [&]() {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const bf16x8 b0 = __builtin_bit_cast(bf16x8, fb[sub][0]);
      const bf16x8 b1 = __builtin_bit_cast(bf16x8, fb[sub][1]);
#pragma unroll
      for (int i = 0; i < NBW; ++i) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, fa[sub][i]);
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[i][0], 0, 0, 0);
        acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[i][1], 0, 0, 0);
      }
    }
  };
  // `drain`: this wavefront's LDS reads must have returned before the barrier
  // (the stage they read is refilled in the next phase).  Otherwise they may
  // still be in flight when the barrier is passed: the MFMAs that use them wait
  // for them one by one.
  auto phase_end = [&](auto drain_c) {
    __builtin_amdgcn_sched_barrier(0);               // nothing of the next phase moves in front of the barrier
    if constexpr (decltype(drain_c)::value) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr std::true_type drain{};
  constexpr std::false_type no_drain{};
  auto step = [&](int ks, auto steady_c) {
    constexpr bool ST = decltype(steady_c)::value;      // this step issues both of its load groups
    const int kb = ks + SB - 1, ka = ks + SA - 1;
    __builtin_amdgcn_sched_barrier(0);
    if (ST || kb < ksteps) issue_b(kb);
    read_half(ks, 0);
    __builtin_amdgcn_sched_barrier(0);
    phase_end(no_drain);
    mma_half();
    __builtin_amdgcn_sched_barrier(0);
    phase_end(no_drain);
    if (ST) issue_a(ka);
    read_half(ks, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (WM == 1) wait_step(ST);
    // row half 1 reads the last fragments of this step's weight stage here, and
    // row half 0 refills that stage in the next phase
    if constexpr (WM == 1) phase_end(drain); else phase_end(no_drain);
    mma_half();
    __builtin_amdgcn_sched_barrier(0);
    if (WM == 0) wait_step(ST);
    phase_end(no_drain);
  };
  wait_step(SA - 2 < ksteps);                                 // step 0 has landed
  phase_end(no_drain);
  if (WM == 1) phase_end(no_drain);                          // one phase behind row half 0
  const int steady_steps = ksteps - (SA - 1);
  int ks = 0;
  for (; ks < steady_steps; ++ks) step(ks, std::true_type{});
  for (; ks < ksteps; ++ks) step(ks, std::false_type{});
  if (WM == 0) phase_end(no_drain);
  } else {
  // One turn of the K loop, rotated by a sub-step so that the synchronisation for
  // step j sits in front of the LAST sub-step of step j-1:
  //   wait for the loads of step j, barrier  (every wavefront holds its last
  //     fragments of step j-1 in registers, so that step's stages are free)
  //   slot 0: issue loads | read fragments (j, 0) | MFMAs (j-1, 3)
  //   slot 1: issue loads | read fragments (j, 1) | MFMAs (j, 0)
  //   slot 2:               read fragments (j, 2) | MFMAs (j, 1)
  //   slot 3:               read fragments (j, 3) | MFMAs (j, 2)
  // The first LDS reads after a barrier are covered by MFMAs that are already
  // fed, and the load instructions of the step's issue group (which stall a
  // wavefront until the load path accepts them) are handed out between MFMAs,
  // ahead of the slot's LDS reads.  SPREAD: the issue group is unconditional (all
  // but the last SA-1 turns); otherwise it is issued in one go behind a range check.
  constexpr int NA2 = NA;
  uint4 fa[2][NA2], fb[2][2];
#pragma unroll
  for (int i = 0; i < NA2; ++i) fa[1][i] = make_uint4(0, 0, 0, 0);
  fb[1][0] = fb[1][1] = make_uint4(0, 0, 0, 0);     // the first turn multiplies zeros
  auto mfmas = [&](int set) {
    const bf16x8 b0 = __builtin_bit_cast(bf16x8, fb[set][0]);
    const bf16x8 b1 = __builtin_bit_cast(bf16x8, fb[set][1]);
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, fa[set][i]);
      acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[i][0], 0, 0, 0);
      acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[i][1], 0, 0, 0);
    }
  };
  constexpr int NSLOT = MOE_SPREAD_SLOTS;                    // slots that issue loads
  constexpr int OPK = (NOPS + NSLOT - 1) / NSLOT;            // load instructions per slot
  auto turn = [&](int ks, auto spread_c) {
    constexpr bool SPREAD = decltype(spread_c)::value && NBW > 0;
    // step ks must have landed
    wait_step(ks + SA - 2 < ksteps);
    // a bare barrier (no fence): __syncthreads() would also drain the younger loads
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // every wavefront has read all of step ks-1, so its stages can be refilled
    const int kb = ks + SB - 1, ka = ks + SA - 1;
    uint4* const stb = ringB + (kb % SB) * BS;
    uint4* const sta = ringA + (ka % SA) * AS;
    if constexpr (!SPREAD) {
      if (kb < ksteps) issue_b(kb);
      if (ka < ksteps) issue_a(ka);
    }
    if constexpr (NBW > 0) {
      const uint4* Ab = ringA + (ks % SA) * AS;
      const uint4* Bb = ringB + (ks % SB) * BS;
      float sc0 = 1.f, sc1 = 1.f;
      if constexpr (F8) { sc0 = Se0[ks >> 1]; sc1 = Se1[ks >> 1]; }   // one block = two K steps
      auto read_frags = [&](int kk, int set) {
        const int piece = kk * 2 + (lane >> 5);
        if constexpr (F8) {
          // sub-step kk: eight codes at bytes kk*16 + (lane/32)*8 of the row's 64
          const uint2 c0 = reinterpret_cast<const uint2*>(&Bb[slot_b(brow0 + (lane & 31), kk)])[lane >> 5];
          const uint2 c1 = reinterpret_cast<const uint2*>(&Bb[slot_b(brow1 + (lane & 31), kk)])[lane >> 5];
          fb[set][0] = widen_scaled(c0, sc0);
          fb[set][1] = widen_scaled(c1, sc1);
        } else {
          fb[set][0] = Bb[slot_b(brow0 + (lane & 31), piece)];
          fb[set][1] = Bb[slot_b(brow1 + (lane & 31), piece)];
        }
#pragma unroll
        for (int i = 0; i < NBW; ++i) fa[set][i] = Ab[slot(arow + i * 32 + (lane & 31), piece)];
      };
#pragma unroll
      for (int sl = 0; sl < NKK; ++sl) {
        const int set = sl & 1;                              // fragments read in this slot
        __builtin_amdgcn_sched_barrier(0);
        constexpr int NLD = OPK;
        const bool loads_here = sl < NSLOT;
        if constexpr (SPREAD) {
          if (sl < NSLOT) {
#pragma unroll
            for (int o = 0; o < OPK; ++o)
              if (sl * OPK + o < NOPS) issue_op(sl * OPK + o, stb, sta, kb * KS, ka * KS);
          }
        }
        read_frags(sl, set);
        mfmas(set ^ 1);
        if (NBW >= 2) {
          // one MFMA, then the loads while no LDS read of this wavefront is
          // outstanding, then MFMA / LDS read pairs
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (SPREAD && loads_here) __builtin_amdgcn_sched_group_barrier(0x020, NLD, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
          for (int i = 0; i < NBW + 1; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 2 * NBW - (NBW + 2), 0);
        }
      }
      if constexpr (SPREAD && AREM > 0) {
        if (extra)
          MOE_LOAD_A(NAQ, ka * KS, sta + (NAQ * 8 + wave) * 64);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  const int spread_steps = ksteps - (SA - 1);
  int ks = 0;
  for (; ks < spread_steps; ++ks) turn(ks, std::true_type{});
  for (; ks < ksteps; ++ks) turn(ks, std::false_type{});
  if constexpr (NBW > 0) mfmas(1);                           // sub-step 3 of the last step

  }
  // A K-split part leaves its fp32 accumulators in the workspace (register order:
  // 8-byte chunk c of thread t at index c*512 + t, so a wavefront's store is 512
  // contiguous bytes); the part that arrives last adds all parts in the
  // order of their K windows and carries on with the epilogue.  No workgroup waits
  // for another: every part counts itself in and all but the last one leave.
  if (job.parts > 1) {
    // The partial sums go past the XCD's own (non-coherent) L2 as device-scope
    // stores and are read back as device-scope loads, so no cache has to be
    // written back or invalidated as a whole; the wait below makes every store of
    // this part complete before the part counts itself in.
    uint64_t* const mine = reinterpret_cast<uint64_t*>(job.partial + size_t(job.slot) * kPartFloats) + threadIdx.x;
    if constexpr (NBW > 0) {
#pragma unroll
      for (int i = 0; i < NBW; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const uint64_t bits = uint64_t(__float_as_uint(acc[i][j][2 * q])) |
                                  (uint64_t(__float_as_uint(acc[i][j][2 * q + 1])) << 32);
            __hip_atomic_store(mine + ((i * 2 + j) * 8 + q) * 512, bits, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
          }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int32_t* const flag = reinterpret_cast<int32_t*>(smem);   // the rings are idle from here on
    if (threadIdx.x == 0) *flag = atomicAdd(job.ticket, 1);
    __syncthreads();
    if (*flag != job.parts - 1) return;
    if constexpr (NBW > 0) {
      // one 32x32 block at a time: its chunks of all (at most four) parts are
      // fetched together, then added in the order of the parts
      const uint64_t* const all = reinterpret_cast<const uint64_t*>(job.partial + size_t(job.slot0) * kPartFloats) + threadIdx.x;
#pragma unroll
      for (int i = 0; i < NBW; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          uint64_t v[kSplitMax][8];
#pragma unroll
          for (int p = 0; p < kSplitMax; ++p)
            if (p < job.parts) {
#pragma unroll
              for (int q = 0; q < 8; ++q)
                v[p][q] = __hip_atomic_load(all + size_t(p) * (kPartFloats / 2) + ((i * 2 + j) * 8 + q) * 512,
                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
#pragma unroll
          for (int p = 0; p < kSplitMax; ++p)
            if (p < job.parts) {
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                acc[i][j][2 * q] += __uint_as_float(uint32_t(v[p][q]));
                acc[i][j][2 * q + 1] += __uint_as_float(uint32_t(v[p][q] >> 32));
              }
            }
        }
    }
  }

  // Epilogue.  Lane l holds column l%32 of each 32x32 block and rows
  // (q/4)*8 + (l/32)*4 + q%4: two rows are rounded to bf16 by one packed convert
  // and stored as the low / high half.  Only the last 32-row block of a tile can
  // hold rows of the next expert's segment; the others are stored unpredicated.
  if constexpr (NBW > 0) {
    const int lrow = arow + (lane >> 5) * 4;                    // first row of this lane, tile-relative
    const int valid = row1 - row0 - lrow;                        // rows r (tile-relative to lrow) < valid exist
    uint16_t* const cl = C + size_t(row0 + lrow) * N + n0 + (lane & 31);
    auto put2 = [&](uint16_t* p, float v0, float v1, bool ok0, bool ok1) {
      uint32_t pk;   // bf16(v0) | bf16(v1) << 16, round to nearest even
      asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(v0), "v"(v1));
      if (ok0) p[0] = uint16_t(pk);
      if (ok1) p[N] = uint16_t(pk >> 16);
    };
    auto store_block = [&](int i, auto pred_c) {
      constexpr bool PRED = decltype(pred_c)::value;
#pragma unroll
      for (int q = 0; q < 16; q += 2) {
        const int r = i * 32 + (q >> 2) * 8 + (q & 3);
        const bool ok0 = !PRED || r < valid, ok1 = !PRED || r + 1 < valid;
        uint16_t* const p = cl + size_t(r) * N;
        if (DUAL) {
          if (n0 + wn * 32 < N)
            put2(p + wn * 32, silu_mul_fast(acc[i][0][q], acc[i][1][q]),
                 silu_mul_fast(acc[i][0][q + 1], acc[i][1][q + 1]), ok0, ok1);
        } else {
#pragma unroll
          for (int j = 0; j < 2; ++j)
            if (n0 + wn * 64 + j * 32 < N)
              put2(p + wn * 64 + j * 32, acc[i][j][q], acc[i][j][q + 1], ok0, ok1);
        }
      }
    };
    const bool full = row1 - row0 == NB * 32;
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      if (i == NBW - 1 && WM * 4 + NBW == NB && !full) store_block(i, std::true_type{});
      else store_block(i, std::false_type{});
    }
  }
}

#undef MOE_LOAD_A
#undef MOE_LOAD_B

template <bool DUAL, int NB, bool F8, bool WIDE>
__device__ __forceinline__ void gemm8w_tile(const uint16_t* A, const char* Be0, const char* Be1,
                                            const float* Se0, const float* Se1, uint16_t* C, int N,
                                            int K, int row0, int row1, int n0, uint4* smem,
                                            int wave, int kbeg, int klen, const SplitJob& job) {
  if constexpr (WIDE) {
    // at most four row blocks: all eight wavefronts work on them, each on its own
    // 32 (DUAL) or 64 weight rows of a 512-row stage
    gemm8w_body<DUAL, NB, 0, F8, 512>(A, Be0, Be1, Se0, Se1, C, N, K, row0, row1, n0, smem, wave, kbeg, klen, job);
  } else {
    if (wave < 4) gemm8w_body<DUAL, NB, 0, F8>(A, Be0, Be1, Se0, Se1, C, N, K, row0, row1, n0, smem, wave, kbeg, klen, job);
    else gemm8w_body<DUAL, NB, 1, F8>(A, Be0, Be1, Se0, Se1, C, N, K, row0, row1, n0, smem, wave, kbeg, klen, job);
  }
}

// Leftover tiles.  The hardware hands workgroups to CUs in the order of their
// ids, so when the number of tiles is not a multiple of the 256 CUs the last
// `left` tiles run on `left` CUs while the rest idle for a whole tile time.  When
// at most half of the CUs would be busy, those tiles are cut along K into `parts`
// workgroups each (parts * left <= 256), placed at the end of the grid; everything
// is derived from the tile count on the device, so there is no host round trip.
// The same rule spreads a launch of a few tiles (a shared expert at a decode
// batch) over the chip.
// WIDE: tiles of at most 128 rows (the table is built with that height) x 512
// weight rows, for GEMM-2 launches whose groups are short: twice the weight bytes
// per K step and barrier, half as many tiles.
template <bool DUAL, bool F8, bool WIDE = false>
__global__ __launch_bounds__(512) void ffn_gemm8w_kernel(
    const uint16_t* __restrict__ A, const void* __restrict__ B0, const void* __restrict__ B1,
    const float* __restrict__ S0, const float* __restrict__ S1, uint16_t* __restrict__ C, int N,
    int K, const int32_t* __restrict__ tiles, int m_fastest, float* __restrict__ partial,
    int32_t* __restrict__ tickets) {
  constexpr int BN = (DUAL ? 128 : 256) * (WIDE ? 2 : 1);
  extern __shared__ uint4 smem[];
  const int n_ntiles = (N + BN - 1) / BN;
  const int total = tiles[0] * n_ntiles;
  const int ksteps_all = K / 64;
  const int pid = blockIdx.x;
  const int left = total % kCUs;
  int parts = 1;
  if (partial && left > 0 && left <= kCUs / 2) {
    parts = kCUs / left;
    parts = parts < kSplitMax ? parts : kSplitMax;
    const int cap = ksteps_all / kSplitMinSteps;
    parts = parts < cap ? parts : cap;
  }
  int logical, part = 0;
  SplitJob job{1, 0, 0, partial, tickets};
  if (parts >= 2) {
    // whole rounds first, every XCD walking a contiguous run of their tiles, then
    // the parts of the leftover tiles
    const int full = total - left;
    if (pid < full) {
      logical = (pid & 7) * (full >> 3) + (pid >> 3);
    } else {
      const int q = pid - full;
      if (q >= left * parts) return;
      const int j = q / parts;
      part = q - j * parts;
      logical = full + j;
      job.parts = parts;
      job.slot = q;
      job.slot0 = j * parts;
      job.ticket = tickets + j;
    }
  } else {
    const int per_xcd = (total + 7) >> 3;
    logical = (pid & 7) * per_xcd + (pid >> 3);
    if ((pid >> 3) >= per_xcd || logical >= total) return;
  }
  int mtile = logical / n_ntiles, ntile = logical - mtile * n_ntiles;
  if (m_fastest) {
    // Inside an expert's block of tiles: groups of up to four M tiles; per group
    // all N tiles, M tile fastest.  The ~32 workgroups an XCD runs at a time then
    // form a (4 M tiles) x (8 N tiles) patch: every weight panel is shared by
    // four of them, every activation panel by eight.
    const int first = tiles[4 + kTileRec * mtile], cnt = tiles[5 + kTileRec * mtile];
    const int local = logical - first * n_ntiles;
    const int gsz = 4 * n_ntiles;
    const int grp = local / gsz, rem = local - grp * gsz;
    const int left_m = cnt - grp * 4;
    const int mc = left_m < 4 ? left_m : 4;
    ntile = rem / mc;
    mtile = first + grp * 4 + (rem - ntile * mc);
  }
  const int e = tiles[1 + kTileRec * mtile], row0 = tiles[2 + kTileRec * mtile],
            row1 = tiles[3 + kTileRec * mtile];
  const int n0 = ntile * BN;
  // this workgroup's window of K steps (even bounds: a block scale spans two steps)
  int kb = 0, ke = ksteps_all;
  if (job.parts > 1) {
    kb = (part * ksteps_all / job.parts) & ~1;
    ke = part == job.parts - 1 ? ksteps_all : (((part + 1) * ksteps_all / job.parts) & ~1);
  }
  constexpr int WB = F8 ? 1 : 2;
  const char* Be0 = static_cast<const char*>(B0) + size_t(e) * N * K * WB;
  const char* Be1 = DUAL ? static_cast<const char*>(B1) + size_t(e) * N * K * WB : nullptr;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // F8: the scales of the 128-row block this wavefront's weight rows lie in
  const float* Se0 = nullptr;
  const float* Se1 = nullptr;
  if constexpr (F8) {
    const int nkb = K / 128, nnb = N / 128;
    int nb = (n0 + (WIDE ? wave : wave & 3) * (DUAL ? 32 : 64)) / 128;
    nb = nb < nnb ? nb : nnb - 1;
    Se0 = S0 + (size_t(e) * nnb + nb) * nkb + (kb >> 1);
    Se1 = DUAL ? S1 + (size_t(e) * nnb + nb) * nkb + (kb >> 1) : Se0;
  }
#define MOE_TILE_(NBV)                                                                        \
  gemm8w_tile<DUAL, NBV, F8, WIDE>(A, Be0, Be1, Se0, Se1, C, N, K, row0, row1, n0, smem, wave,   \
                                   kb * 64, (ke - kb) * 64, job)
  if constexpr (WIDE) {
    switch ((row1 - row0 + 31) >> 5) {   // valid 32-row blocks of the tile: at most four
      case 1: MOE_TILE_(1); break;
      case 2: MOE_TILE_(2); break;
      case 3: MOE_TILE_(3); break;
      default: MOE_TILE_(4); break;
    }
  } else {
    switch ((row1 - row0 + 31) >> 5) {   // valid 32-row blocks of the tile
      case 1: MOE_TILE_(1); break;
      case 2: MOE_TILE_(2); break;
      case 3: MOE_TILE_(3); break;
      case 4: MOE_TILE_(4); break;
      case 5: MOE_TILE_(5); break;
      case 6: MOE_TILE_(6); break;
      case 7: MOE_TILE_(7); break;
      default: MOE_TILE_(8); break;
    }
  }
#undef MOE_TILE_
}

// ----------------------------------------- MFMA GEMM, weight streaming (decode)
// Few rows per expert: the work is reading every weight once.  Tile = 32 rows x
// 64 weight rows (DUAL: 32 gate + the matching 32 up rows); the four wavefronts
// of a workgroup split K between them (wavefront w takes K slices w, w+4, ...,
// a slice being 128 bytes of every weight row: 64 bf16 or 128 e4m3 values), each
// with its own register-staged pipeline: no LDS, no barrier until the partial
// sums are added in a fixed order at the end.  Many small workgroups (n tiles of
// 32 / 64 columns) and two slices of loads in flight per wavefront keep all of
// HBM busy even when a single expert holds most rows; M tiles of one expert are
// neighbours in the grid, so its weights are read from HBM once.
// Inside a slice, MFMA sub-step kk of lane half h covers k = h*W/2 + kk*8 .. +8
// (W = slice width) for BOTH operands, so every lane reads one contiguous run.
template <bool DUAL, bool FP8>
__global__ __launch_bounds__(256) void ffn_skinny_kernel(
    const uint16_t* __restrict__ A, const void* __restrict__ B0, const void* __restrict__ B1,
    const float* __restrict__ S0, const float* __restrict__ S1, uint16_t* __restrict__ C, int N,
    int K, const int32_t* __restrict__ tiles) {
  constexpr int W = FP8 ? 128 : 64;          // K values per slice
  constexpr int NKK = W / 16;                // MFMA sub-steps per slice
  constexpr int BN = DUAL ? 32 : 64;         // output columns per workgroup
  constexpr int BL = FP8 ? NKK / 2 : NKK;    // 16-byte loads per lane, slice and weight block
  __shared__ float red[4][2][16][64];        // partial sums of the four wavefronts

  const int n_ntiles = (N + BN - 1) / BN;
  const int total = tiles[0] * n_ntiles;
  if (int(blockIdx.x) >= total) return;
  int mtile = blockIdx.x / n_ntiles;
  const int first = tiles[4 + kTileRec * mtile], cnt = tiles[5 + kTileRec * mtile];
  const int local = blockIdx.x - first * n_ntiles;      // inside the expert: M tile fastest
  const int ntile = local / cnt;
  mtile = first + (local - ntile * cnt);
  const int e = tiles[1 + kTileRec * mtile], row0 = tiles[2 + kTileRec * mtile],
            row1 = tiles[3 + kTileRec * mtile];
  const int n0 = ntile * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = lane >> 5;
  const size_t wb = FP8 ? 1 : 2;
  // this lane's rows: activation row, and the weight row of each of the two blocks.
  // Lanes past the tile's last row load nothing (their fragment stays zero and
  // their output rows are not stored): a short tile asks the memory pipeline for
  // its real rows only.
  int ar = row0 + (lane & 31);
  const bool a_valid = ar < row1;
  ar = a_valid ? ar : row1 - 1;
  const uint16_t* arow = A + size_t(ar) * K + h * (W / 2);
  const char* brow[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    int n = n0 + (DUAL ? 0 : j * 32) + (lane & 31);
    n = n < N ? n : N - 1;
    const char* base = static_cast<const char*>((DUAL && j == 1) ? B1 : B0) + size_t(e) * N * K * wb;
    brow[j] = base + (size_t(n) * K + h * (W / 2)) * wb;
  }

  f32x16 acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;

  struct Slice { uint4 a[NKK]; uint4 b[2][BL]; };
  auto load = [&](int sl, Slice& r) {
    const int k0 = sl * W;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      if (a_valid) r.a[kk] = *reinterpret_cast<const uint4*>(arow + k0 + kk * 8);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < BL; ++q)
        r.b[j][q] = *reinterpret_cast<const uint4*>(brow[j] + size_t(k0) * wb + q * 16);
  };
  auto compute = [&](int sl, const Slice& r) {
    if constexpr (FP8) {
      // one scale block along K per slice; the 32 columns lie inside one block
      const int nkb = (K + 127) / 128, nnb = (N + 127) / 128;
      f32x16 part[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int q = 0; q < 16; ++q) part[j][q] = 0.f;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          // eight codes of this sub-step -> eight bf16 (exact)
          const uint4 v = r.b[j][kk >> 1];
          const uint32_t c0 = (kk & 1) ? v.z : v.x, c1 = (kk & 1) ? v.w : v.y;
          const f32x2 p0 = __builtin_amdgcn_cvt_pk_f32_fp8(c0, false), p1 = __builtin_amdgcn_cvt_pk_f32_fp8(c0, true);
          const f32x2 p2 = __builtin_amdgcn_cvt_pk_f32_fp8(c1, false), p3 = __builtin_amdgcn_cvt_pk_f32_fp8(c1, true);
          // upper halves of the two floats side by side (the lower halves are zero:
          // an e4m3 value has three mantissa bits), one byte permute per pair
          auto pack = [](f32x2 p) {
            return __builtin_amdgcn_perm(__float_as_uint(p[1]), __float_as_uint(p[0]), 0x07060302u);
          };
          const uint4 w8 = make_uint4(pack(p0), pack(p1), pack(p2), pack(p3));
          part[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, r.a[kk]),
                                                            __builtin_bit_cast(bf16x8, w8), part[j], 0, 0, 0);
        }
        int n = n0 + (DUAL ? 0 : j * 32);
        n = n < N ? n : N - 1;
        const float* S = (DUAL && j == 1) ? S1 : S0;
        const float sc = S[(size_t(e) * nnb + n / 128) * nkb + sl];
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[j][q] = fmaf(sc, part[j][q], acc[j][q]);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, r.a[kk]),
                                                           __builtin_bit_cast(bf16x8, r.b[j][kk]),
                                                           acc[j], 0, 0, 0);
    }
  };

  const int nslices = K / W;
  Slice r0, r1;
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) r0.a[kk] = r1.a[kk] = make_uint4(0, 0, 0, 0);
  int sl = wave;
  if (sl < nslices) load(sl, r0);
  while (sl < nslices) {                     // two slices per trip: r0 and r1 alternate
    if (sl + 4 < nslices) load(sl + 4, r1);
    compute(sl, r0);
    sl += 4;
    if (sl >= nslices) break;
    if (sl + 4 < nslices) load(sl + 4, r0);
    compute(sl, r1);
    sl += 4;
  }

  // add the four partial sums in a fixed order: wavefront w finishes registers 4w..4w+3
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) red[wave][j][q][lane] = acc[j][q];
  __syncthreads();
#pragma unroll
  for (int qq = 0; qq < 4; ++qq) {
    const int q = wave * 4 + qq;
    float v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      v[j] = ((red[0][j][q][lane] + red[1][j][q][lane]) + red[2][j][q][lane]) + red[3][j][q][lane];
    // D layout: lane l, register q -> row (q/4)*8 + (l/32)*4 + q%4, col l%32
    const int row = row0 + (q >> 2) * 8 + (lane >> 5) * 4 + (q & 3);
    if (row >= row1) continue;
    if (DUAL) {
      const int col = n0 + (lane & 31);
      if (col < N) C[size_t(row) * N + col] = f32_to_bf16_bits(silu_mul(v[0], v[1]));
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = n0 + j * 32 + (lane & 31);
        if (col < N) C[size_t(row) * N + col] = f32_to_bf16_bits(v[j]);
      }
    }
  }
}

// ------------------------------------------------------------ fp32 GEMM
// Plain VALU kernel for the fp32 configuration: 64x64 tile, 16x16 threads,
// 4x4 outputs per thread, K step 32; the next step's operands are fetched into
// registers while the current step is computed from LDS.
template <bool DUAL>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ A,
                                                     const float* __restrict__ B0,
                                                     const float* __restrict__ B1,
                                                     float* __restrict__ C, int N, int K,
                                                     const int32_t* __restrict__ tiles) {
  constexpr int TB = 64, TK = 32, PER = TB * TK / 256;
  __shared__ __align__(16) float As[TK][TB + 4];
  __shared__ __align__(16) float Bg[TK][TB + 4];
  __shared__ __align__(16) float Bu[DUAL ? TK : 1][TB + 4];
  const int n_ntiles = (N + TB - 1) / TB;
  const int mtile = blockIdx.x / n_ntiles, ntile = blockIdx.x % n_ntiles;
  if (mtile >= tiles[0]) return;
  const int e = tiles[1 + kTileRec * mtile], row0 = tiles[2 + kTileRec * mtile],
            row1 = tiles[3 + kTileRec * mtile];
  const int n0 = ntile * TB;
  const float* Be0 = B0 + size_t(e) * N * K;
  const float* Be1 = DUAL ? B1 + size_t(e) * N * K : nullptr;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float g[4][4] = {}, u[4][4] = {};
  float ra[PER], rg[PER], ru[PER];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int r = idx / TK, k = k0 + idx % TK;
      int ar = row0 + r; ar = ar < row1 ? ar : row1 - 1;
      int bn = n0 + r;   bn = bn < N ? bn : N - 1;
      ra[i] = k < K ? A[size_t(ar) * K + k] : 0.f;
      rg[i] = k < K ? Be0[size_t(bn) * K + k] : 0.f;
      if (DUAL) ru[i] = k < K ? Be1[size_t(bn) * K + k] : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int r = idx / TK, kk = idx % TK;
      As[kk][r] = ra[i];
      Bg[kk][r] = rg[i];
      if (DUAL) Bu[kk][r] = ru[i];
    }
    __syncthreads();
    if (k0 + TK < K) fetch(k0 + TK);
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      // rows of the LDS tiles are 68 floats, so groups of four stay 16-byte aligned
      const float4 a4 = *reinterpret_cast<const float4*>(&As[kk][ty * 4]);
      const float4 g4 = *reinterpret_cast<const float4*>(&Bg[kk][tx * 4]);
      const float4 u4 = DUAL ? *reinterpret_cast<const float4*>(&Bu[kk][tx * 4]) : make_float4(0.f, 0.f, 0.f, 0.f);
      const float a[4] = {a4.x, a4.y, a4.z, a4.w}, bg[4] = {g4.x, g4.y, g4.z, g4.w},
                  bu[4] = {u4.x, u4.y, u4.z, u4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          g[i][j] = fmaf(a[i], bg[j], g[i][j]);
          if (DUAL) u[i][j] = fmaf(a[i], bu[j], u[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = row0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (row < row1 && col < N) {
        float v = g[i][j];
        if (DUAL) v = v / (1.0f + expf(-v)) * u[i][j];
        C[size_t(row) * N + col] = v;
      }
    }
}

template <int BM, int BN1, int WM, int WN1, int BN2, int WN2>
void launch_mfma_pair(const moe_config& c, int n_experts, const void* xs, const int32_t* offsets,
                      int rows_capacity, const void* w_gate, const void* w_up, const void* w_down,
                      const float* s_gate, const float* s_up, const float* s_down, void* ys,
                      const FfnWs& ws, hipStream_t s) {
  const int H = c.hidden, I = c.inter_local;
  const int max_mt = rows_capacity / BM + n_experts;
  MOE_LAUNCH(MOE_K_FFN_TILES, ffn_tiles_kernel, dim3(1), dim3(256), 0, s, offsets, n_experts, BM,
                     rows_capacity, ws.tiles, max_mt < ws.max_tiles ? max_mt : ws.max_tiles, 0, 0,
             (int32_t*)nullptr, (int32_t*)nullptr);
  const int nt1 = (I + BN1 - 1) / BN1, nt2 = (H + BN2 - 1) / BN2;
  auto k1 = ffn_gemm_kernel<BM, BN1, WM, WN1, true>;
  auto k2 = ffn_gemm_kernel<BM, BN2, WM, WN2, false>;
  constexpr int lds1 = 2 * (BM + 2 * BN1) * 8 * 16, lds2 = 2 * (BM + BN2) * 8 * 16;
  static uint64_t opted1 = 0, opted2 = 0;
  lds_opt_in(reinterpret_cast<const void*>(k1), lds1, opted1);
  lds_opt_in(reinterpret_cast<const void*>(k2), lds2, opted2);
  MOE_LAUNCH(MOE_K_FFN_GEMM1, k1, dim3(size_t(max_mt) * nt1), dim3(256), lds1, s,
                     static_cast<const uint16_t*>(xs), w_gate, w_up,
                     static_cast<uint16_t*>(ws.hmid), I, H, ws.tiles);
  MOE_LAUNCH(MOE_K_FFN_GEMM2, k2, dim3(size_t(max_mt) * nt2), dim3(256), lds2, s,
                     static_cast<const uint16_t*>(ws.hmid), w_down, (const void*)nullptr,
                     static_cast<uint16_t*>(ys), H, I, ws.tiles);
}

template <bool FP8>
void launch_skinny(const moe_config& c, int n_experts, const void* xs, const int32_t* offsets,
                   int rows_capacity, const void* w_gate, const void* w_up, const void* w_down,
                   const float* s_gate, const float* s_up, const float* s_down, void* ys,
                   const FfnWs& ws, hipStream_t s) {
  const int H = c.hidden, I = c.inter_local;
  const int max_mt = rows_capacity / 32 + n_experts;
  MOE_LAUNCH(MOE_K_FFN_TILES, ffn_tiles_kernel, dim3(1), dim3(256), 0, s, offsets, n_experts, 32,
             rows_capacity, ws.tiles, max_mt < ws.max_tiles ? max_mt : ws.max_tiles, 0, 0,
             (int32_t*)nullptr, (int32_t*)nullptr);
  const int nt1 = (I + 31) / 32, nt2 = (H + 63) / 64;
  MOE_LAUNCH(MOE_K_FFN_GEMM1, (ffn_skinny_kernel<true, FP8>), dim3(size_t(max_mt) * nt1), dim3(256),
             0, s, static_cast<const uint16_t*>(xs), w_gate, w_up, s_gate, s_up,
             static_cast<uint16_t*>(ws.hmid), I, H, ws.tiles);
  MOE_LAUNCH(MOE_K_FFN_GEMM2, (ffn_skinny_kernel<false, FP8>), dim3(size_t(max_mt) * nt2), dim3(256),
             0, s, static_cast<const uint16_t*>(ws.hmid), w_down, (const void*)nullptr, s_down,
             (const float*)nullptr, static_cast<uint16_t*>(ys), H, I, ws.tiles);
}

template <bool F8>
void launch_mfma256(const moe_config& c, int n_experts, const void* xs, const int32_t* offsets,
                    int rows_capacity, const void* w_gate, const void* w_up, const void* w_down,
                    const float* s_gate, const float* s_up, const float* s_down, void* ys,
                    const FfnWs& ws, hipStream_t s) {
  const int H = c.hidden, I = c.inter_local;
  // Few rows per expert means the weights are streamed about once: cap the tile
  // height at 160 rows there, which leaves room for a three-stage ring.
  // GEMM-2 (K = I_loc is short, N = H wide) is best with 256-row tiles throughout
  // (measured); when the two heights differ a second workgroup of the table
  // kernel builds GEMM-2's table.
  // GEMM-2 of short groups (at most 96 rows per expert on average: a decode batch or
  // a cold EP share) takes 128-row tiles x 512 weight rows when the experts still
  // give at least one such tile per CU; otherwise the narrower tiles keep more CUs
  // streaming.  Measured on the 128-expert layer (hidden 2048, I 768, bf16): 85 ->
  // 81, 94 -> 86, 102 -> 92 us at 32 / 64 / 96 rows per expert, 110 -> 115 us at 128;
  // e4m3 weights at 64 rows per expert (32 experts, hidden 7168): 73 -> 61 us.
  // GEMM-1 keeps the narrow tiles: its wide form was slower at every size (the
  // 512-row bf16 stage leaves room for two ring stages only).
  const bool wide2 = rows_capacity / n_experts <= 96 && long(n_experts) * ((H + 511) / 512) >= kCUs;
  const int bm = rows_capacity / n_experts <= 320 ? 160 : 256;
  const int bm2 = wide2 ? 128 : 256;
  const int max_mt = rows_capacity / bm + n_experts;
  const int max_mt2 = rows_capacity / bm2 + n_experts;
  // one bound for both tables: the one with the shorter tiles can hold more
  const int most = max_mt > max_mt2 ? max_mt : max_mt2;
  const int cap = most < ws.max_tiles ? most : ws.max_tiles;
  int32_t* const tiles2 = bm2 == bm ? ws.tiles : ws.tiles2;
  MOE_LAUNCH(MOE_K_FFN_TILES, ffn_tiles_kernel, dim3(bm2 == bm ? 1 : 2), dim3(256), 0, s, offsets,
             n_experts, bm, rows_capacity, ws.tiles, cap, 1, bm2, tiles2, ws.tickets);
  const int nt1 = (I + 127) / 128, nt2 = wide2 ? (H + 511) / 512 : (H + 255) / 256;
  constexpr int lds = 160 * 1024;         // all of a CU's LDS: the rings of the tallest tile fill it
  // room for the parts of the leftover tiles behind the whole tiles
  const int g1 = (max_mt * nt1 + 7) / 8 * 8 + kCUs, g2 = (max_mt2 * nt2 + 7) / 8 * 8 + kCUs;
  auto k1 = ffn_gemm8w_kernel<true, F8, false>;
  auto k2 = wide2 ? ffn_gemm8w_kernel<false, F8, true> : ffn_gemm8w_kernel<false, F8, false>;
  static uint64_t opted1 = 0, opted2 = 0, opted2w = 0;
  lds_opt_in(reinterpret_cast<const void*>(k1), lds, opted1);
  lds_opt_in(reinterpret_cast<const void*>(k2), lds, wide2 ? opted2w : opted2);
  MOE_LAUNCH(MOE_K_FFN_GEMM1, k1, dim3(g1), dim3(512), lds, s, static_cast<const uint16_t*>(xs),
             w_gate, w_up, s_gate, s_up, static_cast<uint16_t*>(ws.hmid), I, H, ws.tiles, 1,
             ws.partial, ws.tickets);
  MOE_LAUNCH(MOE_K_FFN_GEMM2, k2, dim3(g2), dim3(512), lds, s,
             static_cast<const uint16_t*>(ws.hmid), w_down, (const void*)nullptr, s_down,
             (const float*)nullptr, static_cast<uint16_t*>(ys), H, I, tiles2, 1, ws.partial,
             ws.tickets + kSplitTickets);
}

// Between the two: a handful of rows per expert.  GEMM-1 (K = H long) streams its
// weights fastest through the LDS rings of the tall-tile kernel even when a tile
// holds one or two row blocks; GEMM-2 (K = I_loc short, N = H wide) is best as
// many small weight-streaming workgroups.  Each kernel gets its own tile table.
template <bool F8>
void launch_mixed(const moe_config& c, int n_experts, const void* xs, const int32_t* offsets,
                  int rows_capacity, const void* w_gate, const void* w_up, const void* w_down,
                  const float* s_gate, const float* s_up, const float* s_down, void* ys,
                  const FfnWs& ws, hipStream_t s) {
  const int H = c.hidden, I = c.inter_local;
  const int bm = 160, bm2 = 32;
  const int max_mt = rows_capacity / bm + n_experts;
  const int max_mt2 = rows_capacity / bm2 + n_experts;
  const int cap = max_mt2 < ws.max_tiles ? max_mt2 : ws.max_tiles;
  MOE_LAUNCH(MOE_K_FFN_TILES, ffn_tiles_kernel, dim3(2), dim3(256), 0, s, offsets, n_experts, bm,
             rows_capacity, ws.tiles, cap, 1, bm2, ws.tiles2, ws.tickets);
  const int nt1 = (I + 127) / 128, nt2 = (H + 63) / 64;
  constexpr int lds = 160 * 1024;
  const int g1 = (max_mt * nt1 + 7) / 8 * 8 + kCUs;
  auto k1 = ffn_gemm8w_kernel<true, F8>;
  static uint64_t opted1 = 0;
  lds_opt_in(reinterpret_cast<const void*>(k1), lds, opted1);
  MOE_LAUNCH(MOE_K_FFN_GEMM1, k1, dim3(g1), dim3(512), lds, s, static_cast<const uint16_t*>(xs),
             w_gate, w_up, s_gate, s_up, static_cast<uint16_t*>(ws.hmid), I, H, ws.tiles, 1,
             ws.partial, ws.tickets);
  MOE_LAUNCH(MOE_K_FFN_GEMM2, (ffn_skinny_kernel<false, F8>), dim3(size_t(max_mt2) * nt2), dim3(256),
             0, s, static_cast<const uint16_t*>(ws.hmid), w_down, (const void*)nullptr, s_down,
             (const float*)nullptr, static_cast<uint16_t*>(ys), H, I, ws.tiles2);
}

}  // namespace

hipError_t launch_expert_ffn(const moe_config& c, int n_experts, const void* xs,
                             const int32_t* offsets, int rows_capacity, const void* w_gate,
                             const void* w_up, const void* w_down, const float* s_gate,
                             const float* s_up, const float* s_down, void* ys, const FfnWs& ws,
                             hipStream_t s) {
  const int H = c.hidden, I = c.inter_local;
  if (c.act_dtype == MOE_F32) {
    const int BM = 64;
    const int max_mt = rows_capacity / BM + n_experts;
    MOE_LAUNCH(MOE_K_FFN_TILES, ffn_tiles_kernel, dim3(1), dim3(256), 0, s, offsets, n_experts, BM,
                       rows_capacity, ws.tiles, max_mt < ws.max_tiles ? max_mt : ws.max_tiles, 0, 0,
             (int32_t*)nullptr, (int32_t*)nullptr);
    MOE_LAUNCH(MOE_K_FFN_GEMM1, ffn_f32_kernel<true>, dim3(size_t(max_mt) * ((I + 63) / 64)), dim3(256), 0,
                       s, static_cast<const float*>(xs), static_cast<const float*>(w_gate),
                       static_cast<const float*>(w_up), static_cast<float*>(ws.hmid), I, H,
                       ws.tiles);
    MOE_LAUNCH(MOE_K_FFN_GEMM2, ffn_f32_kernel<false>, dim3(size_t(max_mt) * ((H + 63) / 64)), dim3(256), 0,
                       s, static_cast<const float*>(ws.hmid), static_cast<const float*>(w_down),
                       nullptr, static_cast<float*>(ys), H, I, ws.tiles);
    return hipGetLastError();
  }
  // rows per expert can only be bounded from above on the host; pick the M
  // tile from that bound (decode batches get the short tiles)
  const int avg = rows_capacity / n_experts;
  const bool fp8 = c.weight_dtype == MOE_FP8_E4M3_B128;
#define MOE_FFN_ARGS c, n_experts, xs, offsets, rows_capacity, w_gate, w_up, w_down, s_gate, s_up, s_down, ys, ws, s
  if (fp8 && H % 128 == 0 && I % 128 == 0 && avg > 12) {
    // e4m3 weight tiles in the LDS rings of the tall-tile kernel (the scaled weight
    // is rounded to bf16 there; below, the scale multiplies fp32 partial sums)
    launch_mfma256<true>(MOE_FFN_ARGS);
  } else if (fp8) {
    // the configuration check admits fp8 weights only with hidden and intermediate
    // sizes that are multiples of 128
    launch_skinny<true>(MOE_FFN_ARGS);
  } else if (H % BK == 0 && I % BK == 0) {
    // measured on the 128-expert layer (hidden 2048, I 768): with at most two rows
    // per expert the weight-streaming kernel wins both GEMMs, from about twelve on
    // the tall-tile kernel does, in between each takes the GEMM it is better at
    if (avg <= 2) launch_skinny<false>(MOE_FFN_ARGS);
    else if (avg <= 12) launch_mixed<false>(MOE_FFN_ARGS);
    else launch_mfma256<false>(MOE_FFN_ARGS);
  } else if (avg <= 32) {
    launch_mfma_pair<32, 128, 32, 32, 256, 64>(MOE_FFN_ARGS);
  } else if (avg <= 64) {
    launch_mfma_pair<64, 128, 64, 32, 256, 64>(MOE_FFN_ARGS);
  } else {
    launch_mfma_pair<128, 64, 64, 32, 128, 64>(MOE_FFN_ARGS);
  }
#undef MOE_FFN_ARGS
  return hipGetLastError();
}

}  // namespace moe

