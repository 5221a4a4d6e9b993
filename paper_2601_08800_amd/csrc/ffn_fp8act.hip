// Expert FFN with 8-bit activations: both GEMM operands are e4m3, the matrix
// cores run `v_mfma_f32_32x32x64_f8f6f4` (twice the rate of the bf16 MFMA).
//
//   quant   one wavefront per row, 16 lanes per block of 128 columns: amax -> scale =
//           amax / 448 (1 for an all-zero block), code = e4m3(x / scale) after a
//           clamp to +-448; codes [rows, K], scales [K/128][rows] (block-major, so
//           that a tile's scales of one K block are contiguous)
//   GEMM    C[rows, N] = sum over K blocks kb of sA[row, kb] * sB[n/128, kb] *
//           (Aq[rows, kb] . Bq[N, kb]^T): the products of a K block are summed by
//           the MFMA into a fresh fp32 accumulator and promoted into the running
//           sum with the two scales (fp32 FMA), block by block
// GEMM-1 applies SwiGLU and stores the intermediate as bf16; it is quantised by
// the same kernel before GEMM-2.
//
// GEMM tile: 128 rows x 128 weight rows (DUAL: 64 gate + the matching 64 up
// rows), K step 128 bytes = one scale block, 256 threads = 4 wavefronts as 2 (M)
// x 2 (N), each 2 x 2 MFMA tiles.  Operands go global -> LDS by DMA (two stages),
// rows of 128 bytes with the piece index XOR-ed by (row/2)&7.  Inside a
// K step, MFMA sub-step s of lane half h takes bytes (2s+h)*32 .. +32 of the row
// for BOTH operands, so the pairing of A and B elements is right whatever order
// the instruction walks K in.
#include "moe_internal.h"

namespace moe {

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kQBlock = 128;     // columns per activation scale, and K bytes per GEMM step
constexpr int kTileRec = 4;      // tile record: expert, first row, end row, (unused)
constexpr int FBM = 128, FBN = 128;

__device__ __forceinline__ uint16_t f32_to_bf16_bits_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ int swz(int row, int piece) {
  return row * 8 + (piece ^ ((row >> 1) & 7));
}

// ------------------------------------------------------------------ quant
// x bf16 [rows, K] -> codes [rows, K], scales_t [K/128][rows_capacity].  One
// wavefront per row walks it in chunks of 512 columns: a lane owns 8
// neighbouring columns (one 16-byte load), 16 lanes share a block of 128.  Two
// chunks are in flight per trip.
__device__ __forceinline__ void quant_piece(const uint4 v, uint2& out, float& scale) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float f[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
  for (int s = 1; s < 16; s <<= 1) amax = fmaxf(amax, __shfl_xor(amax, s));
  scale = amax > 0.f ? amax / 448.0f : 1.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) f[i] = fminf(fmaxf(f[i] / scale, -448.0f), 448.0f);
  int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);      // round to nearest even
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
  int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
  out = make_uint2((uint32_t)lo, (uint32_t)hi);
}

__global__ __launch_bounds__(256) void fp8act_quant_kernel(const uint16_t* __restrict__ x,
                                                          const int32_t* __restrict__ offsets,
                                                          int n_experts, int K, int rows_capacity,
                                                          uint8_t* __restrict__ codes,
                                                          float* __restrict__ scales_t) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int rows = offsets ? offsets[n_experts] : rows_capacity;     // no offsets: every row
  rows = rows < rows_capacity ? rows : rows_capacity;
  if (row >= rows) return;
  const uint4* xr = reinterpret_cast<const uint4*>(x + size_t(row) * K);     // 8 columns per piece
  uint2* cr = reinterpret_cast<uint2*>(codes + size_t(row) * K);
  const int pieces = K / 8;                       // a multiple of 16
  const int g = lane >> 4, sub = lane & 15;
  for (int p0 = 0; p0 < pieces; p0 += 128) {      // the loop bounds are the same in every lane
    const int pa = p0 + lane, pb = p0 + 64 + lane;
    const bool ina = pa < pieces, inb = pb < pieces;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const uint4 va = ina ? xr[pa] : zero, vb = inb ? xr[pb] : zero;
    uint2 ca, cb;
    float sa, sb;
    quant_piece(va, ca, sa);
    quant_piece(vb, cb, sb);
    if (ina) {
      cr[pa] = ca;
      if (sub == 0) scales_t[size_t(p0 / 16 + g) * rows_capacity + row] = sa;
    }
    if (inb) {
      cr[pb] = cb;
      if (sub == 0) scales_t[size_t(p0 / 16 + 4 + g) * rows_capacity + row] = sb;
    }
  }
}

// ------------------------------------------------------------- tile table
// tiles[0] = number of M tiles, then (expert, first row, end row, 0) per tile of
// up to FBM rows.  One thread per expert; experts have few tiles.
__global__ __launch_bounds__(512) void fp8act_tiles_kernel(const int32_t* __restrict__ offsets,
                                                          int n_experts, int rows_capacity,
                                                          int32_t* __restrict__ tiles, int max_tiles) {
  __shared__ int32_t start[513];
  const int e = threadIdx.x;
  int lo = 0, hi = 0;
  if (e < n_experts) {
    lo = min(max(offsets[e], 0), rows_capacity);
    hi = min(max(offsets[e + 1], lo), rows_capacity);
  }
  const int nt = (hi - lo + FBM - 1) / FBM;
  if (e < 513) start[e] = nt;
  __syncthreads();
  if (threadIdx.x == 0) {                      // n_experts <= 512: a serial scan is a few hundred adds
    int run = 0;
    for (int i = 0; i < n_experts; ++i) { const int c = start[i]; start[i] = run; run += c; }
    tiles[0] = run < max_tiles ? run : max_tiles;
  }
  __syncthreads();
  if (e >= n_experts) return;
  int t = start[e];
  for (int r = lo; r < hi && t < max_tiles; r += FBM, ++t) {
    tiles[1 + kTileRec * t] = e;
    tiles[2 + kTileRec * t] = r;
    tiles[3 + kTileRec * t] = r + FBM < hi ? r + FBM : hi;
    tiles[4 + kTileRec * t] = 0;
  }
}

// ------------------------------------------------------------------- GEMM
// A codes [rows, K], sA_t [K/128][rows_capacity]; B codes [n_experts][N][K] (DUAL:
// B0 = gate, B1 = up), S [n_experts][N/128][K/128]; C bf16 [rows, N].
// Operands go global -> LDS directly (`global_load_lds_dwordx4`) into two
// stages: the loads of step k+1 are issued right after the barrier of step k and
// waited for before the barrier of step k+1; two workgroups share a CU and fill
// each other's waits.  LDS slot s of a stage holds (row s/8, piece (s%8) ^
// (row/2)&7); the lane that owns the slot fetches that piece.
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <bool DUAL>
__device__ __forceinline__ void fp8act_gemm_body(
    const uint8_t* __restrict__ A, const float* __restrict__ sA_t, int rows_capacity,
    const uint8_t* __restrict__ B0, const uint8_t* __restrict__ B1, const float* __restrict__ S0,
    const float* __restrict__ S1, uint16_t* __restrict__ C, int N, int K,
    const int32_t* __restrict__ tiles, uint4* smem) {
  uint4* const As = smem;                         // [2][FBM * 8]
  uint4* const Bs = smem + 2 * FBM * 8;           // [2][FBN * 8]
  float* const Ss = reinterpret_cast<float*>(smem + 2 * FBM * 8 + 2 * FBN * 8);   // [2][FBM]
  constexpr int CN = DUAL ? 64 : 128;             // output columns per workgroup
  const int n_ntiles = N / CN;
  const int mtile = blockIdx.x / n_ntiles, ntile = blockIdx.x % n_ntiles;
  if (mtile >= tiles[0]) return;
  const int e = tiles[1 + kTileRec * mtile], row0 = tiles[2 + kTileRec * mtile],
            row1 = tiles[3 + kTileRec * mtile];
  const int n0 = ntile * CN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int h = lane >> 5, l31 = lane & 31;
  const int nkb = K / kQBlock, nnb = N / 128;

  // this thread's slots: tid + 256 i (i < 4) of the A stage and of the B stage: rows
  // (tid >> 3) + 32 i, and (row / 2) & 7 does not depend on i
  const int lrow = tid >> 3;
  const int gpiece = (tid & 7) ^ ((lrow >> 1) & 7);
  const uint8_t* ap[4];
  const uint8_t* bp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int r = row0 + lrow + 32 * i;
    r = r < row1 ? r : row1 - 1;
    ap[i] = A + size_t(r) * K + gpiece * 16;
    const int br = lrow + 32 * i;                 // row of the B tile: DUAL 0..63 gate, 64..127 up
    const uint8_t* base = (DUAL && br >= 64) ? B1 : B0;
    const int n = n0 + ((DUAL && br >= 64) ? br - 64 : br);
    bp[i] = base + (size_t(e) * N + n) * K + gpiece * 16;
  }
  const int srow = row0 + (tid & 127) < row1 ? row0 + (tid & 127) : row1 - 1;
  const float* s0p = S0 + (size_t(e) * nnb + n0 / 128) * nkb;
  const float* s1p = DUAL ? S1 + (size_t(e) * nnb + n0 / 128) * nkb : nullptr;

  float rs;                                       // this thread's row scale of the step in flight
  auto issue = [&](int kb) {
    const int st = kb & 1;
    rs = sA_t[size_t(kb) * rows_capacity + srow];          // first: the oldest load of the group
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(ap[i] + size_t(kb) * kQBlock),
                                       (lptr_t)(As + st * FBM * 8 + (i * 4 + wave) * 64), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(bp[i] + size_t(kb) * kQBlock),
                                       (lptr_t)(Bs + st * FBN * 8 + (i * 4 + wave) * 64), 16, 0, 0);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  // B rows of this wavefront's two 32-column blocks
  const int brow0 = DUAL ? wn * 32 : wn * 64;             // DUAL: gate block; else first block
  const int brow1 = DUAL ? 64 + wn * 32 : wn * 64 + 32;   // DUAL: the matching up block

  issue(0);
  for (int kb = 0; kb < nkb; ++kb) {
    const int buf = kb & 1;
    // step kb has landed (nothing younger is in flight); park its row scales
    __builtin_amdgcn_s_waitcnt(0x0f70);                   // vmcnt(0)
    if (tid < FBM) Ss[buf * FBM + tid] = rs;
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // every wavefront is done with step kb-1: refill its stage
    if (kb + 1 < nkb) issue(kb + 1);
    const uint4* Ab = As + buf * FBM * 8;
    const uint4* Bb = Bs + buf * FBN * 8;
    f32x16 part[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int p = (2 * s + h) * 2;                  // first of the lane's two 16-byte pieces
      i32x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int r = wm * 64 + i * 32 + l31;
        const uint4 lo = Ab[swz(r, p)], hi = Ab[swz(r, p + 1)];
        fa[i] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int r = (j == 0 ? brow0 : brow1) + l31;
        const uint4 lo = Bb[swz(r, p)], hi = Bb[swz(r, p + 1)];
        fb[j] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          f32x16 c;
          if (s == 0) {
#pragma unroll
            for (int q = 0; q < 16; ++q) c[q] = 0.f;
          } else {
            c = part[i][j];
          }
          part[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], c, 0, 0, 0,
                                                                      0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
    }
    // promote the block's sums: acc += part * sA[row] * sB
    const float sb0 = s0p[kb];
    const float sb1 = DUAL ? s1p[kb] : sb0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float sa[16];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 v = *reinterpret_cast<const float4*>(Ss + buf * FBM + wm * 64 + i * 32 + q4 * 8 + h * 4);
        sa[q4 * 4 + 0] = v.x; sa[q4 * 4 + 1] = v.y; sa[q4 * 4 + 2] = v.z; sa[q4 * 4 + 3] = v.w;
      }
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        acc[i][0][q] = fmaf(part[i][0][q], sa[q] * sb0, acc[i][0][q]);
        acc[i][1][q] = fmaf(part[i][1][q], sa[q] * sb1, acc[i][1][q]);
      }
    }
  }

  // D layout: lane l, register q -> row (q/4)*8 + (l/32)*4 + q%4, col l%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int row = row0 + wm * 64 + i * 32 + (q >> 2) * 8 + h * 4 + (q & 3);
      if (row >= row1) continue;
      if (DUAL) {
        const float g = acc[i][0][q], u = acc[i][1][q];
        const float v = g / (1.0f + __expf(-g)) * u;
        C[size_t(row) * N + n0 + wn * 32 + l31] = f32_to_bf16_bits_rne(v);
      } else {
        C[size_t(row) * N + n0 + wn * 64 + l31] = f32_to_bf16_bits_rne(acc[i][0][q]);
        C[size_t(row) * N + n0 + wn * 64 + 32 + l31] = f32_to_bf16_bits_rne(acc[i][1][q]);
      }
    }
}

template <bool DUAL>
__global__ __launch_bounds__(256, 2) void fp8act_gemm_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ sA_t, int rows_capacity,
    const uint8_t* __restrict__ B0, const uint8_t* __restrict__ B1, const float* __restrict__ S0,
    const float* __restrict__ S1, uint16_t* __restrict__ C, int N, int K,
    const int32_t* __restrict__ tiles) {
  extern __shared__ uint4 fsmem[];
  // handed on as a generic pointer: with the LDS array named in the loop the
  // compiler drains every DMA in flight before each LDS read
  fp8act_gemm_body<DUAL>(A, sA_t, rows_capacity, B0, B1, S0, S1, C, N, K, tiles, fsmem);
}

}  // namespace

// workspace: tiles | x codes | x scales | hmid bf16 | hmid codes | hmid scales
struct Fp8ActWs {
  int32_t* tiles;
  uint8_t* xq;
  float* xs_t;
  uint16_t* hmid;
  uint8_t* hq;
  float* hs_t;
  int max_tiles;
  size_t bytes;
};

static Fp8ActWs carve_fp8act(void* ws, int rows_capacity, int n_experts, int H, int I) {
  Fp8ActWs f;
  char* p = static_cast<char*>(ws);
  size_t off = 0;
  f.max_tiles = rows_capacity / FBM + n_experts + 1;
  f.tiles = reinterpret_cast<int32_t*>(p + off); off += align_up(size_t(1 + kTileRec * f.max_tiles) * 4);
  f.xq = reinterpret_cast<uint8_t*>(p + off);    off += align_up(size_t(rows_capacity) * H);
  f.xs_t = reinterpret_cast<float*>(p + off);    off += align_up(size_t(H / kQBlock) * rows_capacity * 4);
  f.hmid = reinterpret_cast<uint16_t*>(p + off); off += align_up(size_t(rows_capacity) * I * 2);
  f.hq = reinterpret_cast<uint8_t*>(p + off);    off += align_up(size_t(rows_capacity) * I);
  f.hs_t = reinterpret_cast<float*>(p + off);    off += align_up(size_t(I / kQBlock) * rows_capacity * 4);
  f.bytes = off;
  return f;
}

static bool fp8act_ok(const moe_config* c) {
  return c && c->act_dtype == MOE_BF16 && c->weight_dtype == MOE_FP8_E4M3_B128 && c->hidden > 0 &&
         c->inter_local > 0 && c->hidden % 128 == 0 && c->inter_local % 128 == 0;
}

}  // namespace moe

using namespace moe;

extern "C" {

size_t moe_fp8act_workspace_bytes(const moe_config* cfg, int32_t n_experts_here,
                                  int32_t rows_capacity) {
  if (!fp8act_ok(cfg) || n_experts_here < 1 || n_experts_here > 512 || rows_capacity < 0) return 0;
  return carve_fp8act(nullptr, rows_capacity, n_experts_here, cfg->hidden, cfg->inter_local).bytes;
}

// shared by the two FFN entry points: xs_q / xs_scales given -> no input quantisation
static moe_status fp8act_run(const moe_config* cfg, int32_t n_experts_here, const void* xs,
                             const void* xs_q, const float* xs_scales, const int32_t* offsets,
                             int32_t rows_capacity, const void* w_gate, const void* w_up,
                             const void* w_down, const float* s_gate, const float* s_up,
                             const float* s_down, void* ys, void* ws, size_t ws_bytes, void* stream) {
  if (!cfg) return MOE_ERR_INVALID_ARG;
  if (!fp8act_ok(cfg)) return MOE_ERR_UNSUPPORTED;
  if (n_experts_here < 1 || n_experts_here > 512 || rows_capacity < 0) return MOE_ERR_INVALID_ARG;
  if (rows_capacity == 0) return MOE_OK;
  const void* ptrs[] = {xs ? xs : xs_q, xs ? xs : static_cast<const void*>(xs_scales), offsets, w_gate,
                        w_up, w_down, s_gate, s_up, s_down, ys, ws};
  for (const void* p : ptrs)
    if (!p || (reinterpret_cast<uintptr_t>(p) & 15)) return MOE_ERR_INVALID_ARG;
  const int H = cfg->hidden, I = cfg->inter_local;
  Fp8ActWs f = carve_fp8act(ws, rows_capacity, n_experts_here, H, I);
  if (ws_bytes < f.bytes) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  constexpr int lds = (2 * FBM * 8 + 2 * FBN * 8) * 16 + 2 * FBM * 4;
  auto k1 = fp8act_gemm_kernel<true>;
  auto k2 = fp8act_gemm_kernel<false>;
  static uint64_t opted1 = 0, opted2 = 0;
  lds_opt_in(reinterpret_cast<const void*>(k1), lds, opted1);
  lds_opt_in(reinterpret_cast<const void*>(k2), lds, opted2);
  const dim3 qgrid((rows_capacity + 3) / 4);
  MOE_LAUNCH(MOE_K_FFN_TILES, fp8act_tiles_kernel, dim3(1), dim3(512), 0, s, offsets, n_experts_here,
             rows_capacity, f.tiles, f.max_tiles);
  const uint8_t* aq = static_cast<const uint8_t*>(xs_q);
  const float* as = xs_scales;
  if (xs) {
    MOE_LAUNCH(MOE_K_FFN_TILES, fp8act_quant_kernel, qgrid, dim3(256), 0, s,
               static_cast<const uint16_t*>(xs), offsets, n_experts_here, H, rows_capacity, f.xq, f.xs_t);
    aq = f.xq;
    as = f.xs_t;
  }
  MOE_LAUNCH(MOE_K_FFN_GEMM1, k1, dim3(size_t(f.max_tiles) * (I / 64)), dim3(256), lds, s, aq, as,
             rows_capacity, static_cast<const uint8_t*>(w_gate), static_cast<const uint8_t*>(w_up),
             s_gate, s_up, f.hmid, I, H, f.tiles);
  MOE_LAUNCH(MOE_K_FFN_TILES, fp8act_quant_kernel, qgrid, dim3(256), 0, s, f.hmid, offsets,
             n_experts_here, I, rows_capacity, f.hq, f.hs_t);
  MOE_LAUNCH(MOE_K_FFN_GEMM2, k2, dim3(size_t(f.max_tiles) * (H / 128)), dim3(256), lds, s, f.hq, f.hs_t,
             rows_capacity, static_cast<const uint8_t*>(w_down), static_cast<const uint8_t*>(nullptr),
             s_down, static_cast<const float*>(nullptr), static_cast<uint16_t*>(ys), H, I, f.tiles);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

moe_status moe_quant_act(const moe_config* cfg, int32_t rows, const void* x, void* codes,
                         float* scales, void* stream) {
  if (!cfg) return MOE_ERR_INVALID_ARG;
  if (cfg->act_dtype != MOE_BF16 || cfg->hidden <= 0 || cfg->hidden % 128) return MOE_ERR_UNSUPPORTED;
  if (rows < 0) return MOE_ERR_INVALID_ARG;
  if (rows == 0) return MOE_OK;
  const void* ptrs[] = {x, codes, scales};
  for (const void* p : ptrs)
    if (!p || (reinterpret_cast<uintptr_t>(p) & 15)) return MOE_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  MOE_LAUNCH(MOE_K_FFN_TILES, fp8act_quant_kernel, dim3((rows + 3) / 4), dim3(256), 0, s,
             static_cast<const uint16_t*>(x), static_cast<const int32_t*>(nullptr), 0, cfg->hidden, rows,
             static_cast<uint8_t*>(codes), scales);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_DEVICE;
}

moe_status moe_expert_ffn_fp8act(const moe_config* cfg, int32_t n_experts_here, const void* xs,
                                 const int32_t* offsets, int32_t rows_capacity, const void* w_gate,
                                 const void* w_up, const void* w_down, const float* s_gate,
                                 const float* s_up, const float* s_down, void* ys, void* ws,
                                 size_t ws_bytes, void* stream) {
  if (!xs) return MOE_ERR_INVALID_ARG;
  return fp8act_run(cfg, n_experts_here, xs, nullptr, nullptr, offsets, rows_capacity, w_gate, w_up,
                    w_down, s_gate, s_up, s_down, ys, ws, ws_bytes, stream);
}

moe_status moe_expert_ffn_fp8q(const moe_config* cfg, int32_t n_experts_here, const void* xs_q,
                               const float* xs_scales, const int32_t* offsets,
                               int32_t rows_capacity, const void* w_gate, const void* w_up,
                               const void* w_down, const float* s_gate, const float* s_up,
                               const float* s_down, void* ys, void* ws, size_t ws_bytes,
                               void* stream) {
  if (!xs_q || !xs_scales) return MOE_ERR_INVALID_ARG;
  return fp8act_run(cfg, n_experts_here, nullptr, xs_q, xs_scales, offsets, rows_capacity, w_gate,
                    w_up, w_down, s_gate, s_up, s_down, ys, ws, ws_bytes, stream);
}

}  // extern "C"
