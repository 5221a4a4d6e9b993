/*
 * libmoe -- one GPU's share of a Mixture-of-Experts layer on MI355X (gfx950).
 *
 * The share follows the paper's statement of the MoE block under hybrid
 * TP-EP parallelism: tokens are routed to their top-k activated experts
 * (Sec. III-B-2 "A2A"; the `route` step of Alg. 2), sent to the device that
 * hosts the expert ("Dispatch", Sec. II), pushed through that expert's MLP,
 * whose weights are an intra-node TP slice (Sec. II "TP", Sec. III-C), and
 * returned along the original route weighted by the top-k weights
 * ("Combine", Sec. II; the accumulation step of Alg. 1), giving the
 * partial sum that the intra-node all-reduce completes (Sec. III-B-2 "AR").
 * The exchanges themselves (A2A, AR) are outside this library: it builds the
 * buffer the A2A would carry and the tensor the AR would reduce.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers unless marked "host".  The caller
 *    owns every buffer, including the workspace; the library never allocates,
 *    frees or synchronises.  All work is enqueued on `stream` (a hipStream_t
 *    passed as void*; NULL is the default stream).
 *  - Tensors are dense and row-major.  Device pointers must be 16-byte aligned.
 *  - Outputs are overwritten.  Rows / entries beyond the valid count of a
 *    capacity-sized output are unspecified.
 *  - Arguments are validated on the host before anything is launched; on any
 *    error nothing is enqueued and outputs are untouched.  T == 0 returns
 *    MOE_OK and launches nothing.
 *  - The return value is the only error channel; nothing is thrown.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = 1, /* NULL / misaligned pointer, negative size, inconsistent config */
  MOE_ERR_UNSUPPORTED = 2, /* dtype combination or shape the kernels do not cover          */
  MOE_ERR_WORKSPACE = 3,   /* ws_bytes smaller than moe_workspace_bytes()                   */
  MOE_ERR_DEVICE = 4       /* a launch failed (hipGetLastError after the launch)            */
} moe_status;

typedef enum {
  MOE_F32 = 0,
  MOE_BF16 = 1,
  MOE_FP8_E4M3_B128 = 2 /* OCP e4m3 codes + one fp32 scale per 128x128 block (weights only) */
} moe_dtype;

typedef enum { MOE_SCORE_SOFTMAX = 0, MOE_SCORE_SIGMOID = 1 } moe_score_fn;

/*
 * Layer description.  Symbols follow the paper where it has them: h = hidden,
 * k = experts activated per token, d_EP / d_TP enter through the expert range
 * and the intermediate slice.
 */
typedef struct {
  int32_t hidden;        /* H, multiple of 8                                              */
  int32_t n_experts;     /* E, global routed experts, E <= 512                            */
  int32_t top_k;         /* k, 1 <= k <= 32, k <= E                                       */
  int32_t score_fn;      /* moe_score_fn                                                  */
  int32_t renormalize;   /* 1: weights of the k picked experts sum to routed_scale        */
  float routed_scale;    /* multiplies the weights (1.0, or 2.5 for the DeepSeek shape)   */
  int32_t n_groups;      /* G; 1 = no group limit; E % G == 0; G <= 64                    */
  int32_t topk_groups;   /* groups kept, 1 <= topk_groups <= G                            */
  int32_t group_score_n; /* group score = sum of this many largest keys of the group     */
  int32_t expert_lo;     /* this GPU hosts global experts [expert_lo, expert_hi)          */
  int32_t expert_hi;
  int32_t inter_local;   /* I_loc = I / d_TP, multiple of 8 (128 for fp8 weights)         */
  int32_t act_dtype;     /* MOE_F32 or MOE_BF16: x, xs, ys, gate weights                  */
  int32_t weight_dtype;  /* MOE_F32 (with F32 act), MOE_BF16 or MOE_FP8_E4M3_B128         */
} moe_config;

/* Upper bound, in bytes, of the workspace any entry point needs for T tokens
 * (0 if the config is invalid).  Host-only, launches nothing. */
size_t moe_workspace_bytes(const moe_config* cfg, int32_t T);

/* Static description of a status code (host pointer, never NULL). */
const char* moe_status_string(moe_status s);

/*
 * Gate scoring and top-k routing (Sec. III-B-2: every token goes to its top-k
 * activated experts; Alg. 2: the expert map is computed from local states).
 *   logit z[t,e]  = sum_h x[t,h] * gate_w[e,h]  (+ logit_bias[e])
 *   score         = softmax_e(z)  or  sigmoid(z)
 *   selection key = z (softmax)   or  sigmoid(z) + select_bias[e]
 *   group limit   = keep the topk_groups groups with the largest sum of their
 *                   group_score_n largest keys; other experts are ineligible
 *   topk_ids[t,:] = the k eligible experts with the largest keys, in descending
 *                   key order; ties go to the lowest expert (group) index
 *   topk_w[t,j]   = score (without select_bias), divided by the sum over the
 *                   k picked when renormalize, times routed_scale
 * The ids are those of exact arithmetic on the stored inputs: keys are first
 * computed fast (bf16 MFMA, fp32 accumulation in short chains) and every token
 * whose decisive key gaps are within the error bound of that computation is
 * re-scored in fp64.  After the call the first int32 of `ws` holds the number
 * of tokens that were re-scored.
 *   x          [T,H]  act dtype            gate_w [E,H] act dtype
 *   logit_bias [E] fp32 or NULL            select_bias [E] fp32 or NULL
 *   logits_in  [T,E] fp32 or NULL: when given the dot products are skipped and
 *              these are the logits (x and gate_w may then be NULL)
 *   topk_ids   out [T,k] int32 global expert ids     topk_w out [T,k] fp32
 * T * E must stay below 2^31 (MOE_ERR_UNSUPPORTED otherwise).
 */
moe_status moe_route(const moe_config* cfg, int32_t T, const void* x, const void* gate_w,
                     const float* logit_bias, const float* select_bias,
                     const float* logits_in, int32_t* topk_ids, float* topk_w, void* ws,
                     size_t ws_bytes, void* stream);

/*
 * Dispatch (Sec. II "EP": each token is sent to the device hosting its
 * expert; Alg. 2: per-destination lists built from the expert map).  Builds
 * the expert-contiguous send buffer for the assignments whose expert is in
 * [expert_lo, expert_hi).  Flat assignment index a = t*k + j.
 *   counts  out [E_loc]     assignments per local expert
 *   offsets out [E_loc+1]   exclusive scan of counts; offsets[E_loc] = A_loc
 *   perm    out [T*k]       first A_loc valid: position -> a; experts ascending,
 *                           inside an expert ascending a (stable, atomic-free)
 *   inv     out [T*k]       a -> position, or -1 when the expert is not local
 *   xs      out [T*k, H]    act dtype; first A_loc rows valid: xs[pos] = x[perm[pos]/k]
 * counts/offsets stay on the device; later calls read them there.
 * T * k must not exceed 2^30 (MOE_ERR_UNSUPPORTED otherwise).
 */
moe_status moe_dispatch(const moe_config* cfg, int32_t T, const void* x,
                        const int32_t* topk_ids, int32_t* counts, int32_t* offsets,
                        int32_t* perm, int32_t* inv, void* xs, void* ws, size_t ws_bytes,
                        void* stream);

/*
 * moe_dispatch for callers that cannot allocate or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same arguments, outputs and errors as moe_dispatch, minus the
 * workspace: the index scratch (one int32 per local expert and sub-chunk of 64
 * assignments, E_loc * ceil(T*k / 64) * 4 bytes) lives in a fixed device array
 * inside the library, moe_dispatch_noalloc_max_bytes() = 4 MiB per GPU, held
 * until the process ends.  A call whose scratch would exceed that returns
 * MOE_ERR_WORKSPACE and enqueues nothing (the largest workload here, 65 536
 * tokens x top-8 over 128 local experts, needs exactly 4 MiB).  The call
 * allocates and frees nothing and synchronises nothing; the array's device
 * address is looked up once per device on the first call there.  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and must be serialised by the caller; calls in
 * stream order are safe, every call overwrites what it reads.
 */
size_t moe_dispatch_noalloc_max_bytes(void);
moe_status moe_dispatch_noalloc(const moe_config* cfg, int32_t T, const void* x,
                                const int32_t* topk_ids, int32_t* counts, int32_t* offsets,
                                int32_t* perm, int32_t* inv, void* xs, void* stream);

/*
 * Dispatch for the fused AG-Dispatch schedule (Alg. 2; Sec. III-C-2: hidden
 * states are replicated inside the MoE TP group, so they can be sharded there).
 * TP rank `tp_rank` of `tp_size` computes the expert map as moe_dispatch does
 * and builds the send buffer from its own hidden-column shard X_{r_TP} only;
 * the all-gather on the receiving node completes the rows.  counts / offsets /
 * perm / inv are those of moe_dispatch;
 *   xs_shard out [T*k, H/tp_size] act dtype:
 *     xs_shard[pos, c] = x[perm[pos]/k, tp_rank*H/tp_size + c]
 * H must be a multiple of tp_size and H/tp_size a multiple of 8.  tp_rank 0 of
 * 1 is moe_dispatch.
 */
moe_status moe_dispatch_shard(const moe_config* cfg, int32_t T, const void* x,
                              const int32_t* topk_ids, int32_t tp_rank, int32_t tp_size,
                              int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                              void* xs_shard, void* ws, size_t ws_bytes, void* stream);

/*
 * Grouped expert MLP (Sec. II: each expert is an independent MLP; under TP the
 * projections are sliced and the partial results are summed afterwards).  For
 * expert e in [0, n_experts_here) and every row r in [offsets[e], offsets[e+1]):
 *   ys[r,:] = w_down[e] * ( silu(w_gate[e] * xs[r,:]) .* (w_up[e] * xs[r,:]) )
 * with fp32 accumulation; the intermediate is held in the act dtype.
 *   xs      [rows_capacity, H] act dtype        offsets [n_experts_here+1] int32 (device)
 *   w_gate, w_up [n, I_loc, H]   w_down [n, H, I_loc]   weight dtype
 *   s_gate, s_up [n, I_loc/128, ceil(H/128)]  s_down [n, ceil(H/128), I_loc/128]
 *           fp32 block scales, required for MOE_FP8_E4M3_B128, else NULL
 *           (the weight is code * scale; with more than twelve rows per expert to
 *           expect, rows_capacity / n_experts_here > 12, that product is rounded
 *           to bf16 before the matrix instruction, otherwise the scale multiplies
 *           the fp32 partial sum of its 128-deep block: both within the stated
 *           fp8 tolerance of the exact product)
 *   ys      out [rows_capacity, H] act dtype
 * rows_capacity bounds offsets[n]; rows beyond offsets[n] are not touched.
 * The shared expert is the same call with n_experts_here = 1, offsets = {0,T},
 * xs = x.
 */
moe_status moe_expert_ffn(const moe_config* cfg, int32_t n_experts_here, const void* xs,
                          const int32_t* offsets, int32_t rows_capacity, const void* w_gate,
                          const void* w_up, const void* w_down, const float* s_gate,
                          const float* s_up, const float* s_down, void* ys, void* ws,
                          size_t ws_bytes, void* stream);

/*
 * Combine (Sec. II: results return along the original route; Alg. 1: they are
 * weighted by the top-k weights) into the partial sum the intra-node
 * all-reduce would finish (Sec. III-B-2 "AR"):
 *   out[t,:] = sum_{j : inv[t*k+j] >= 0} topk_w[t,j] * ys[inv[t*k+j],:]  (+ shared_ys[t,:])
 * summed over ascending j in fp32.
 *   ys [>= A_loc, H] act dtype   inv [T*k]   topk_w [T,k]
 *   shared_ys [T,H] act dtype or NULL       out [T,H] fp32, overwritten
 */
moe_status moe_combine(const moe_config* cfg, int32_t T, const void* ys, const int32_t* inv,
                       const float* topk_w, const void* shared_ys, float* out, void* stream);

/*
 * One stage of the fused RS-Combine schedule (Alg. 1): the hidden dimension is
 * split into tp_size blocks; stage i hands this rank S_i, the reduce-scattered
 * expert outputs that one source node returned, restricted to the rank's block,
 * and the stage result, scaled by the top-k weights, is added to the running
 * block (the accumulation step of Alg. 1).
 *   ys_block  [>= rows, H/tp_size] act dtype (rows addressed through inv)
 *   inv [T*k], topk_w [T,k]: as in moe_combine, for the assignments of this stage
 *   out_block [T, H/tp_size] fp32:
 *     s[t,c] = sum_{j : inv[t*k+j] >= 0} topk_w[t,j] * ys_block[inv[t*k+j], c]
 *              (ascending j, fp32)
 *     accumulate == 0: out_block = s (first stage; out_block need not be
 *     initialised); accumulate == 1: out_block = out_block + s
 * tp_size 1 with accumulate 0 is moe_combine without a shared expert.
 */
moe_status moe_combine_stage(const moe_config* cfg, int32_t T, const void* ys_block,
                             const int32_t* inv, const float* topk_w, int32_t tp_size,
                             int32_t accumulate, float* out_block, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the layer; Sec. III-A calls for
 * profiling data as the analyzer's observations, and the roofline figures need
 * each kernel's duration on the stream it runs on).  When enabled, every
 * kernel launch of the four entry points is bracketed by a hipEvent pair taken
 * from a pool created by moe_profile_enable(); launches beyond the pool are
 * not recorded.  Events are host objects; no device memory is involved.
 */
typedef enum {
  MOE_K_GATE_NORMS = 0,   /* gate-row norms + counter clear                 */
  MOE_K_GATE_GEMM = 1,    /* gate logits                                    */
  MOE_K_SELECT = 2,       /* wavefront top-k                                */
  MOE_K_RESCORE = 3,      /* fp64 re-scoring of doubtful tokens             */
  MOE_K_DISPATCH_HIST = 4,
  MOE_K_DISPATCH_SCAN = 5,
  MOE_K_DISPATCH_SCATTER = 6,
  MOE_K_DISPATCH_GATHER = 7,
  MOE_K_FFN_TILES = 8,
  MOE_K_FFN_GEMM1 = 9,    /* gate|up projection + SwiGLU                    */
  MOE_K_FFN_GEMM2 = 10,   /* down projection                                */
  MOE_K_COMBINE = 11,
  MOE_K_COUNT = 12
} moe_kernel_id;

/* max_records > 0: (re)create a pool of that many event pairs and start
 * recording; 0: stop recording and destroy the pool.  Not thread-safe. */
moe_status moe_profile_enable(int32_t max_records);

/* Restrict recording to the kernels whose bit (1 << moe_kernel_id) is set in
 * `mask` (default: all).  Recording one kernel costs two event records per
 * launch, so a benchmark can time its dominant kernel inside the timed region
 * without slowing the region down by the other launches' events. */
moe_status moe_profile_filter(uint32_t mask);

/* Synchronises on the recorded events, then adds up, per moe_kernel_id, the
 * elapsed milliseconds and the number of recorded launches (host arrays of
 * MOE_K_COUNT entries), and clears the records (recording stays enabled). */
moe_status moe_profile_read(double* total_ms, int32_t* launches);

/* Calibration for the MFMA roofline (benchmark helper, not part of the layer):
 * launches `workgroups` workgroups of eight wavefronts that do nothing but
 * `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 on register
 * operands, times the launch with an event pair on `stream`, waits for it, and
 * returns the rate in TFLOP/s: what the matrix units of this machine sustain at
 * the clock its power limit allows, with no loads, LDS traffic or barriers.
 * Allocates no device memory; synchronises on its own events. */
moe_status moe_probe_mfma_rate(int32_t workgroups, int32_t iters, void* stream, double* tflops);

/* ---- expert FFN with 8-bit activations (an extension beyond the paper: both
 * GEMM operands e4m3, fp8 matrix instructions) --------------------------------
 * Same arguments and semantics as moe_expert_ffn for cfg->act_dtype = MOE_BF16,
 * cfg->weight_dtype = MOE_FP8_E4M3_B128, hidden and inter_local multiples of
 * 128 (otherwise MOE_ERR_UNSUPPORTED), except for the arithmetic: every input
 * row is quantised on the fly, one fp32 scale per row and block of 128 columns
 * (scale = max|x| / 448, 1 for an all-zero block; code = e4m3(x / scale),
 * round to nearest even after a clamp to +-448; fp32 operations), the products
 * of a 128-deep K block are summed in fp32 and multiplied by the row's and the
 * weight block's scales, and the SwiGLU intermediate, stored as bf16 in the
 * workspace, is quantised the same way before the down projection.  ys is bf16.
 * Workspace: moe_fp8act_workspace_bytes(cfg, n_experts_here, rows_capacity)
 * bytes (0 for an unsupported configuration). */
size_t moe_fp8act_workspace_bytes(const moe_config* cfg, int32_t n_experts_here,
                                  int32_t rows_capacity);

/* The same path with the quantisation taken out of the FFN call, so that a token
 * is quantised once and its 1-byte codes are what dispatch copies:
 *   moe_quant_act      x bf16 [rows, hidden] -> codes uint8 [rows, hidden] and
 *                      scales fp32 [hidden/128][rows] (block-major), by the rule above
 *   moe_dispatch_fp8q  moe_dispatch on quantised rows: xq [T, hidden] codes with
 *                      xq_scales [hidden/128][T] -> xs_q [T*k, hidden] codes with
 *                      xs_scales [hidden/128][T*k] (first A_loc positions valid);
 *                      counts / offsets / perm / inv exactly as moe_dispatch
 *   moe_expert_ffn_fp8q  moe_expert_ffn_fp8act on rows that are already quantised:
 *                      xs_q [rows_capacity, hidden], xs_scales [hidden/128][rows_capacity]
 * Quantising a row before or after it is copied gives the same codes, so the
 * results equal those of moe_dispatch + moe_expert_ffn_fp8act bit for bit. */
moe_status moe_quant_act(const moe_config* cfg, int32_t rows, const void* x, void* codes,
                         float* scales, void* stream);
moe_status moe_dispatch_fp8q(const moe_config* cfg, int32_t T, const void* xq,
                             const float* xq_scales, const int32_t* topk_ids, int32_t* counts,
                             int32_t* offsets, int32_t* perm, int32_t* inv, void* xs_q,
                             float* xs_scales, void* ws, size_t ws_bytes, void* stream);
moe_status moe_expert_ffn_fp8q(const moe_config* cfg, int32_t n_experts_here, const void* xs_q,
                               const float* xs_scales, const int32_t* offsets,
                               int32_t rows_capacity, const void* w_gate, const void* w_up,
                               const void* w_down, const float* s_gate, const float* s_up,
                               const float* s_down, void* ys, void* ws, size_t ws_bytes,
                               void* stream);
moe_status moe_expert_ffn_fp8act(const moe_config* cfg, int32_t n_experts_here, const void* xs,
                                 const int32_t* offsets, int32_t rows_capacity, const void* w_gate,
                                 const void* w_up, const void* w_down, const float* s_gate,
                                 const float* s_up, const float* s_down, void* ys, void* ws,
                                 size_t ws_bytes, void* stream);

/* Static name of a kernel id (host pointer). */
const char* moe_kernel_name(int32_t id);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
