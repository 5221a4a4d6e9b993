/* Analytic parallel-strategy selector: the latency model of Sec. III-A and the
 * enumeration of Sec. III-B-2, evaluated on the host.  Pure arithmetic on the
 * arguments: no device, no allocation, no global state.  Every function is
 * thread-safe.
 *
 * The paper states its collective costs up to a proportionality constant; here
 * the constant is 1 / bandwidth, sizes are bytes and times are seconds:
 *   RS(size, d) = AG(size, d) = size / d / bw                  (Sec. III-A-2, first equation)
 *   AR(size, d) = RS(size / d, d) + AG(size / d, d)            (second equation, as printed)
 *   A2A(size, d) = size / d * (d - 1) / bw                     (third equation)
 * A group of one device costs nothing.  A group that fits into one node
 * (its devices times the TP degree they are nested in <= n_proc) moves at
 * bw_intra, any other group at bw_inter.
 */
#ifndef MOE_STRATEGY_H_
#define MOE_STRATEGY_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The cluster: n_node nodes of n_proc devices (both powers of two). */
typedef struct {
  int32_t n_node;
  int32_t n_proc;
  double mem_bytes;     /* M: memory of one device, bytes */
  double bw_intra;      /* bytes/s a device moves in a collective inside its node */
  double bw_inter;      /* bytes/s a device moves in a collective across nodes */
  double bw_p2p;        /* bytes/s of a pipeline-stage point-to-point transfer */
  double compute_rate;  /* calibration constant of the compute term: units of
                           (weight bytes x tokens x hidden) one device retires per second */
} moe_cluster;

/* The model (Sec. III-A-4 "Constraints": weights = attention + MoE blocks of l layers). */
typedef struct {
  double psi_attn;      /* bytes of all attention-block weights */
  double psi_moe;       /* bytes of all MoE-block weights */
  int32_t layers;       /* l */
  int32_t hidden;       /* h */
  int32_t top_k;        /* k */
  double act_bytes;     /* bytes per element of hidden states and K/V cache */
} moe_model;

/* The request mix the indicators are evaluated on. */
typedef struct {
  int32_t batch;        /* b */
  int32_t len_in;       /* L_in: prompt length (prefill runs with s = L_in) */
  int32_t len_out;      /* L_out: generated tokens (decode runs with s = 1) */
  double arrival_rate;  /* lambda_a, tokens/s; 0 = no queueing term */
  double max_ttft;      /* seconds, 0 = no limit */
  double max_itl;       /* seconds, 0 = no limit */
} moe_request_mix;

/* One evaluated strategy. */
typedef struct {
  int32_t d_tp, d_ep, d_dp, d_pp;
  double tau_prf, lambda_prf;   /* per-layer compute / communication latency at s = L_in */
  double tau_dec, lambda_dec;   /* the same at s = 1 */
  double svc_prf, svc_dec;      /* service latency per token through l layers (+ pipeline P2P) */
  double wq;                    /* M/M/1 queueing delay; +inf when lambda_a >= mu */
  double ttft, itl, throughput; /* Sec. III-A-5 indicators (throughput in tokens/s) */
  double mem_bytes;             /* left side of the memory constraint */
  int32_t feasible;             /* memory constraint, queue stability and the limits all hold */
} moe_strategy;

/* Collective costs (see the head of this file).  degree < 1 or bw <= 0 gives NaN. */
double moe_cost_rs(double bytes, int32_t degree, double bw);
double moe_cost_ag(double bytes, int32_t degree, double bw);
double moe_cost_ar(double bytes, int32_t degree, double bw);
double moe_cost_a2a(double bytes, int32_t degree, double bw);

/* Communication of one decoder layer under pure EP in the MoE block and under
 * the hybrid TP-EP scheme (Sec. III-B-2, the two equations for lambda_EP and
 * lambda_mix), for hidden states of `tokens` = b*s tokens:
 *   lambda_EP  = AR(bsh, n_proc) + 2 A2A(bshk, n_node)
 *   lambda_mix = AR(bsh, n_proc) + AG(bshk / n_proc, n_proc) + 2 A2A(bshk / n_proc, n_node)
 * AR and AG run inside a node, A2A across nodes.  Returns NaN on invalid arguments. */
double moe_lambda_ep(const moe_cluster* c, const moe_model* m, double tokens);
double moe_lambda_mix(const moe_cluster* c, const moe_model* m, double tokens);

/* Evaluate one strategy: tau (computational latency), lambda (communication
 * latency, with the d_DP >= d_EP case split), service latency, queueing delay,
 * the memory constraint and TTFT / ITL / throughput (Sec. III-A-4, III-A-5).
 * Degrees must be powers of two with d_tp * d_ep = n_node * n_proc, d_dp * d_tp
 * <= n_node * n_proc and d_dp <= batch.  Returns 0 on success, 1 on invalid
 * arguments (then *out is untouched). */
int32_t moe_strategy_eval(const moe_cluster* c, const moe_model* m, const moe_request_mix* r,
                          int32_t d_tp, int32_t d_ep, int32_t d_dp, int32_t d_pp,
                          moe_strategy* out);

/* Enumerate every (d_tp, d_ep, d_dp) that moe_strategy_eval accepts for the given
 * d_pp, in ascending (d_tp, d_dp) order, and pick the feasible one with the
 * largest throughput (ties: smaller ITL, then smaller d_tp, then larger d_dp).
 * `all` (may be NULL) receives up to max_all evaluated strategies, *n_all (may be
 * NULL) their total number.  Returns 0 and fills *best; 1 on invalid arguments;
 * 2 when no strategy is feasible (*best untouched). */
int32_t moe_strategy_select(const moe_cluster* c, const moe_model* m, const moe_request_mix* r,
                            int32_t d_pp, moe_strategy* best, moe_strategy* all, int32_t max_all,
                            int32_t* n_all);

#ifdef __cplusplus
}
#endif

#endif /* MOE_STRATEGY_H_ */
