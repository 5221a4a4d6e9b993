// Analytic strategy selector (Sec. III-A latency model, Sec. III-B-2 enumeration).
// Host code only: closed-form arithmetic on the caller's numbers.
#include <math.h>

#include "moe_strategy.h"

namespace {

bool pow2(int v) { return v >= 1 && (v & (v - 1)) == 0; }

bool cluster_ok(const moe_cluster* c) {
  return c && pow2(c->n_node) && pow2(c->n_proc) && c->mem_bytes > 0 && c->bw_intra > 0 &&
         c->bw_inter > 0 && c->bw_p2p > 0 && c->compute_rate > 0;
}
bool model_ok(const moe_model* m) {
  return m && m->psi_attn >= 0 && m->psi_moe >= 0 && m->layers >= 1 && m->hidden >= 1 &&
         m->top_k >= 1 && m->act_bytes > 0;
}
bool mix_ok(const moe_request_mix* r) {
  return r && r->batch >= 1 && r->len_in >= 1 && r->len_out >= 0 && r->arrival_rate >= 0 &&
         r->max_ttft >= 0 && r->max_itl >= 0;
}

// bandwidth of a group of `devices` consecutive ranks
double group_bw(const moe_cluster& c, long devices) {
  return devices <= c.n_proc ? c.bw_intra : c.bw_inter;
}

struct Layer { double tau, lambda; };

// Computational and communication latency of one decoder layer for sequence
// length s (Sec. III-A-4: the equations for tau and lambda).
Layer layer_latency(const moe_cluster& c, const moe_model& m, const moe_request_mix& r, int d_tp,
                    int d_ep, int d_dp, double s) {
  const double psi_layer = (m.psi_attn + m.psi_moe) / m.layers;
  const double b_dp = double(r.batch) / d_dp;
  Layer L;
  L.tau = psi_layer / (double(d_tp) * d_ep) * b_dp * s * m.hidden / c.compute_rate;
  const double hid = b_dp * s * m.hidden * m.act_bytes;                 // b/d_DP * s * h
  const double ar = moe_cost_ar(hid, d_tp, group_bw(c, d_tp));
  double a2a;
  if (d_dp >= d_ep) {
    a2a = moe_cost_a2a(hid * m.top_k, d_ep, group_bw(c, long(d_tp) * d_ep));
  } else {
    const double red = double(r.batch) / d_ep * s * m.hidden * m.top_k * m.act_bytes;
    a2a = moe_cost_a2a(red, d_dp, group_bw(c, long(d_tp) * d_dp));
  }
  L.lambda = 2.0 * ar + 2.0 * a2a;
  return L;
}

bool degrees_ok(const moe_cluster& c, const moe_request_mix& r, int d_tp, int d_ep, int d_dp,
                int d_pp) {
  const long n = long(c.n_node) * c.n_proc;
  return pow2(d_tp) && pow2(d_ep) && pow2(d_dp) && d_pp >= 1 && long(d_tp) * d_ep == n &&
         long(d_dp) * d_tp <= n && d_dp <= r.batch;
}

// a is a better choice than b
bool better(const moe_strategy& a, const moe_strategy& b) {
  if (a.throughput != b.throughput) return a.throughput > b.throughput;
  if (a.itl != b.itl) return a.itl < b.itl;
  if (a.d_tp != b.d_tp) return a.d_tp < b.d_tp;
  return a.d_dp > b.d_dp;
}

}  // namespace

extern "C" {

double moe_cost_rs(double bytes, int32_t degree, double bw) {
  if (degree < 1 || !(bw > 0)) return NAN;
  return degree == 1 ? 0.0 : bytes / degree / bw;
}

double moe_cost_ag(double bytes, int32_t degree, double bw) { return moe_cost_rs(bytes, degree, bw); }

double moe_cost_ar(double bytes, int32_t degree, double bw) {
  if (degree < 1 || !(bw > 0)) return NAN;
  return moe_cost_rs(bytes / degree, degree, bw) + moe_cost_ag(bytes / degree, degree, bw);
}

double moe_cost_a2a(double bytes, int32_t degree, double bw) {
  if (degree < 1 || !(bw > 0)) return NAN;
  return bytes / degree * (degree - 1) / bw;
}

double moe_lambda_ep(const moe_cluster* c, const moe_model* m, double tokens) {
  if (!cluster_ok(c) || !model_ok(m) || !(tokens >= 0)) return NAN;
  const double bsh = tokens * m->hidden * m->act_bytes;
  return moe_cost_ar(bsh, c->n_proc, c->bw_intra) +
         2.0 * moe_cost_a2a(bsh * m->top_k, c->n_node, c->bw_inter);
}

double moe_lambda_mix(const moe_cluster* c, const moe_model* m, double tokens) {
  if (!cluster_ok(c) || !model_ok(m) || !(tokens >= 0)) return NAN;
  const double bsh = tokens * m->hidden * m->act_bytes;
  const double shard = bsh * m->top_k / c->n_proc;
  return moe_cost_ar(bsh, c->n_proc, c->bw_intra) + moe_cost_ag(shard, c->n_proc, c->bw_intra) +
         2.0 * moe_cost_a2a(shard, c->n_node, c->bw_inter);
}

int32_t moe_strategy_eval(const moe_cluster* c, const moe_model* m, const moe_request_mix* r,
                          int32_t d_tp, int32_t d_ep, int32_t d_dp, int32_t d_pp,
                          moe_strategy* out) {
  if (!cluster_ok(c) || !model_ok(m) || !mix_ok(r) || !out) return 1;
  if (!degrees_ok(*c, *r, d_tp, d_ep, d_dp, d_pp)) return 1;
  moe_strategy s;
  s.d_tp = d_tp; s.d_ep = d_ep; s.d_dp = d_dp; s.d_pp = d_pp;
  const Layer prf = layer_latency(*c, *m, *r, d_tp, d_ep, d_dp, double(r->len_in));
  const Layer dec = layer_latency(*c, *m, *r, d_tp, d_ep, d_dp, 1.0);
  s.tau_prf = prf.tau; s.lambda_prf = prf.lambda;
  s.tau_dec = dec.tau; s.lambda_dec = dec.lambda;
  // service latency: l layers, plus the pipeline's point-to-point hops
  const double hop = double(r->batch) / d_dp * m->hidden * m->act_bytes / c->bw_p2p;   // per unit of s
  s.svc_prf = m->layers * (prf.tau + prf.lambda) + (d_pp - 1) * hop * r->len_in;
  s.svc_dec = m->layers * (dec.tau + dec.lambda) + (d_pp - 1) * hop;
  // M/M/1 queue with service rate mu = 1 / (per-token service latency)
  const double mu = 1.0 / s.svc_dec;
  if (r->arrival_rate == 0) s.wq = 0.0;
  else if (r->arrival_rate < mu) s.wq = r->arrival_rate / (mu * (mu - r->arrival_rate));
  else s.wq = INFINITY;
  s.ttft = s.wq + s.svc_prf;
  s.itl = s.svc_dec;
  s.throughput = double(r->len_in + r->len_out) / (s.wq + s.svc_prf + r->len_out * s.svc_dec);
  // memory: weights of this device + K/V cache of the longest context
  const double ctx = double(r->len_in) + r->len_out;
  s.mem_bytes = m->psi_attn / d_tp + m->psi_moe / (double(d_ep) * d_tp) +
                2.0 * r->batch * ctx * m->hidden * m->act_bytes * m->layers / d_pp;
  s.feasible = s.mem_bytes < c->mem_bytes && isfinite(s.wq) &&
               (r->max_ttft == 0 || s.ttft <= r->max_ttft) &&
               (r->max_itl == 0 || s.itl <= r->max_itl);
  *out = s;
  return 0;
}

int32_t moe_strategy_select(const moe_cluster* c, const moe_model* m, const moe_request_mix* r,
                            int32_t d_pp, moe_strategy* best, moe_strategy* all, int32_t max_all,
                            int32_t* n_all) {
  if (!cluster_ok(c) || !model_ok(m) || !mix_ok(r) || !best || d_pp < 1 || max_all < 0) return 1;
  const long n = long(c->n_node) * c->n_proc;
  int count = 0;
  bool have = false;
  moe_strategy top;
  for (long d_tp = 1; d_tp <= n; d_tp *= 2) {
    const long d_ep = n / d_tp;
    for (long d_dp = 1; d_dp * d_tp <= n && d_dp <= r->batch; d_dp *= 2) {
      moe_strategy s;
      if (moe_strategy_eval(c, m, r, int32_t(d_tp), int32_t(d_ep), int32_t(d_dp), d_pp, &s)) return 1;
      if (all && count < max_all) all[count] = s;
      ++count;
      if (s.feasible && (!have || better(s, top))) { top = s; have = true; }
    }
  }
  if (n_all) *n_all = count;
  if (!have) return 2;
  *best = top;
  return 0;
}

}  // extern "C"
