// pass-KV / pass-Q selection rules (Section 3.3 Algorithm 1, Appendix C Algorithm 5,
// Appendix D). Host arithmetic only.
#include <cmath>

#include "cp_attn.h"

extern "C" int cp_select_order(const cp_select_params* p, int64_t t_new, int64_t p_cached,
                               int32_t rule, int32_t* order_out) {
  if (p == nullptr || order_out == nullptr) return CP_ERR_NULL;
  if (t_new < 1 || p_cached < 0 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_ranks < 1 ||
      p->reserved != 0)
    return CP_ERR_SHAPE;
  const double T = (double)t_new, P = (double)p_cached;
  const double miss = T / (T + P);  // KV cache miss rate
  bool pass_kv;
  if (rule == CP_RULE_EMPIRICAL) {
    double a = p->alpha, b = p->beta, g = p->gamma;
    if (a == 0.0 && b == 0.0 && g == 0.0) { a = -1.059; b = 1.145; g = 12.112; }
    pass_kv = a * std::log(T) + b * std::log(miss) + g > 0.0;
  } else if (rule == CP_RULE_ANALYTIC || rule == CP_RULE_ANALYTIC_ALL2ALL) {
    if (!(p->peak_flops > 0.0) || !(p->bandwidth > 0.0) || !(p->bytes_per_elem > 0.0))
      return CP_ERR_SHAPE;
    const double N = p->n_ranks, C = p->peak_flops, BW = p->bandwidth, e = p->bytes_per_elem;
    const double ratio = (double)p->n_kv_heads / (double)p->n_q_heads;
    const double t_hidden = N * C * ratio * e / (2.0 * BW);  // Equation 2
    double miss_limit = 2.0 * ratio;                          // Equation 1
    if (rule == CP_RULE_ANALYTIC_ALL2ALL) miss_limit -= 4.0 * T * BW / (N * C * e);
    pass_kv = T >= t_hidden || miss >= miss_limit;
  } else {
    return CP_ERR_UNSUPPORTED;
  }
  *order_out = pass_kv ? CP_ORDER_PASS_KV : CP_ORDER_PASS_Q;
  return CP_OK;
}
