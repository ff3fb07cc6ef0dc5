// Closed forms of the paper's Sec. 3.2 (host only).
#include <cmath>
#include <limits>

#include "../../include/moesd.h"

extern "C" {

// Eq. N(t): each expert is missed by one token with probability (E-K)/E.
double moesd_expected_active_experts(int32_t E, int32_t K, int64_t t) {
  if (E < 1 || K < 0 || K > E || t < 0) return std::numeric_limits<double>::quiet_NaN();
  if (K == E) return t > 0 ? (double)E : 0.0;
  // log1p keeps the small-rho, large-t corner accurate
  const double log_miss = (double)t * std::log1p(-(double)K / (double)E);
  return (double)E * -std::expm1(log_miss);
}

// The per-expert form of the step before Eq. N(t): expert e is missed by one token
// with probability 1 - p[e].
double moesd_expected_active_experts_p(const double *p, int32_t E, int64_t t) {
  if (!p || E < 1 || t < 0) return std::numeric_limits<double>::quiet_NaN();
  double n = 0.0;
  for (int32_t e = 0; e < E; ++e) {
    if (!(p[e] >= 0.0) || !(p[e] <= 1.0)) return std::numeric_limits<double>::quiet_NaN();
    n += p[e] >= 1.0 ? (t > 0 ? 1.0 : 0.0) : -std::expm1((double)t * std::log1p(-p[e]));
  }
  return n;
}

// Eq. Texp: t*K routed rows spread over N(t) activated experts.
double moesd_expected_tokens_per_expert(int32_t E, int32_t K, int64_t t) {
  if (E < 1 || K < 0 || K > E || t < 0) return std::numeric_limits<double>::quiet_NaN();
  if (t == 0 || K == 0) return 0.0;
  return (double)t * (double)K / moesd_expected_active_experts(E, K, t);
}

// Eq. T_thres: ceil(log_{1-rho}(1-tau)), corrected by one step either way so the
// result is exactly the first t with N(t) >= tau*E despite rounding in the logs.
int64_t moesd_token_threshold(int32_t E, int32_t K, double tau) {
  if (E < 1 || K < 1 || K > E || !(tau >= 0.0) || !(tau < 1.0)) return -1;
  if (K == E || tau == 0.0) return 1;
  const double rho = (double)K / (double)E;
  int64_t t = (int64_t)std::ceil(std::log1p(-tau) / std::log1p(-rho));
  if (t < 1) t = 1;
  while (t > 1 && moesd_expected_active_experts(E, K, t - 1) >= tau * E) --t;
  while (moesd_expected_active_experts(E, K, t) < tau * E) ++t;
  return t;
}

}  // extern "C"
