// Host-only decision logic: norm test and batch rule (Section 3.3.1, eq. 4), SwitchMode
// (Section 4.2; Algorithm 3) and CheckMerge (Algorithm 1).  fp64 and int64 throughout.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

#include "adloco.h"

extern "C" int adloco_switch_mode(int64_t b_req, int64_t b_max, int32_t n_switch,
                                  int32_t* accumulate, int64_t* accum_steps, int64_t* b_micro) {
  if (b_req < 1 || b_max < 1 || n_switch < 1 || !accumulate || !accum_steps || !b_micro)
    return ADLOCO_EINVAL;
  // n_switch * b_max without overflow: compare by division
  const bool over = b_req / n_switch > b_max || (b_req / n_switch == b_max && b_req % n_switch != 0);
  if (over) {
    *accumulate = 1;
    *accum_steps = b_req / b_max + (b_req % b_max != 0 ? 1 : 0);
    *b_micro = b_max;
  } else {
    *accumulate = 0;
    *accum_steps = 1;
    *b_micro = std::min(b_req, b_max);
  }
  return ADLOCO_OK;
}

extern "C" int adloco_norm_test_decide(double S1, double S2, int64_t n_samples, double eta,
                                       int64_t b_cur, int64_t b_max, int32_t n_switch,
                                       int64_t b_cap, uint32_t flags,
                                       adloco_norm_test_result* out) {
  if (!out || n_samples < 1 || !(eta > 0.0) || b_cur < 1 || b_max < 1 || n_switch < 1 ||
      b_cap < 0 || (flags & ~(ADLOCO_BIASED_VAR | ADLOCO_ALLOW_SHRINK)) || std::isnan(S1) ||
      std::isnan(S2) || S1 < 0.0 || S2 < 0.0)
    return ADLOCO_EINVAL;
  const bool biased = flags & ADLOCO_BIASED_VAR;
  const bool shrink = flags & ADLOCO_ALLOW_SHRINK;
  const int64_t ceiling = b_cap > 0 ? b_cap : std::numeric_limits<int64_t>::max();
  const double Bd = static_cast<double>(n_samples);
  adloco_norm_test_result r{};
  r.S1 = S1;
  r.S2 = S2;
  r.n_samples = n_samples;
  r.b_cur = b_cur;
  r.batch_grad_sqnorm = S2 / (Bd * Bd);
  int64_t b_req;
  if (n_samples < 2 && !biased) {
    // one sample: the sample variance is 0/0; ask for two so that it becomes defined
    r.variance = std::numeric_limits<double>::quiet_NaN();
    r.stat = std::numeric_limits<double>::quiet_NaN();
    r.stat_undefined = 1;
    r.test_passed = 0;
    b_req = std::min(ceiling, std::max<int64_t>(b_cur, 2));
  } else {
    // sum_i ||g_i - g_k||^2 = S1 - S2/B; rounding can push it slightly below zero
    const double dev = std::max(S1 - S2 / Bd, 0.0);
    r.variance = biased ? dev / Bd : dev / (Bd - 1.0);
    if (r.batch_grad_sqnorm > 0.0)
      r.stat = r.variance / (eta * eta * r.batch_grad_sqnorm);
    else
      r.stat = r.variance > 0.0 ? std::numeric_limits<double>::infinity() : 0.0;
    r.test_passed = r.stat <= static_cast<double>(b_cur) ? 1 : 0;
    int64_t b_raw;
    if (std::isinf(r.stat) || r.stat >= static_cast<double>(ceiling))
      b_raw = ceiling;
    else
      b_raw = static_cast<int64_t>(std::ceil(r.stat));
    b_req = shrink ? b_raw : std::max(b_cur, b_raw);
    b_req = std::min(ceiling, std::max<int64_t>(b_req, 1));
  }
  r.b_req = b_req;
  int rc = adloco_switch_mode(b_req, b_max, n_switch, &r.accumulate, &r.accum_steps, &r.b_micro);
  if (rc != ADLOCO_OK) return rc;
  *out = r;
  return ADLOCO_OK;
}

extern "C" int adloco_check_merge(const int64_t* b_req, int k, int w, int* sel_out, int* n_sel) {
  if (!n_sel || k < 0 || w < 0 || (k > 0 && !b_req)) return ADLOCO_EINVAL;
  *n_sel = 0;
  if (w == 0 || k <= 1) return ADLOCO_OK;
  if (w > k) return ADLOCO_OK;
  if (!sel_out) return ADLOCO_EINVAL;
  std::vector<int> order(k);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int x, int y) { return b_req[x] < b_req[y]; });
  for (int i = 0; i < w; ++i) sel_out[i] = order[i];
  *n_sel = w;
  return ADLOCO_OK;
}

// Inner-product test and augmented inner-product test (Section 3.3.2) from the batch sums.
extern "C" int adloco_inner_product_decide(double S1, double S2, double sum_ip, double sum_ip_sq,
                                           int64_t n_samples, double vartheta, double nu,
                                           int64_t b_cur, int64_t b_max, int32_t n_switch,
                                           int64_t b_cap, adloco_ip_test_result* out) {
  if (!out || n_samples < 1 || !(vartheta > 0.0) || !(nu > 0.0) || b_cur < 1 || b_max < 1 ||
      n_switch < 1 || b_cap < 0 || std::isnan(S1) || std::isnan(S2) || std::isnan(sum_ip) ||
      std::isnan(sum_ip_sq) || S1 < 0.0 || S2 < 0.0 || sum_ip_sq < 0.0)
    return ADLOCO_EINVAL;
  const int64_t ceiling = b_cap > 0 ? b_cap : std::numeric_limits<int64_t>::max();
  const double Bd = static_cast<double>(n_samples);
  adloco_ip_test_result r{};
  r.S1 = S1;
  r.S2 = S2;
  r.n_samples = n_samples;
  r.b_cur = b_cur;
  r.batch_grad_sqnorm = S2 / (Bd * Bd);
  const double nan = std::numeric_limits<double>::quiet_NaN();
  const double inf = std::numeric_limits<double>::infinity();
  if (n_samples < 2) {
    r.var_ip = r.stat_ip = r.var_aug = r.stat_aug = nan;
    r.stat_undefined = 1;
    r.b_req_ip = r.b_req_aug = std::min(ceiling, std::max<int64_t>(b_cur, 2));
  } else {
    const double gk2 = r.batch_grad_sqnorm;
    // <g_i, g_k> = c_i / B:  sum = sum_ip / B,  sum of squares = sum_ip_sq / B^2
    const double s = sum_ip / Bd, s2 = sum_ip_sq / (Bd * Bd);
    r.var_ip = std::max(s2 - s * s / Bd, 0.0) / (Bd - 1.0);
    // g_k = 0: no direction to project on, the residual is g_i itself
    r.var_aug = std::max(S1 - (gk2 > 0.0 ? s2 / gk2 : 0.0), 0.0) / (Bd - 1.0);
    auto ratio = [&](double num, double den) {
      if (den > 0.0) return num / den;
      return num > 0.0 ? inf : 0.0;
    };
    r.stat_ip = ratio(r.var_ip, vartheta * vartheta * gk2 * gk2);
    r.stat_aug = ratio(r.var_aug, nu * nu * gk2);
    auto to_batch = [&](double stat) {
      if (std::isinf(stat) || stat >= static_cast<double>(ceiling)) return ceiling;
      return static_cast<int64_t>(std::ceil(stat));
    };
    const int64_t ip_raw = to_batch(r.stat_ip);
    const int64_t aug_raw = to_batch(std::max(static_cast<double>(ip_raw), r.stat_aug));
    r.b_req_ip = std::min(ceiling, std::max<int64_t>(std::max(b_cur, ip_raw), 1));
    r.b_req_aug = std::min(ceiling, std::max<int64_t>(std::max(b_cur, aug_raw), 1));
  }
  int rc = adloco_switch_mode(r.b_req_ip, b_max, n_switch, &r.accumulate_ip, &r.accum_steps_ip,
                              &r.b_micro_ip);
  if (rc != ADLOCO_OK) return rc;
  rc = adloco_switch_mode(r.b_req_aug, b_max, n_switch, &r.accumulate_aug, &r.accum_steps_aug,
                          &r.b_micro_aug);
  if (rc != ADLOCO_OK) return rc;
  *out = r;
  return ADLOCO_OK;
}
