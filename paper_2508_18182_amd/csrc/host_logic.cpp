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
