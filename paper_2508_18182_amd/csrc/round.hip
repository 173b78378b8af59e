// adloco_round: the host loop of Algorithm 3 (one outer step) over the library's own entry
// points.  No arithmetic of the method lives here: CheckMerge / DoMerge, SwitchMode, the
// statistics, the norm test, InnerOpt and OuterOpt are the calls of adloco.h.
#include <algorithm>
#include <vector>

#include "common.h"

using namespace adloco;

extern "C" int adloco_round(adloco_ctx* ctx, const adloco_round_config* cfg, adloco_trainer* trainers,
                            int* k_io, const adloco_linear_desc* layers, int n_layers, size_t N,
                            adloco_batch_fn batch_fn, adloco_round_report* reports, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!cfg || !trainers || !k_io || !layers || !batch_fn)
    return fail(ctx, ADLOCO_EINVAL, "round: NULL argument");
  const int k_in = *k_io;
  if (k_in < 1 || n_layers < 1 || N == 0)
    return fail(ctx, ADLOCO_EINVAL, "round: k = %d, n_layers = %d, N = %zu", k_in, n_layers, N);
  if (cfg->T < 1 || cfg->inner_steps < 1 || cfg->n_switch < 1 || cfg->merge_w < 0 || cfg->b_max < 1 ||
      cfg->b_cap < 0 || !(cfg->eta > 0.0))
    return fail(ctx, ADLOCO_EINVAL, "round: bad configuration");
  size_t total = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (layers[l].d_in < 1 || layers[l].d_out < 1)
      return fail(ctx, ADLOCO_EINVAL, "round: layer %d has no size", l);
    total += size_t(layers[l].d_in) * size_t(layers[l].d_out);
  }
  if (total != N)
    return fail(ctx, ADLOCO_EINVAL, "round: the blocks hold %zu parameters, N = %zu", total, N);
  for (int i = 0; i < k_in; ++i) {
    const adloco_trainer& t = trainers[i];
    if (!t.theta_outer || !t.workers || t.n_workers < 1 || t.n_workers > ADLOCO_MAX_INSTANCES ||
        t.b_req < 1 || !t.acc || !t.per_sample_sqnorm || t.reserved != 0)
      return fail(ctx, ADLOCO_EINVAL, "round: trainer %d is incomplete", i);
    for (int m = 0; m < t.n_workers; ++m) {
      const adloco_worker& w = t.workers[m];
      if (!w.theta || !w.exp_avg || !w.exp_avg_sq || !w.grad || w.step < 0)
        return fail(ctx, ADLOCO_EINVAL, "round: worker %d of trainer %d is incomplete", m, i);
    }
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  std::vector<adloco_round_report> rep(k_in);
  for (auto& r : rep) r = adloco_round_report{};

  // ---- 1. CheckMerge / DoMerge on the trainers' outer models
  int k = k_in;
  if (k > 1 && cfg->merge_w > 0) {
    std::vector<int64_t> b(k);
    for (int i = 0; i < k; ++i) b[i] = trainers[i].b_req;
    std::vector<int> sel(std::max(cfg->merge_w, 1));
    int n_sel = 0;
    int rc = adloco_check_merge(b.data(), k, cfg->merge_w, sel.data(), &n_sel);
    if (rc) return fail(ctx, rc, "round: CheckMerge rejected its arguments");
    if (n_sel > ADLOCO_MAX_INSTANCES)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "round: %d trainers to merge exceed %d", n_sel,
                  ADLOCO_MAX_INSTANCES);
    if (n_sel > 0) {
      std::vector<float*> x(n_sel);
      std::vector<double> w(n_sel);
      for (int j = 0; j < n_sel; ++j) {
        x[j] = trainers[sel[j]].theta_outer;
        w[j] = double(trainers[sel[j]].b_req);
      }
      int rep_j = -1;
      rc = adloco_merge(ctx, x.data(), w.data(), n_sel, N, -1, &rep_j, stream);
      if (rc) return rc;
      const int keep = sel[rep_j];
      // the representative stays where it is; the others go to the end, order preserved
      std::vector<char> gone(k, 0);
      for (int j = 0; j < n_sel; ++j)
        if (sel[j] != keep) gone[sel[j]] = 1;
      std::vector<adloco_trainer> left, removed;
      int keep_new = -1;
      for (int i = 0; i < k; ++i) {
        if (gone[i]) {
          removed.push_back(trainers[i]);
        } else {
          if (i == keep) keep_new = int(left.size());
          left.push_back(trainers[i]);
        }
      }
      k = int(left.size());
      for (int i = 0; i < k; ++i) trainers[i] = left[i];
      for (size_t i = 0; i < removed.size(); ++i) trainers[k + i] = removed[i];
      rep[keep_new].merged_from = n_sel - 1;
    }
  }

  // ---- 2. inner steps of every worker of every trainer
  std::vector<adloco_linear_desc> desc(n_layers);
  for (int i = 0; i < k; ++i) {
    adloco_trainer& t = trainers[i];
    adloco_round_report& R = rep[i];
    R.b_req_used = t.b_req;
    int rc = adloco_switch_mode(t.b_req, cfg->b_max, cfg->n_switch, &R.accumulate, &R.accum_steps,
                                &R.b_micro);
    if (rc) return fail(ctx, rc, "round: SwitchMode rejected b_req = %lld", (long long)t.b_req);
    if (R.b_micro > 0x7fffffffLL)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "round: micro-batch too large");
    int64_t b_next = t.b_req;
    for (int m = 0; m < t.n_workers; ++m) {
      adloco_worker& w = t.workers[m];
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(w.theta, t.theta_outer, N * sizeof(float),
                                           hipMemcpyDeviceToDevice, st));
      for (int h = 0; h < cfg->inner_steps; ++h) {
        for (int64_t s = 0; s < R.accum_steps; ++s) {
          size_t off = 0;
          for (int l = 0; l < n_layers; ++l) {
            desc[l] = layers[l];
            desc[l].a = nullptr;
            desc[l].delta = nullptr;
            desc[l].a_row_stride = desc[l].delta_row_stride = 0;
            desc[l].grad_sum = w.grad + off;
            desc[l].reserved = 0;
            off += size_t(layers[l].d_in) * size_t(layers[l].d_out);
          }
          if (batch_fn(t.user, m, h, int(s), R.b_micro, w.theta, desc.data(), n_layers, stream) != 0)
            return fail(ctx, ADLOCO_ESTATE, "round: batch_fn failed (trainer %d, worker %d, inner step "
                        "%d, micro-batch %lld)", i, m, h, (long long)s);
          // only the first inner step of worker 0 feeds the norm test: every other batch is a plain
          // gradient accumulation
          const uint32_t want = (m == 0 && h == 0) ? 0u : ADLOCO_SUM_ONLY;
          rc = adloco_grad_stats(ctx, desc.data(), n_layers, int(R.b_micro), cfg->T, cfg->dtype,
                                 t.per_sample_sqnorm, nullptr, t.acc,
                                 (s > 0 ? ADLOCO_ACCUMULATE : 0u) | want, stream);
          if (rc) return rc;
        }
        if (m == 0 && h == 0) {
          // b_cur = the samples this batch really held (SwitchMode may have cut the request to
          // b_max); the previous request stays the floor of the next one
          rc = adloco_norm_test(ctx, desc.data(), n_layers, t.acc, cfg->eta,
                                R.accum_steps * R.b_micro, cfg->b_max, cfg->n_switch, cfg->b_cap, 0,
                                &R.test, stream);
          if (rc) return rc;
          b_next = std::max<int64_t>(t.b_req, R.test.b_req);
        }
        ++w.step;
        rc = adloco_inner_step(ctx, w.theta, w.exp_avg, w.exp_avg_sq, w.grad, N,
                               1.0 / (double(R.accum_steps) * double(R.b_micro)), cfg->lr_inner,
                               cfg->beta1, cfg->beta2, cfg->eps, cfg->weight_decay, w.step, stream);
        if (rc) return rc;
      }
    }
    t.b_req = b_next;
  }

  // ---- 3. pseudo-gradient and OuterOpt per trainer
  for (int i = 0; i < k; ++i) {
    adloco_trainer& t = trainers[i];
    float* inst[ADLOCO_MAX_INSTANCES];
    for (int m = 0; m < t.n_workers; ++m) inst[m] = t.workers[m].theta;
    int rc = adloco_outer_step(ctx, t.theta_outer, inst, t.n_workers, N, t.momentum, cfg->lr_outer,
                               cfg->mu_outer, cfg->nesterov, 0, nullptr, stream);
    if (rc) return rc;
  }
  if (reports)
    for (int i = 0; i < k_in; ++i) reports[i] = rep[i];
  *k_io = k;
  return ADLOCO_OK;
}
