// Context life cycle, scratch memory, tuning knobs.
#include "common.h"

namespace adloco {

static thread_local std::string g_create_err;

int ensure_scratch(adloco_ctx* ctx, Scratch& s, size_t bytes) {
  if (bytes <= s.bytes) return ADLOCO_OK;
  // round up generously so that growth is rare
  size_t want = (bytes + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
  if (s.ptr) {
    ADLOCO_HIP_CHECK(ctx, hipFree(s.ptr));  // waits for work that may still use the old block
    s.ptr = nullptr;
    s.bytes = 0;
  }
  hipError_t e = hipMalloc(&s.ptr, want);
  if (e != hipSuccess) {
    s.ptr = nullptr;
    return fail(ctx, ADLOCO_ENOMEM, "scratch allocation of %zu bytes failed: %s", want,
                hipGetErrorString(e));
  }
  s.bytes = want;
  return ADLOCO_OK;
}

static hipEvent_t get_event(adloco_ctx* ctx) {
  if (!ctx->prof_free.empty()) {
    hipEvent_t e = ctx->prof_free.back();
    ctx->prof_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

hipEvent_t prof_begin(adloco_ctx* ctx, hipStream_t st) {
  if (!ctx->profile) return nullptr;
  hipEvent_t e = get_event(ctx);
  if (e) (void)hipEventRecord(e, st);
  return e;
}

void prof_end(adloco_ctx* ctx, int kernel, hipEvent_t start, hipStream_t st) {
  if (!start) return;
  hipEvent_t stop = get_event(ctx);
  if (!stop) {
    ctx->prof_free.push_back(start);
    return;
  }
  (void)hipEventRecord(stop, st);
  ctx->prof.push_back({kernel, start, stop});
}

}  // namespace adloco

using namespace adloco;

static const char* const kProfNames[kProfCount] = {"gram", "wgrad", "finalize", "sqnorm",
                                                   "outer_step", "merge", "vector_table",
                                                   "inner_step", "inner_products", "tile_stats"};

extern "C" int adloco_profile_read(adloco_ctx* ctx, const char* kernel, double* total_ms,
                                   int* launches) {
  if (!ctx || !kernel || !total_ms || !launches) return ADLOCO_EINVAL;
  int which = -1;
  for (int k = 0; k < kProfCount; ++k)
    if (std::strcmp(kernel, kProfNames[k]) == 0) which = k;
  if (which < 0) return fail(ctx, ADLOCO_EINVAL, "profile_read: unknown kernel '%s'", kernel);
  double ms = 0.0;
  int n = 0;
  std::vector<adloco_ctx::ProfRec> keep;
  for (auto& r : ctx->prof) {
    if (r.kernel != which) {
      keep.push_back(r);
      continue;
    }
    ADLOCO_HIP_CHECK(ctx, hipEventSynchronize(r.stop));
    float t = 0.f;
    ADLOCO_HIP_CHECK(ctx, hipEventElapsedTime(&t, r.start, r.stop));
    ms += t;
    ++n;
    ctx->prof_free.push_back(r.start);
    ctx->prof_free.push_back(r.stop);
  }
  ctx->prof.swap(keep);
  *total_ms = ms;
  *launches = n;
  return ADLOCO_OK;
}

extern "C" int adloco_version(void) { return 101; }

extern "C" int adloco_table_builds(const adloco_ctx* ctx) { return ctx ? ctx->table_builds : -1; }

extern "C" int adloco_create(adloco_ctx** out, int device) {
  if (!out) {
    g_create_err = "adloco_create: out is NULL";
    return ADLOCO_EINVAL;
  }
  *out = nullptr;
  int n = 0;
  hipError_t e = hipGetDeviceCount(&n);
  if (e != hipSuccess || n <= 0) {
    g_create_err = std::string("adloco_create: no HIP device: ") + hipGetErrorString(e);
    return ADLOCO_EHIP;
  }
  if (device < 0 || device >= n) {
    g_create_err = "adloco_create: device index out of range";
    return ADLOCO_EINVAL;
  }
  e = hipSetDevice(device);
  if (e != hipSuccess) {
    g_create_err = std::string("adloco_create: hipSetDevice: ") + hipGetErrorString(e);
    return ADLOCO_EHIP;
  }
  adloco_ctx* c = new adloco_ctx();
  c->device = device;
  e = hipHostMalloc(reinterpret_cast<void**>(&c->pinned), 8 * sizeof(double), hipHostMallocDefault);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->dev_scalars), 8 * sizeof(double));
  if (e != hipSuccess) {
    g_create_err = std::string("adloco_create: allocation failed: ") + hipGetErrorString(e);
    if (c->pinned) (void)hipHostFree(c->pinned);
    delete c;
    return ADLOCO_ENOMEM;
  }
  if (int rc = no_alloc_init(c)) {
    g_create_err = "adloco_create: " + c->err;
    (void)hipFree(c->dev_scalars);
    (void)hipHostFree(c->pinned);
    delete c;
    return rc;
  }
  *out = c;
  return ADLOCO_OK;
}

extern "C" int adloco_destroy(adloco_ctx* ctx) {
  if (!ctx) return ADLOCO_EINVAL;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  Scratch* all[] = {&ctx->partials, &ctx->layer_tab, &ctx->red_f64, &ctx->sample_f64,
                    &ctx->order_tab, &ctx->group_tab, &ctx->job_tab, &ctx->wgx_tab,
                    &ctx->wgx_split, &ctx->wgx_part, &ctx->vec_tab, &ctx->emb_tab,
                    &ctx->aux_vec, &ctx->aux_perm, &ctx->aux_part, &ctx->ip_tab, &ctx->ip_tile_out,
                    &ctx->ip_dot, &ctx->ip_sq, &ctx->ip_part, &ctx->ip_flags, &ctx->ts_tab,
                    &ctx->ts_part_idx, &ctx->ts_split, &ctx->ts_ptiles, &ctx->ts_out, &ctx->ts_csr};
  for (Scratch* s : all)
    if (s->ptr) (void)hipFree(s->ptr);
  for (auto& r : ctx->prof) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  for (hipEvent_t e : ctx->prof_free) (void)hipEventDestroy(e);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  if (ctx->side_stream) (void)hipStreamDestroy(ctx->side_stream);
  if (ctx->dev_scalars) (void)hipFree(ctx->dev_scalars);
  if (ctx->pinned) (void)hipHostFree(ctx->pinned);
  delete ctx;
  return ADLOCO_OK;
}

extern "C" const char* adloco_last_error(const adloco_ctx* ctx) {
  if (!ctx) return g_create_err.c_str();
  return ctx->err.c_str();
}

extern "C" int adloco_set_tuning(adloco_ctx* ctx, const char* name, int value) {
  if (!ctx || !name) return ADLOCO_EINVAL;
  std::string n(name);
  if (n == "gram_variant") ctx->gram_variant = value;
  else if (n == "gram_job_order") {
    ctx->gram_job_order = value;
    ctx->job_tab_nt = -1;
  }
  else if (n == "wgrad_variant") ctx->wgrad_variant = value;
  else if (n == "stream_blocks_per_cu") {
    if (value < 0 || value > 64) return fail(ctx, ADLOCO_EINVAL, "stream_blocks_per_cu out of range");
    ctx->stream_blocks_per_cu = value;
  } else if (n == "ip_group") {
    if (value < 0 || value > 0x7fff) return fail(ctx, ADLOCO_EINVAL, "ip_group out of range");
    ctx->ip_group_tuning = value;
    ctx->ip_B = ctx->ip_T = -1;
  } else if (n == "overlap_aux") {
    ctx->overlap_aux = value ? 1 : 0;
  } else if (n == "stats_variant") {
    ctx->stats_variant = value ? 1 : 0;
  } else if (n == "stream_variant") ctx->stream_variant = value;
  else if (n == "profile") ctx->profile = value ? 1 : 0;
  else return fail(ctx, ADLOCO_EINVAL, "unknown tuning knob '%s'", name);
  return ADLOCO_OK;
}
