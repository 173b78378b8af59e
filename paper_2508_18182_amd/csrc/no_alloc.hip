// adloco_norm_test_noalloc: the norm test for callers that must not allocate.
//
// adloco_norm_test keeps the partial sums of S2 = sum_l ||grad_sum_l||^2 and the device copy of the
// layer table in scratch memory that the context allocates (and reallocates when a larger list
// comes along).  Here both live in ONE file-scope device array of fixed size, `scratch`: nothing is
// allocated, freed or resized by the call, at the price of a ceiling on the size of the list.  The
// kernels are those of adloco_norm_test; they take the array's address as an argument exactly as
// they take the context's buffers there, so the two entry points return the same numbers.
#include <algorithm>

#include "common.h"

namespace adloco {
namespace {

constexpr int kNaMaxLayers = 512;                    // blocks in one call
constexpr size_t kNaMaxPartials = 131072;            // workgroups of the squared-norm kernel: 2^31 gradient entries
struct NaScratch {
  double out[32];                                    // [0]: S2
  LayerDev tab[kNaMaxLayers];
  double partial[kNaMaxPartials];
};
// Each GPU holds its own copy of this array, at its own address, until the process ends (about
// 1.1 MB).  In host code the name is only a handle for hipGetSymbolAddress: what kernels, copies
// and fills are given is the address that call returned for the device at hand.
static __device__ __align__(256) unsigned char scratch[sizeof(NaScratch)];

constexpr int kNaMaxDevices = 64;
void* g_scratch_ptr[kNaMaxDevices] = {};             // per device: address of its copy of `scratch`

// The layer table is written by a kernel from its argument (a few blocks per launch).
constexpr int kNaTabChunk = 40;
struct NaTabChunk {
  int first, count;
  LayerDev rows[kNaTabChunk];
};
__global__ void na_fill_table_kernel(LayerDev* tab, NaTabChunk c) {
  const int i = threadIdx.x;
  if (i < c.count) tab[c.first + i] = c.rows[i];
}

}  // namespace

int no_alloc_init(adloco_ctx* ctx) {
  if (ctx->device < 0 || ctx->device >= kNaMaxDevices)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "device index %d beyond %d", ctx->device, kNaMaxDevices - 1);
  if (g_scratch_ptr[ctx->device]) return ADLOCO_OK;
  void* p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));    // for the current device
  if (e != hipSuccess || !p)
    return fail(ctx, ADLOCO_EHIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
  g_scratch_ptr[ctx->device] = p;
  return ADLOCO_OK;
}

}  // namespace adloco

using namespace adloco;

extern "C" int adloco_norm_test_noalloc(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                                        const adloco_stats_acc* acc, double eta, int64_t b_cur,
                                        int64_t b_max, int32_t n_switch, int64_t b_cap, uint32_t flags,
                                        adloco_norm_test_result* out, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!layers || n_layers < 1) return fail(ctx, ADLOCO_EINVAL, "norm_test_noalloc: no layers");
  if (n_layers > kNaMaxLayers)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "norm_test_noalloc: n_layers = %d exceeds the fixed table of %d "
                "blocks (adloco_norm_test has no such limit)", n_layers, kNaMaxLayers);
  if (!acc || !out) return fail(ctx, ADLOCO_EINVAL, "norm_test_noalloc: NULL acc or out");
  if (!(eta > 0.0) || b_cur < 1 || b_max < 1 || n_switch < 1 || b_cap < 0 ||
      (flags & ~(ADLOCO_BIASED_VAR | ADLOCO_ALLOW_SHRINK)))
    return fail(ctx, ADLOCO_EINVAL, "norm_test_noalloc: bad eta, b_cur, b_max, n_switch, b_cap or flags");
  NaScratch* const S = static_cast<NaScratch*>(g_scratch_ptr[ctx->device]);
  if (!S) return fail(ctx, ADLOCO_ESTATE, "norm_test_noalloc: the device array was not looked up");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int chunk = sqnorm_chunk();
  // the table of the squared-norm kernel: grad_sum, its size, and the first workgroup of each block
  long long nblk = 0;
  NaTabChunk c;
  for (int first = 0; first < n_layers; first += kNaTabChunk) {
    c.first = first;
    c.count = std::min(kNaTabChunk, n_layers - first);
    for (int i = 0; i < c.count; ++i) {
      const adloco_linear_desc& d = layers[first + i];
      if (d.d_in < 1 || d.d_out < 1 || !d.grad_sum || (reinterpret_cast<uintptr_t>(d.grad_sum) % 4))
        return fail(ctx, ADLOCO_EINVAL, "norm_test_noalloc: layer %d has no size or no (aligned) grad_sum",
                    first + i);
      LayerDev L{};
      L.grad_sum = d.grad_sum;
      L.d_in = d.d_in;
      L.d_out = d.d_out;
      L.sq_blk_start = int(nblk);
      c.rows[i] = L;
      nblk += ((long long)d.d_in * d.d_out + chunk - 1) / chunk;
      if (nblk > (long long)kNaMaxPartials)
        return fail(ctx, ADLOCO_EUNSUPPORTED, "norm_test_noalloc: the gradient needs more than %zu partial "
                    "sums of %d entries (adloco_norm_test has no such limit)", kNaMaxPartials, chunk);
    }
    hipLaunchKernelGGL(na_fill_table_kernel, dim3(1), dim3(64), 0, st, S->tab, c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
      return fail(ctx, ADLOCO_EHIP, "norm_test_noalloc: table launch failed: %s", hipGetErrorString(e));
  }
  // every partial sum in [0, nblk) and out[0] are overwritten: nothing of an earlier call is read
  hipError_t e = launch_sqnorm_table(S->tab, n_layers, size_t(nblk), S->partial, S->out, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "norm_test_noalloc: reduction launch failed: %s", hipGetErrorString(e));
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->pinned, S->out, sizeof(double), hipMemcpyDeviceToHost, st));
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->pinned + 2, acc, sizeof(adloco_stats_acc),
                                       hipMemcpyDeviceToHost, st));
  ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
  const double S2 = ctx->pinned[0];
  adloco_stats_acc h;
  std::memcpy(&h, ctx->pinned + 2, sizeof h);
  if (h.n_samples < 1)
    return fail(ctx, ADLOCO_ESTATE, "norm_test_noalloc: accumulator holds no samples (n_samples = %lld)",
                (long long)h.n_samples);
  int rc = adloco_norm_test_decide(h.sum_sample_sqnorm, S2, h.n_samples, eta, b_cur, b_max, n_switch,
                                   b_cap, flags, out);
  if (rc) return fail(ctx, rc, "norm_test_noalloc: decision rejected S1 = %g, S2 = %g", h.sum_sample_sqnorm, S2);
  return ADLOCO_OK;
}
