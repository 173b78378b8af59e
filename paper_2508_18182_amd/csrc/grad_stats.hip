// Entry points of the statistics half: adloco_grad_stats (per-sample norms by the Gram
// identity, gradient sum, S1 accumulation) and adloco_norm_test (S2 on the device, then the
// decision on the host).
#include <algorithm>
#include <numeric>

#include "common.h"

using namespace adloco;

namespace {

constexpr int kMaxLayers = 4096;

// The device copy of the layer table keeps its shapes, strides and launch positions from call to
// call; only the three pointers of every block change when the caller hands in other tensors (fresh
// activations of the next micro-batch, another worker's gradient buffers).  They travel in the
// argument of a small kernel, so that a call on a known list of shapes uploads nothing, waits for
// nothing, and can be captured into a graph with its pointers in it.
constexpr int kPtrChunk = 120;
struct PtrChunk {
  int first, count, which;            // which: 1 = a and delta, 2 = grad_sum, 3 = all
  int pad;
  const void* a[kPtrChunk];
  const void* delta[kPtrChunk];
  float* grad_sum[kPtrChunk];
};
__global__ void set_layer_pointers_kernel(LayerDev* tab, PtrChunk c) {
  const int i = threadIdx.x;
  if (i >= c.count) return;
  LayerDev& L = tab[c.first + i];
  if (c.which & 1) {
    L.a = c.a[i];
    L.delta = c.delta[i];
  }
  if (c.which & 2) L.grad_sum = c.grad_sum[i];
}

int upload_pointers(adloco_ctx* ctx, const std::vector<LayerDev>& tab, int which, hipStream_t st) {
  PtrChunk c;
  for (size_t first = 0; first < tab.size(); first += kPtrChunk) {
    c.first = int(first);
    c.count = int(std::min<size_t>(kPtrChunk, tab.size() - first));
    c.which = which;
    c.pad = 0;
    for (int i = 0; i < c.count; ++i) {
      c.a[i] = tab[first + i].a;
      c.delta[i] = tab[first + i].delta;
      c.grad_sum[i] = tab[first + i].grad_sum;
    }
    hipLaunchKernelGGL(set_layer_pointers_kernel, dim3(1), dim3(128), 0, st,
                       static_cast<LayerDev*>(ctx->layer_tab.ptr), c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
      return fail(ctx, ADLOCO_EHIP, "pointer table launch failed: %s", hipGetErrorString(e));
  }
  return ADLOCO_OK;
}

// Everything of a block that the tables, tile lists and kernel choices depend on: all of LayerDev
// but the addresses themselves (their alignment class is in `fast`, whether they are there at all
// is compared).
bool same_shape(const LayerDev& x, const LayerDev& y) {
  return x.a_stride == y.a_stride && x.delta_stride == y.delta_stride && x.d_in == y.d_in &&
         x.d_out == y.d_out && x.fast == y.fast && x.provided == y.provided && x.kind == y.kind &&
         x.wg_blk_start == y.wg_blk_start && x.sq_blk_start == y.sq_blk_start && x.delta_twin == y.delta_twin && x.a_twin == y.a_twin &&
         (x.a == nullptr) == (y.a == nullptr) && (x.delta == nullptr) == (y.delta == nullptr) &&
         (x.grad_sum == nullptr) == (y.grad_sum == nullptr);
}

// Build the device view of the layer list.  A list whose shapes (widths, strides, kinds, flags,
// alignment classes) equal those of the previous call only has its pointers refreshed, by a kernel on
// the caller's stream; any other list rebuilds every table that depends on it, which allocates,
// copies from pageable memory and waits for the stream.
int prepare_tables(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers, int dtype,
                   bool need_inputs, hipStream_t st) {
  const size_t esize = is_16bit(dtype) ? 2 : 4;
  std::vector<LayerDev> tab(n_layers);
  const int wt = wgrad_tile_edge(dtype);
  const int chunk = sqnorm_chunk();
  long long wg = 0, sq = 0;
  for (int l = 0; l < n_layers; ++l) {
    const adloco_linear_desc& d = layers[l];
    if (d.d_in < 1 || d.d_out < 1)
      return fail(ctx, ADLOCO_EINVAL, "layer %d: d_in = %d, d_out = %d must be >= 1", l, d.d_in, d.d_out);
    if (d.reserved != 0 || (d.flags & ~(ADLOCO_GRAD_PROVIDED | ADLOCO_KIND_MASK)))
      return fail(ctx, ADLOCO_EINVAL, "layer %d: unknown flags or non-zero reserved field", l);
    const bool provided = d.flags & ADLOCO_GRAD_PROVIDED;
    const int kind = int(d.flags & ADLOCO_KIND_MASK);
    if (kind != ADLOCO_KIND_LINEAR && kind != ADLOCO_KIND_VECTOR && kind != ADLOCO_KIND_EMBED)
      return fail(ctx, ADLOCO_EINVAL, "layer %d: unknown kind 0x%x", l, kind);
    if (kind == ADLOCO_KIND_VECTOR && d.d_in != 1)
      return fail(ctx, ADLOCO_EINVAL, "layer %d: a vector block needs d_in = 1", l);
    if (kind == ADLOCO_KIND_EMBED && !provided)
      return fail(ctx, ADLOCO_EINVAL, "layer %d: an embedding block needs ADLOCO_GRAD_PROVIDED", l);
    LayerDev L{};
    L.a = d.a;
    L.delta = d.delta;
    L.grad_sum = d.grad_sum;
    L.a_stride = d.a_row_stride ? d.a_row_stride : (kind == ADLOCO_KIND_VECTOR ? d.d_out : d.d_in);
    L.delta_stride = d.delta_row_stride ? d.delta_row_stride : d.d_out;
    L.d_in = d.d_in;
    L.d_out = d.d_out;
    L.provided = provided ? 1 : 0;
    L.kind = kind;
    if (need_inputs) {
      if (!d.delta || (!d.a && kind != ADLOCO_KIND_VECTOR))
        return fail(ctx, ADLOCO_EINVAL, "layer %d: a or delta is NULL", l);
      const long long a_width = kind == ADLOCO_KIND_LINEAR ? d.d_in : d.d_out;
      if ((kind != ADLOCO_KIND_EMBED && d.a && L.a_stride < a_width) || L.delta_stride < d.d_out)
        return fail(ctx, ADLOCO_EINVAL, "layer %d: row stride smaller than the row", l);
      const size_t a_esize = kind == ADLOCO_KIND_EMBED ? 4 : esize;
      if ((reinterpret_cast<uintptr_t>(d.a) % a_esize) || (reinterpret_cast<uintptr_t>(d.delta) % esize))
        return fail(ctx, ADLOCO_EINVAL, "layer %d: a or delta not aligned to its element size", l);
      if (!provided && !d.grad_sum)
        return fail(ctx, ADLOCO_EINVAL, "layer %d: grad_sum is NULL without ADLOCO_GRAD_PROVIDED", l);
      const bool d_fast = (reinterpret_cast<uintptr_t>(d.delta) % 16 == 0) && (d.d_out % 8 == 0) &&
                          (L.delta_stride % 8 == 0);
      if (kind == ADLOCO_KIND_LINEAR)
        L.fast = d_fast && (reinterpret_cast<uintptr_t>(d.a) % 16 == 0) && (d.d_in % 8 == 0) &&
                 (L.a_stride % 8 == 0);
      else if (kind == ADLOCO_KIND_VECTOR)
        L.fast = d_fast && (!d.a || ((reinterpret_cast<uintptr_t>(d.a) % 16 == 0) &&
                                     (L.a_stride % 8 == 0)));
      else
        L.fast = 0;
    } else if (!d.grad_sum) {
      return fail(ctx, ADLOCO_EINVAL, "layer %d: grad_sum is NULL", l);
    }
    if (d.grad_sum && (reinterpret_cast<uintptr_t>(d.grad_sum) % 4))
      return fail(ctx, ADLOCO_EINVAL, "layer %d: grad_sum not 4-byte aligned", l);
    L.a_twin = -1;
    if (need_inputs && kind == ADLOCO_KIND_LINEAR && d.a)
      for (int j = 0; j < l; ++j)
        if (tab[j].kind == ADLOCO_KIND_LINEAR && tab[j].a == L.a && tab[j].a_stride == L.a_stride &&
            tab[j].d_in == L.d_in && tab[j].d_out == L.d_out && tab[j].delta_stride == L.delta_stride) {
          L.a_twin = j;
          break;
        }
    L.delta_twin = -1;
    if (need_inputs && kind == ADLOCO_KIND_VECTOR)
      for (int j = 0; j < l; ++j)
        if (tab[j].kind == ADLOCO_KIND_VECTOR && tab[j].delta == L.delta && tab[j].d_out == L.d_out &&
            tab[j].delta_stride == L.delta_stride) {
          L.delta_twin = j;
          break;
        }
    L.wg_blk_start = int(wg);
    L.sq_blk_start = int(sq);
    if (!provided && kind == ADLOCO_KIND_LINEAR)
      wg += (long long)((d.d_out + wt - 1) / wt) * ((d.d_in + wt - 1) / wt);
    sq += ((long long)d.d_in * d.d_out + chunk - 1) / chunk;
    if (wg > 0x7fffffffLL || sq > 0x7fffffffLL)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "layer list too large for one launch");
    tab[l] = L;
  }
  bool same = ctx->table_dtype == dtype && ctx->table_inputs == int(need_inputs) &&
              tab.size() == ctx->layer_tab_host.size();
  for (size_t l = 0; same && l < tab.size(); ++l) same = same_shape(tab[l], ctx->layer_tab_host[l]);
  if (same) {
    int rc = upload_pointers(ctx, tab, 3, st);
    if (rc) return rc;
    ctx->layer_tab_host = std::move(tab);
    return ADLOCO_OK;
  }
  ++ctx->table_builds;
  // linear layers, heaviest first, so that the tail of the Gram launch is made of cheap workgroups
  std::vector<int> order;
  for (int l = 0; l < n_layers; ++l)
    if (tab[l].kind == ADLOCO_KIND_LINEAR) order.push_back(l);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
    return (long long)tab[x].d_in + tab[x].d_out > (long long)tab[y].d_in + tab[y].d_out;
  });
  int rc = ensure_scratch(ctx, ctx->layer_tab, tab.size() * sizeof(LayerDev));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->order_tab, std::max<size_t>(order.size(), 1) * sizeof(int));
  if (rc) return rc;
  ctx->layer_tab_host.clear();          // invalid until both copies are enqueued
  ctx->table_dtype = -1;
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->layer_tab.ptr, tab.data(), tab.size() * sizeof(LayerDev),
                                       hipMemcpyHostToDevice, st));
  if (!order.empty())
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->order_tab.ptr, order.data(), order.size() * sizeof(int),
                                         hipMemcpyHostToDevice, st));
  // pageable sources: make sure the runtime has consumed them before they go out of scope
  ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
  bool f64 = need_inputs;
  for (const LayerDev& L : tab)
    if (L.kind == ADLOCO_KIND_LINEAR) f64 = f64 && L.fast && L.d_in % 64 == 0 && L.d_out % 64 == 0;
  ctx->all_fast64 = f64;
  long long widest = 0;
  for (const LayerDev& L : tab)
    if (L.kind == ADLOCO_KIND_LINEAR) widest = std::max(widest, std::max(L.a_stride, L.delta_stride));
  ctx->max_lin_stride = widest;
  bool fast = need_inputs;
  for (const LayerDev& L : tab)
    if (L.kind == ADLOCO_KIND_LINEAR) fast = fast && (L.provided || L.fast);
  ctx->all_fast = fast;
  ctx->n_linear = int(order.size());
  {
    // groups of linear layers that read the same activation tensor, for the dual-tile Gram kernel
    std::vector<GramGroup> groups;
    std::vector<int> group_of(tab.size(), -1);
    for (int l = 0; l < n_layers; ++l) {
      if (tab[l].kind != ADLOCO_KIND_LINEAR) continue;
      const int t = tab[l].a_twin;
      if (t >= 0 && group_of[t] >= 0 && groups[group_of[t]].n < kGramGroupMax && tab[t].fast == tab[l].fast) {
        GramGroup& G = groups[group_of[t]];
        G.layer[G.n++] = l;
        group_of[l] = group_of[t];
      } else {
        GramGroup G{};
        G.n = 1;
        G.layer[0] = l;
        group_of[l] = int(groups.size());
        groups.push_back(G);
      }
    }
    // a second table with every layer in a group of its own, for sequences with a ragged last tile
    std::vector<GramGroup> single;
    for (int l : order) {
      GramGroup G{};
      G.n = 1;
      G.layer[0] = l;
      single.push_back(G);
    }
    std::vector<int> gorder(groups.size()), sorder(single.size());
    std::iota(gorder.begin(), gorder.end(), 0);
    std::iota(sorder.begin(), sorder.end(), 0);       // `order` is sorted already
    auto weight = [&](int gi) {
      const GramGroup& G = groups[gi];
      return (long long)tab[G.layer[0]].d_in + (long long)G.n * tab[G.layer[0]].d_out;
    };
    std::stable_sort(gorder.begin(), gorder.end(), [&](int x, int y) { return weight(x) > weight(y); });
    // layout: groups | their order | singleton groups | their order
    std::vector<char> blob;
    auto append = [&](const void* p, size_t n) {
      const char* c = static_cast<const char*>(p);
      blob.insert(blob.end(), c, c + n);
    };
    append(groups.data(), groups.size() * sizeof(GramGroup));
    append(gorder.data(), gorder.size() * sizeof(int));
    ctx->single_off = blob.size();
    append(single.data(), single.size() * sizeof(GramGroup));
    append(sorder.data(), sorder.size() * sizeof(int));
    rc = ensure_scratch(ctx, ctx->group_tab, std::max<size_t>(blob.size(), 16));
    if (rc) return rc;
    if (!blob.empty()) {
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->group_tab.ptr, blob.data(), blob.size(), hipMemcpyHostToDevice, st));
      ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
    }
    ctx->n_groups = int(groups.size());
  }
  ctx->aux_B = ctx->aux_T = -1;         // the vector / table descriptor lists follow the table
  ctx->ip_B = ctx->ip_T = -1;           // and so does the inner-product tile table
  ctx->ts_B = -1;                       // and the statistics tile table
  {
    // (the tile kernels address the rows of a chunk with 32-bit byte offsets)
    bool ok = need_inputs && is_16bit(dtype) && !order.empty() && widest < (1 << 25);
    for (const LayerDev& L : tab)
      if (L.kind == ADLOCO_KIND_LINEAR) ok = ok && !L.provided && L.fast;
    ctx->ts_ok = ok;
  }
  ctx->wgx_slots = 0;
  if (fast && is_16bit(dtype) && wg > 0 && widest < (1 << 25)) {
    std::vector<int4> tiles, split;
    int n_pieces = 0;
    const int slots = make_wgrad_x_tiles(tab, tiles, split, n_pieces);
    rc = ensure_scratch(ctx, ctx->wgx_tab, tiles.size() * sizeof(int4));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->wgx_split, std::max<size_t>(split.size(), 1) * sizeof(int4));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->wgx_part, std::max<size_t>(n_pieces, 1) * 256 * 256 * sizeof(float));
    if (rc) return rc;
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->wgx_tab.ptr, tiles.data(), tiles.size() * sizeof(int4),
                                         hipMemcpyHostToDevice, st));
    if (!split.empty())
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->wgx_split.ptr, split.data(),
                                           split.size() * sizeof(int4), hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
    ctx->wgx_slots = slots;
    ctx->wgx_n_split = int(split.size());
  }
  ctx->layer_tab_host = std::move(tab);
  ctx->order_host = std::move(order);
  ctx->wgrad_blocks = int(wg);
  ctx->table_dtype = dtype;
  ctx->table_inputs = int(need_inputs);
  return ADLOCO_OK;
}

// Descriptor lists of the vector and embedding-table blocks for a batch of B x T tokens, and
// the scratch they need.  Rebuilt when the layer table or the batch shape changed.
int prepare_vector_table(adloco_ctx* ctx, int B, int T, hipStream_t st) {
  if (ctx->aux_B == B && ctx->aux_T == T) return ADLOCO_OK;
  ++ctx->table_builds;
  const int slab = vector_table_slab();
  std::vector<AuxDesc> vec, emb;
  std::vector<char> fused;     // per vector block: 1 = its row sums are formed by another block's workgroups
  long long vb = 0, vb2 = 0, eb = 0, voff = 0, poff = 0, partoff = 0;
  for (size_t l = 0; l < ctx->layer_tab_host.size(); ++l) {
    const LayerDev& L = ctx->layer_tab_host[l];
    if (L.kind == ADLOCO_KIND_LINEAR) continue;
    AuxDesc A{};
    A.layer = int(l);
    const int w = L.kind == ADLOCO_KIND_VECTOR ? slab : embed_table_slab();
    A.slabs = (L.d_out + w - 1) / w;
    if (L.kind == ADLOCO_KIND_VECTOR) {
      A.blk_start = int(vb);
      A.blk_start2 = int(vb2);
      A.vec_off = voff;
      A.vec_off_bias = -1;
      // a gain (x given) and a bias (x = 1) that read the same delta rows -- the two vectors of a
      // normalisation layer -- are formed in one pass over delta by the gain block's workgroups
      int host = -1;
      if (L.delta_twin >= 0) {
        for (size_t k = 0; k < vec.size(); ++k)
          if (vec[k].layer == L.delta_twin) host = int(k);
      }
      const bool pair = host >= 0 && vec[host].vec_off_bias < 0 && !fused[host] &&
                        (ctx->layer_tab_host[vec[host].layer].a == nullptr) != (L.a == nullptr);
      if (pair && L.a == nullptr) {
        // this bias rides on the earlier gain block: no row-sum workgroups of its own
        vec[host].vec_off_bias = voff;
        fused.push_back(1);
      } else if (pair) {
        // this gain also serves the earlier bias block, whose workgroups are withdrawn
        A.vec_off_bias = vec[host].vec_off;
        const long long gone = (long long)B * vec[host].slabs;
        for (size_t k = host + 1; k < vec.size(); ++k) vec[k].blk_start -= int(gone);
        vb -= gone;
        A.blk_start = int(vb);
        fused[host] = 1;
        fused.push_back(0);
      } else {
        fused.push_back(0);
      }
      if (!(pair && L.a == nullptr)) vb += (long long)B * A.slabs;
      vb2 += A.slabs;
      voff += (long long)B * L.d_out;
      vec.push_back(A);
    } else {
      A.blk_start = int(eb);
      A.perm_off = poff;
      A.part_off = partoff;
      eb += (long long)B * A.slabs;
      poff += (long long)B * T;
      partoff += (long long)B * A.slabs;
      emb.push_back(A);
    }
    if (vb > 0x7fffffffLL || eb > 0x7fffffffLL)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: too many vector / table blocks for one launch");
  }
  if (!emb.empty() && T > 8192)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: embedding blocks need T <= 8192, got %d", T);
  int rc = ensure_scratch(ctx, ctx->vec_tab, std::max<size_t>(vec.size(), 1) * sizeof(AuxDesc));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->emb_tab, std::max<size_t>(emb.size(), 1) * sizeof(AuxDesc));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->aux_vec, std::max<size_t>(size_t(voff), 1) * sizeof(float));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->aux_perm, std::max<size_t>(size_t(poff), 1) * sizeof(int));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->aux_part, std::max<size_t>(size_t(partoff), 1) * sizeof(double));
  if (rc) return rc;
  ctx->aux_B = ctx->aux_T = -1;
  if (!vec.empty())
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->vec_tab.ptr, vec.data(), vec.size() * sizeof(AuxDesc),
                                         hipMemcpyHostToDevice, st));
  if (!emb.empty())
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->emb_tab.ptr, emb.data(), emb.size() * sizeof(AuxDesc),
                                         hipMemcpyHostToDevice, st));
  if (!vec.empty() || !emb.empty()) ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
  ctx->vec_host = std::move(vec);
  ctx->emb_host = std::move(emb);
  ctx->vec_blocks = int(vb);
  ctx->vec_blocks2 = int(vb2);
  ctx->emb_blocks = int(eb);
  ctx->aux_B = B;
  ctx->aux_T = T;
  return ADLOCO_OK;
}

}  // namespace

extern "C" int adloco_grad_stats(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                                 int B, int T, int dtype, float* per_sample_sqnorm,
                                 float* per_layer_sample_sqnorm, adloco_stats_acc* acc,
                                 uint32_t flags, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!layers || n_layers < 1) return fail(ctx, ADLOCO_EINVAL, "grad_stats: no layers");
  if (n_layers > kMaxLayers)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: n_layers = %d exceeds %d", n_layers, kMaxLayers);
  if (B < 1 || T < 1) return fail(ctx, ADLOCO_EINVAL, "grad_stats: B = %d, T = %d must be >= 1", B, T);
  if (dtype != ADLOCO_F32 && !is_16bit(dtype))
    return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: dtype %d not supported", dtype);
  if (flags & ~(ADLOCO_ACCUMULATE | ADLOCO_SUM_ONLY)) return fail(ctx, ADLOCO_EINVAL, "grad_stats: unknown flags");
  const bool sum_only = (flags & ADLOCO_SUM_ONLY) != 0;
  if (!sum_only && (!per_sample_sqnorm || !acc)) return fail(ctx, ADLOCO_EINVAL, "grad_stats: NULL output");
  if (reinterpret_cast<uintptr_t>(acc) % 8)
    return fail(ctx, ADLOCO_EINVAL, "grad_stats: acc not 8-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int accumulate = (flags & ADLOCO_ACCUMULATE) ? 1 : 0;

  int rc = prepare_tables(ctx, layers, n_layers, dtype, true, st);
  if (rc) return rc;
  rc = prepare_vector_table(ctx, B, T, st);
  if (rc) return rc;

  const int tile = gram_tile_edge(dtype, ctx->gram_variant);
  const long long nt = (T + tile - 1) / tile;
  if (nt > 4096) return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: T = %d gives too many tiles", T);
  // (the dual-tile kernel addresses a sample's rows with 32-bit byte offsets)
  const bool dual = is_16bit(dtype) && ctx->gram_variant != 0 && ctx->all_fast64 &&
                    (long long)T * ctx->max_lin_stride < (1LL << 31) - 64;
  long long n_pairs = nt * (nt + 1) / 2;      // partial sums per (layer, sample)
  if (dual) {
    if (ctx->job_tab_nt != int(nt)) {
      ++ctx->table_builds;
      std::vector<GramJob> jobs = make_gram_jobs(int(nt), ctx->gram_job_order >= 0 ? ctx->gram_job_order : (nt >= 6 ? 0 : 1));
      rc = ensure_scratch(ctx, ctx->job_tab, jobs.size() * sizeof(GramJob));
      if (rc) return rc;
      ctx->job_tab_nt = -1;
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->job_tab.ptr, jobs.data(), jobs.size() * sizeof(GramJob),
                                           hipMemcpyHostToDevice, st));
      ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
      ctx->job_tab_nt = int(nt);
      ctx->job_tab_n = int(jobs.size());
    }
    n_pairs = gram_dual_parts(ctx->job_tab_n);
  }
  const long long n_part = (long long)n_layers * B * n_pairs;
  if (n_pairs > 0x7fffffffLL || n_part > (1LL << 40))
    return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: T = %d gives too many tile pairs", T);
  rc = ensure_scratch(ctx, ctx->partials, size_t(n_part) * sizeof(float));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->sample_f64, size_t(B) * sizeof(double));
  if (rc) return rc;

  // Per-sample gradient tiles (explicit form) when every linear block qualifies: the tiles that
  // add up to the gradient sum are squared on the way, no Gram contraction is needed.
  const bool tile_form = !sum_only && ctx->stats_variant != 0 && ctx->ts_ok && T % 32 == 0 &&
                         T <= (1 << 20) && B <= 0x7fff;
  if (tile_form && ctx->ts_B != B) {
    ++ctx->table_builds;
    const std::vector<LayerDev>& tab = ctx->layer_tab_host;
    std::vector<char> use(n_layers, 0);
    for (int l = 0; l < n_layers; ++l) use[l] = tab[l].kind == ADLOCO_KIND_LINEAR;
    std::vector<int4> tiles, split;
    std::vector<int> part, lay, ptr, idx;
    int n_pieces = 0;
    const int slots = make_stats_tiles(tab, use, B, tiles, part, split, lay, ptr, idx, n_pieces);
    if ((long long)slots * kNumXcd > 0x7fffffffLL)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "grad_stats: too many tiles for one launch");
    std::vector<int> csr;
    csr.insert(csr.end(), lay.begin(), lay.end());
    csr.insert(csr.end(), ptr.begin(), ptr.end());
    csr.insert(csr.end(), idx.begin(), idx.end());
    rc = ensure_scratch(ctx, ctx->ts_tab, tiles.size() * sizeof(int4));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ts_part_idx, part.size() * sizeof(int));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ts_split, std::max<size_t>(split.size(), 1) * sizeof(int4));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ts_ptiles, std::max<size_t>(n_pieces, 1) * 256 * 128 * sizeof(float));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ts_out, tiles.size() * size_t(B) * 16 * sizeof(float));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ts_csr, csr.size() * sizeof(int));
    if (rc) return rc;
    ctx->ts_B = -1;
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ts_tab.ptr, tiles.data(), tiles.size() * sizeof(int4),
                                         hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ts_part_idx.ptr, part.data(), part.size() * sizeof(int),
                                         hipMemcpyHostToDevice, st));
    if (!split.empty())
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ts_split.ptr, split.data(), split.size() * sizeof(int4),
                                           hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ts_csr.ptr, csr.data(), csr.size() * sizeof(int),
                                         hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
    ctx->ts_slots = slots;
    ctx->ts_n_split = int(split.size());
    ctx->ts_n_listed = int(lay.size());
    ctx->ts_idx_len = int(idx.size());
    ctx->ts_B = B;
  }

  GramLaunch g;
  g.layers = static_cast<const LayerDev*>(ctx->layer_tab.ptr);
  g.order = static_cast<const int*>(ctx->order_tab.ptr);
  g.n_layers = ctx->n_linear;   // the Gram launch walks order_tab: linear weights only
  g.B = B;
  g.T = T;
  g.partials = static_cast<float*>(ctx->partials.ptr);
  g.n_pairs = int(n_pairs);
  g.tile = tile;
  g.dtype = dtype;
  // ---- vector / table blocks.  With linear blocks in the same call they go to a second stream:
  // they are HBM-bound, the kernels of the linear blocks MFMA / L2-bound, and both fit on a CU.
  const bool have_aux = !ctx->vec_host.empty() || !ctx->emb_host.empty();
  bool fork = have_aux && ctx->n_linear > 0 && ctx->overlap_aux != 0;
  if (fork && !ctx->side_stream) {
    if (hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      fork = false;                      // no second stream: run in line
    }
  }
  hipStream_t aux_st = fork ? ctx->side_stream : st;
  auto launch_aux = [&]() -> int {
    hipEvent_t ev_aux = prof_begin(ctx, aux_st);
    hipError_t ea = launch_vector_stats(g.layers, static_cast<const AuxDesc*>(ctx->vec_tab.ptr),
                                        int(ctx->vec_host.size()), ctx->vec_blocks, ctx->vec_blocks2, B, T,
                                        dtype, static_cast<float*>(ctx->aux_vec.ptr), g.partials,
                                        int(n_pairs), accumulate, true, aux_st);
    if (ea == hipSuccess && !sum_only)
      ea = launch_embed_stats(g.layers, static_cast<const AuxDesc*>(ctx->emb_tab.ptr),
                              int(ctx->emb_host.size()), ctx->emb_blocks, B, T, dtype,
                              static_cast<int*>(ctx->aux_perm.ptr),
                              static_cast<double*>(ctx->aux_part.ptr), g.partials, int(n_pairs), aux_st);
    prof_end(ctx, kProfVecTab, ev_aux, aux_st);
    if (ea != hipSuccess)
      return fail(ctx, ADLOCO_EHIP, "grad_stats: vector / table launch failed: %s", hipGetErrorString(ea));
    return ADLOCO_OK;
  };
  if (fork) {
    ADLOCO_HIP_CHECK(ctx, hipEventRecord(ctx->ev_fork, st));
    ADLOCO_HIP_CHECK(ctx, hipStreamWaitEvent(aux_st, ctx->ev_fork, 0));
    rc = launch_aux();
    if (rc) return rc;
  }
  hipEvent_t ev = nullptr;
  hipError_t e = hipSuccess;
  if (tile_form) {
    ev = prof_begin(ctx, st);
    const int* csr = static_cast<const int*>(ctx->ts_csr.ptr);
    const int nl = ctx->ts_n_listed;
    e = launch_stats_tiles(g.layers, ctx->ts_tab.ptr, static_cast<const int*>(ctx->ts_part_idx.ptr),
                           ctx->ts_slots, ctx->ts_split.ptr, ctx->ts_n_split,
                           static_cast<float*>(ctx->ts_ptiles.ptr), B, T, dtype, accumulate,
                           static_cast<float*>(ctx->ts_out.ptr), csr, csr + nl, csr + nl + nl + 1, nl,
                           g.partials, int(n_pairs), st);
    prof_end(ctx, kProfTileStats, ev, st);
    if (e != hipSuccess)
      return fail(ctx, ADLOCO_EHIP, "grad_stats: tile statistics launch failed: %s", hipGetErrorString(e));
  }
  ev = (!tile_form && !sum_only && ctx->n_linear > 0) ? prof_begin(ctx, st) : nullptr;
  if (tile_form || sum_only || ctx->n_linear == 0)
    ;
  else if (dual) {
    // the dual-tile kernel walks groups of layers that share their activations (A A^T once per group)
    // when some do and no tile is ragged, else every layer by itself
    GramLaunch gd = g;
    const bool grouped = ctx->n_groups < ctx->n_linear && T % tile == 0;
    const char* base = static_cast<const char*>(ctx->group_tab.ptr) + (grouped ? 0 : ctx->single_off);
    gd.n_layers = grouped ? ctx->n_groups : ctx->n_linear;
    gd.order = reinterpret_cast<const int*>(base + size_t(gd.n_layers) * sizeof(GramGroup));
    e = launch_gram_bf16_dual(gd, reinterpret_cast<const GramGroup*>(base),
                              static_cast<const GramJob*>(ctx->job_tab.ptr), ctx->job_tab_n,
                              grouped ? kGramGroupMax : 1, st);
  }
  else if (is_16bit(dtype))
    e = launch_gram_bf16(g, ctx->gram_variant, st);
  else
    e = launch_gram_f32(g, st);
  prof_end(ctx, kProfGram, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "grad_stats: Gram launch failed: %s", hipGetErrorString(e));
  ev = (!tile_form && ctx->wgrad_blocks > 0) ? prof_begin(ctx, st) : nullptr;
  const long long rows = (long long)B * T;
  if (tile_form)
    ;
  else if (is_16bit(dtype) && ctx->wgrad_variant >= 2 && ctx->wgx_slots > 0 && rows % 32 == 0 &&
           rows / 32 <= 0x7fffffffLL)
    e = launch_wgrad_x(g.layers, ctx->wgx_tab.ptr, ctx->wgx_slots, ctx->wgx_split.ptr,
                       ctx->wgx_n_split, static_cast<float*>(ctx->wgx_part.ptr), rows, accumulate,
                       dtype, st);
  else
    e = launch_wgrad(g.layers, n_layers, ctx->wgrad_blocks, rows, dtype, accumulate,
                     ctx->wgrad_variant >= 2 ? 1 : ctx->wgrad_variant, st);
  prof_end(ctx, kProfWgrad, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "grad_stats: gradient-sum launch failed: %s", hipGetErrorString(e));
  if (have_aux && !fork) {
    rc = launch_aux();
    if (rc) return rc;
  }
  if (fork) {
    ADLOCO_HIP_CHECK(ctx, hipEventRecord(ctx->ev_join, aux_st));
    ADLOCO_HIP_CHECK(ctx, hipStreamWaitEvent(st, ctx->ev_join, 0));
  }
  if (sum_only) return ADLOCO_OK;       // the gradient sums are all this call was asked for
  e = launch_finalize_stats(g.partials, n_layers, B, int(n_pairs), per_sample_sqnorm,
                            per_layer_sample_sqnorm, static_cast<double*>(ctx->sample_f64.ptr),
                            acc, accumulate, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "grad_stats: reduction launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_norm_test(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                                const adloco_stats_acc* acc, double eta, int64_t b_cur,
                                int64_t b_max, int32_t n_switch, int64_t b_cap, uint32_t flags,
                                adloco_norm_test_result* out, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!layers || n_layers < 1) return fail(ctx, ADLOCO_EINVAL, "norm_test: no layers");
  if (n_layers > kMaxLayers)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "norm_test: n_layers = %d exceeds %d", n_layers, kMaxLayers);
  if (!acc || !out) return fail(ctx, ADLOCO_EINVAL, "norm_test: NULL acc or out");
  if (!(eta > 0.0) || b_cur < 1 || b_max < 1 || n_switch < 1 || b_cap < 0 ||
      (flags & ~(ADLOCO_BIASED_VAR | ADLOCO_ALLOW_SHRINK)))
    return fail(ctx, ADLOCO_EINVAL, "norm_test: bad eta, b_cur, b_max, n_switch, b_cap or flags");
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the table is shared with grad_stats: same layer list -> no upload
  const int dtype = ctx->table_dtype >= 0 ? ctx->table_dtype : ADLOCO_BF16;
  // (same widths as the table of the last call: only the grad_sum pointers are refreshed)
  bool cached = ctx->layer_tab_host.size() == size_t(n_layers);
  if (cached)
    for (int l = 0; l < n_layers && cached; ++l) {
      const LayerDev& L = ctx->layer_tab_host[l];
      cached = L.grad_sum != nullptr && L.d_in == layers[l].d_in && L.d_out == layers[l].d_out &&
               layers[l].grad_sum != nullptr && (reinterpret_cast<uintptr_t>(layers[l].grad_sum) % 4) == 0;
    }
  if (cached) {
    // (written on every call: a graph replayed in between may have left other pointers in the table)
    for (int l = 0; l < n_layers; ++l) ctx->layer_tab_host[l].grad_sum = layers[l].grad_sum;
    int rc = upload_pointers(ctx, ctx->layer_tab_host, 2, st);
    if (rc) return rc;
  } else {
    int rc = prepare_tables(ctx, layers, n_layers, dtype, false, st);
    if (rc) return rc;
  }
  const size_t nblk = sqnorm_partials(ctx->layer_tab_host);
  int rc = ensure_scratch(ctx, ctx->red_f64, nblk * sizeof(double));
  if (rc) return rc;
  hipEvent_t ev = prof_begin(ctx, st);
  hipError_t e = launch_sqnorm(static_cast<const LayerDev*>(ctx->layer_tab.ptr), ctx->layer_tab_host,
                               static_cast<double*>(ctx->red_f64.ptr), ctx->dev_scalars, st);
  prof_end(ctx, kProfSqnorm, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "norm_test: reduction launch failed: %s", hipGetErrorString(e));
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->pinned, ctx->dev_scalars, sizeof(double),
                                       hipMemcpyDeviceToHost, st));
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->pinned + 2, acc, sizeof(adloco_stats_acc),
                                       hipMemcpyDeviceToHost, st));
  ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
  const double S2 = ctx->pinned[0];
  adloco_stats_acc h;
  std::memcpy(&h, ctx->pinned + 2, sizeof h);
  if (h.n_samples < 1)
    return fail(ctx, ADLOCO_ESTATE, "norm_test: accumulator holds no samples (n_samples = %lld)",
                (long long)h.n_samples);
  rc = adloco_norm_test_decide(h.sum_sample_sqnorm, S2, h.n_samples, eta, b_cur, b_max, n_switch,
                               b_cap, flags, out);
  if (rc) return fail(ctx, rc, "norm_test: decision rejected S1 = %g, S2 = %g", h.sum_sample_sqnorm, S2);
  return ADLOCO_OK;
}

// ---------------------------------------------------------------------------------------------
// Inner products c_i = <g_i, G> (Section 3.3.2)
// ---------------------------------------------------------------------------------------------
extern "C" int adloco_inner_products(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                                     int B, int T, int dtype, float* per_sample_ip,
                                     float* per_sample_sqnorm, adloco_ip_acc* acc, uint32_t flags,
                                     void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!layers || n_layers < 1) return fail(ctx, ADLOCO_EINVAL, "inner_products: no layers");
  if (n_layers > kMaxLayers)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "inner_products: n_layers = %d exceeds %d", n_layers, kMaxLayers);
  if (B < 1 || T < 1) return fail(ctx, ADLOCO_EINVAL, "inner_products: B = %d, T = %d must be >= 1", B, T);
  if (B > 0x7fff) return fail(ctx, ADLOCO_EUNSUPPORTED, "inner_products: B = %d exceeds 32767", B);
  if (dtype != ADLOCO_F32 && !is_16bit(dtype))
    return fail(ctx, ADLOCO_EUNSUPPORTED, "inner_products: dtype %d not supported", dtype);
  if (!per_sample_ip || !acc) return fail(ctx, ADLOCO_EINVAL, "inner_products: NULL output");
  if (reinterpret_cast<uintptr_t>(acc) % 8)
    return fail(ctx, ADLOCO_EINVAL, "inner_products: acc not 8-byte aligned");
  if (flags & ~ADLOCO_ACCUMULATE) return fail(ctx, ADLOCO_EINVAL, "inner_products: unknown flags");
  for (int l = 0; l < n_layers; ++l)
    if (!layers[l].grad_sum)
      return fail(ctx, ADLOCO_EINVAL, "inner_products: layer %d has no grad_sum (G is read here)", l);
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = prepare_tables(ctx, layers, n_layers, dtype, true, st);
  if (rc) return rc;
  rc = prepare_vector_table(ctx, B, T, st);
  if (rc) return rc;
  const std::vector<LayerDev>& tab = ctx->layer_tab_host;

  // ---- which blocks go through the tile GEMM, and its tile table
  if (ctx->ip_B != B || ctx->ip_T != T) {
    ++ctx->table_builds;
    std::vector<char> use(n_layers, 0);
    bool any = false;
    for (int l = 0; l < n_layers; ++l) {
      // the tile kernel counts an entry's chunks of 32 rows in 32 bits and addresses the rows of a
      // chunk with 32-bit byte offsets
      use[l] = tab[l].kind == ADLOCO_KIND_LINEAR && is_16bit(dtype) && tab[l].fast && T % 32 == 0 &&
               T <= (1 << 20) && tab[l].a_stride < (1 << 25) && tab[l].delta_stride < (1 << 25);
      any = any || use[l];
    }
    std::vector<int4> tiles;
    int group = 1;
    const int slots = any ? make_ip_tiles(tab, use, B, T, ctx->ip_group_tuning, tiles, group) : 0;
    if ((long long)slots * kNumXcd > 0x7fffffffLL)
      return fail(ctx, ADLOCO_EUNSUPPORTED, "inner_products: too many tiles for one launch");
    rc = ensure_scratch(ctx, ctx->ip_tab, std::max<size_t>(tiles.size(), 1) * sizeof(int4));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ip_tile_out,
                        std::max<size_t>(tiles.size(), 1) * group * 16 * sizeof(float));
    if (rc) return rc;
    rc = ensure_scratch(ctx, ctx->ip_flags, size_t(n_layers));
    if (rc) return rc;
    ctx->ip_B = ctx->ip_T = -1;
    if (!tiles.empty())
      ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ip_tab.ptr, tiles.data(), tiles.size() * sizeof(int4),
                                           hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->ip_flags.ptr, use.data(), size_t(n_layers),
                                         hipMemcpyHostToDevice, st));
    ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
    ctx->ip_use = std::move(use);
    ctx->ip_slots = slots;
    ctx->ip_group = group;
    ctx->ip_B = B;
    ctx->ip_T = T;
  }
  rc = ensure_scratch(ctx, ctx->ip_dot, size_t(n_layers) * B * sizeof(float));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->ip_sq, size_t(n_layers) * B * sizeof(float));
  if (rc) return rc;
  rc = ensure_scratch(ctx, ctx->sample_f64, size_t(B) * sizeof(double));
  if (rc) return rc;
  size_t part_doubles = 1;
  for (int l = 0; l < n_layers; ++l)
    if (tab[l].kind == ADLOCO_KIND_LINEAR && !ctx->ip_use[l])
      part_doubles = std::max(part_doubles, ip_generic_part_doubles(tab[l], B));
  rc = ensure_scratch(ctx, ctx->ip_part, part_doubles * sizeof(double));
  if (rc) return rc;

  const LayerDev* dl = static_cast<const LayerDev*>(ctx->layer_tab.ptr);
  float* dot = static_cast<float*>(ctx->ip_dot.ptr);
  float* sq = static_cast<float*>(ctx->ip_sq.ptr);
  hipEvent_t ev = prof_begin(ctx, st);
  hipError_t e = launch_ip_tiles(dl, ctx->ip_tab.ptr, ctx->ip_slots, T, ctx->ip_group, dtype,
                                 per_sample_sqnorm != nullptr,
                                 static_cast<float*>(ctx->ip_tile_out.ptr), st);
  for (int l = 0; l < n_layers && e == hipSuccess; ++l)
    if (tab[l].kind == ADLOCO_KIND_LINEAR && !ctx->ip_use[l])
      e = launch_ip_generic(tab[l], l, B, T, dtype, static_cast<double*>(ctx->ip_part.ptr), dot, sq, st);
  if (e == hipSuccess && !ctx->vec_host.empty())
    e = launch_vector_stats(dl, static_cast<const AuxDesc*>(ctx->vec_tab.ptr), int(ctx->vec_host.size()),
                            ctx->vec_blocks, ctx->vec_blocks2, B, T, dtype,
                            static_cast<float*>(ctx->aux_vec.ptr), sq, 1, 0, false, st);
  if (e == hipSuccess && !ctx->emb_host.empty())
    e = launch_embed_stats(dl, static_cast<const AuxDesc*>(ctx->emb_tab.ptr), int(ctx->emb_host.size()),
                           ctx->emb_blocks, B, T, dtype, static_cast<int*>(ctx->aux_perm.ptr),
                           static_cast<double*>(ctx->aux_part.ptr), sq, 1, st);
  if (e == hipSuccess)
    e = launch_ip_vector_table(dl, static_cast<const AuxDesc*>(ctx->vec_tab.ptr), int(ctx->vec_host.size()),
                               static_cast<const AuxDesc*>(ctx->emb_tab.ptr), int(ctx->emb_host.size()),
                               B, T, dtype, static_cast<const float*>(ctx->aux_vec.ptr), dot, st);
  if (e == hipSuccess)
    e = launch_ip_finalize(ctx->ip_tab.ptr, static_cast<const float*>(ctx->ip_tile_out.ptr),
                           (long long)ctx->ip_slots * kNumXcd, ctx->ip_group, dot, sq,
                           static_cast<const unsigned char*>(ctx->ip_flags.ptr), n_layers, B,
                           per_sample_ip, per_sample_sqnorm, static_cast<double*>(ctx->sample_f64.ptr),
                           acc, (flags & ADLOCO_ACCUMULATE) ? 1 : 0, st);
  prof_end(ctx, kProfIp, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "inner_products: launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_inner_product_test(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                                         const adloco_stats_acc* acc, const adloco_ip_acc* ip,
                                         double vartheta, double nu, int64_t b_cur, int64_t b_max,
                                         int32_t n_switch, int64_t b_cap, adloco_ip_test_result* out,
                                         void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (!acc || !ip || !out) return fail(ctx, ADLOCO_EINVAL, "inner_product_test: NULL acc, ip or out");
  // S2 exactly as the norm test forms it (also validates the layer list)
  adloco_norm_test_result nt;
  int rc = adloco_norm_test(ctx, layers, n_layers, acc, 1.0, b_cur, b_max, n_switch, b_cap, 0, &nt, stream);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  adloco_ip_acc h;
  ADLOCO_HIP_CHECK(ctx, hipMemcpyAsync(ctx->pinned + 4, ip, sizeof h, hipMemcpyDeviceToHost, st));
  ADLOCO_HIP_CHECK(ctx, hipStreamSynchronize(st));
  std::memcpy(&h, ctx->pinned + 4, sizeof h);
  if (h.n_samples != nt.n_samples)
    return fail(ctx, ADLOCO_ESTATE, "inner_product_test: the inner products cover %lld samples, the "
                "statistics %lld", (long long)h.n_samples, (long long)nt.n_samples);
  rc = adloco_inner_product_decide(nt.S1, nt.S2, h.sum_ip, h.sum_ip_sq, nt.n_samples, vartheta, nu,
                                   b_cur, b_max, n_switch, b_cap, out);
  if (rc) return fail(ctx, rc, "inner_product_test: decision rejected its arguments");
  return ADLOCO_OK;
}
