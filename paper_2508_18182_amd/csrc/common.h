// Internal definitions shared by the translation units of libadloco (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "adloco.h"
#include "adloco_internal.h"

namespace adloco {

// 16-bit element types: bf16 and IEEE half share every data path (they are moved as 16-bit lanes);
// only the MFMA instruction and the conversion to fp32 differ.
inline bool is_16bit(int dtype) { return dtype == ADLOCO_BF16 || dtype == ADLOCO_F16; }
typedef __attribute__((ext_vector_type(8))) __bf16 mfma_bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 mfma_f16x8;
typedef __attribute__((ext_vector_type(16))) float mfma_f32x16;
// One 32x32x16 MFMA on fragments held as bf16x8 bit patterns; F16 reinterprets them as halves.
template <bool F16>
__device__ __forceinline__ mfma_f32x16 mfma_32x32x16(mfma_bf16x8 a, mfma_bf16x8 b, mfma_f32x16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mfma_f16x8, a),
                                                  __builtin_bit_cast(mfma_f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// MI355X: 256 compute units in 8 XCDs; consecutive workgroup ids are dealt round-robin to
// the XCDs, each of which has its own L2.
constexpr int kNumXcd = 8;
constexpr int kNumCu = 256;

// Order of the ne x nc output tiles of one layer for the tile tables of the MFMA kernels: blocks of
// about 32 tiles (one round of an XCD's workgroups, which share that XCD's L2) whose shape streams
// the fewest distinct rows of a and delta -- as many tile columns as tile rows for square tiles,
// `aspect` times as many when a tile is `aspect` times as high as wide.  f(e, c) is called once per
// tile, e = tile row (d_out side), c = tile column (d_in side).
template <typename F>
inline void for_tiles_blocked(int ne, int nc, int aspect, F f) {
  const int per_round = kNumCu / kNumXcd;
  int nc_blk = 1;
  while (nc_blk * nc_blk < per_round * aspect) ++nc_blk;            // ~ sqrt(32 * aspect)
  nc_blk = nc_blk < nc ? nc_blk : nc;
  const int ne_blk = per_round / nc_blk > 1 ? per_round / nc_blk : 1;
  for (int eb = 0; eb < ne; eb += ne_blk)
    for (int cb = 0; cb < nc; cb += nc_blk)
      for (int e = eb; e < eb + ne_blk && e < ne; ++e)
        for (int c = cb; c < cb + nc_blk && c < nc; ++c) f(e, c);
}

// Device-side view of one linear layer (built on the host, uploaded once per change).
struct LayerDev {
  const void* a;
  const void* delta;
  float* grad_sum;
  long long a_stride;      // elements between token rows
  long long delta_stride;
  int d_in;
  int d_out;
  int fast;                // 1: rows 16-byte aligned and d % 8 == 0 for both operands
  int provided;            // 1: caller maintains grad_sum (no wgrad for this layer)
  int wg_blk_start;        // first workgroup of this layer in the wgrad launch
  int sq_blk_start;        // first workgroup of this layer in the squared-norm launch
  int kind;                // ADLOCO_KIND_* (0: linear weight)
  int delta_twin;          // vector blocks: first earlier vector block reading the same delta rows, or -1
  int a_twin;              // linear blocks: first earlier linear block reading the same activation rows
                           // (same a, stride, d_in) with the same d_out and delta stride, or -1
};

// One vector (bias / gain) or embedding-table block in the launches of its kernels.
struct AuxDesc {
  int layer;               // index into the layer table
  int slabs;               // column slabs of d_out (256 wide for vectors, 64 for tables)
  int blk_start;           // first workgroup in the (sample, slab) launch: B * slabs per block
  int blk_start2;          // first workgroup in the per-slab launch (vectors: column sums)
  long long vec_off;       // vectors: offset (floats) of this block's [B, d_out] sums
  long long vec_off_bias;  // vectors: >= 0: this gain block also forms the row sums of the bias block that
                           // reads the same delta, stored at this offset (that block has no workgroups of its own)
  long long perm_off;      // tables: offset (ints) of this block's [B, T] token order
  long long part_off;      // tables: offset (doubles) of this block's [B, slabs] slab totals
};

// One wave-wide direct load global -> LDS: lane l's 16 bytes at `src` land at LDS byte address
// `lds_addr` + 16*l (`lds_addr` is wave-uniform and travels in M0).  Written as inline assembly
// on purpose: the compiler orders the builtin form against every later LDS read with a full
// `s_waitcnt vmcnt(0)`, which would expose the whole memory latency in each pipeline step.  The
// caller therefore owns the ordering: its own s_waitcnt vmcnt(N) + workgroup barrier before any
// wave reads the bytes, and vmcnt(0) before compiler-visible memory traffic that must see them.
__device__ __forceinline__ void direct_load_lds16(const void* src, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "s"(lds_addr) : "m0");
}
// The same with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit
// byte offset per lane: a kernel that walks along its rows bumps the base on the scalar unit and
// keeps the lane offsets constant, so that no vector instruction is spent on addresses.
__device__ __forceinline__ void direct_load_lds16_s(unsigned lane_off, const void* base, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_off), "s"(base), "s"(lds_addr) : "m0");
}
// A wave-uniform pointer that the compiler may hold in vector registers, moved to scalar registers
// (the direct loads above take their base address there).
template <typename P> __device__ __forceinline__ const P* uniform_ptr(const P* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane(unsigned(v));
  const unsigned hi = __builtin_amdgcn_readfirstlane(unsigned(v >> 32));
  return reinterpret_cast<const P*>((unsigned long long)hi << 32 | lo);
}
// LDS byte address of a pointer into the workgroup's dynamic shared memory, as a scalar.
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)(const __attribute__((address_space(3))) unsigned char*)p);
}

struct Scratch {
  void* ptr = nullptr;
  size_t bytes = 0;
};

}  // namespace adloco

struct adloco_ctx {
  int device = 0;
  std::string err;
  // scratch
  adloco::Scratch partials;    // float  [n_units * pairs] Gram partial sums
  adloco::Scratch layer_tab;   // LayerDev[n_layers]
  adloco::Scratch red_f64;     // double partial sums of the streaming reductions
  adloco::Scratch sample_f64;  // double [B] per-sample totals
  adloco::Scratch order_tab;   // int [n_layers] launch order (heaviest first)
  adloco::Scratch group_tab;   // GramGroup[n_groups], int[n_groups] launch order of the groups; then, at
                               // single_off, the same with every linear layer in a group of its own
  int n_groups = 0;
  size_t single_off = 0;
  std::vector<adloco::LayerDev> layer_tab_host;  // last uploaded copy
  std::vector<int> order_host;
  adloco::Scratch job_tab;     // GramJob[] of the dual-tile Gram kernel
  int job_tab_nt = -1;         // number of row blocks the uploaded job table was built for
  int job_tab_n = 0;
  int gram_job_order = -1;     // where the jobs of two diagonal tile pairs go among a unit's jobs: 0 first,
                               // 1 last, 2 spread; -1: first for long sequences (T >= 768), last for short
                               // ones (measured: +9 % at T = 1024, -1.5 % at T = 512 for `first`)
  bool all_fast64 = false;     // every layer: aligned rows and widths that are multiples of 64
  adloco::Scratch wgx_tab;     // tile table of the fast gradient-sum kernel
  int wgx_slots = 0;           // tiles per XCD in that table (0: not built for this layer table)
  adloco::Scratch wgx_split;   // split tiles (layer, e0, c0, pieces) for the reduction
  adloco::Scratch wgx_part;    // partial tiles of the split contraction, 256 KiB each
  int wgx_n_split = 0;
  bool all_fast = false;       // every layer without a provided gradient: aligned, widths % 8 == 0
  int n_linear = 0;            // linear-weight blocks in the table (= entries of order_tab)
  // vector (bias / gain) and embedding-table blocks
  std::vector<adloco::AuxDesc> vec_host, emb_host;
  adloco::Scratch vec_tab, emb_tab;   // device copies of the two descriptor lists
  adloco::Scratch aux_vec;     // float  per vector block [B, d_out]
  adloco::Scratch aux_perm;    // int    per table block  [B, T]
  adloco::Scratch aux_part;    // double per table block  [B, slabs]
  int aux_B = -1, aux_T = -1;  // batch shape the descriptor lists were built for
  int vec_blocks = 0, vec_blocks2 = 0, emb_blocks = 0;
  // inner products (Section 3.3.2)
  adloco::Scratch ip_tab;      // int4 tile table of the inner-product form of the tile GEMM
  adloco::Scratch ip_tile_out; // float [tiles][ip_group][8 waves][2]
  adloco::Scratch ip_dot, ip_sq;   // float [n_layers][B] of the blocks outside the tile table
  adloco::Scratch ip_part;     // double scratch of the plain path
  adloco::Scratch ip_flags;    // unsigned char [n_layers]: 1 = block is in the tile table
  std::vector<char> ip_use;    // host copy of ip_flags
  int ip_slots = 0, ip_group = 1, ip_B = -1, ip_T = -1;
  int ip_group_tuning = 0;     // 0: cost model; else samples per tile entry
  // statistics by per-sample gradient tiles (explicit form fused with the gradient sum)
  adloco::Scratch ts_tab, ts_part_idx, ts_split, ts_ptiles, ts_out, ts_csr;
  int ts_slots = 0, ts_n_split = 0, ts_n_listed = 0, ts_idx_len = 0, ts_B = -1;
  bool ts_ok = false;          // every linear block is aligned bf16 with its gradient sum formed here
  int stats_variant = 1;       // 1: tile form when eligible; 0: Gram + gradient-sum kernels
  // the vector / table kernels (HBM-bound) can run next to the kernels of the linear blocks (MFMA /
  // L2-bound) on a second stream, forked from and joined to the caller's stream by events; measured,
  // that buys nothing (both go through the same L2), so it is off unless "overlap_aux" asks for it
  hipStream_t side_stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  int overlap_aux = 0;
  int wgrad_blocks = 0;        // workgroups of the wgrad launch for the uploaded table
  int table_dtype = -1;        // dtype the uploaded table was built for
  int table_inputs = -1;       // 1: the table was built by a call that reads a and delta
  int table_builds = 0;        // how often a shape-dependent table has been (re)built
  long long max_lin_stride = 0;  // widest row stride (elements) among the linear blocks of the table
  double* pinned = nullptr;    // 8 doubles of pinned host memory (read-back of the tests' sums)
  double* dev_scalars = nullptr;  // 4 doubles on the device (S2, ...)
  // optional per-kernel event timing ("profile" knob)
  struct ProfRec { int kernel; hipEvent_t start, stop; };
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> prof_free;
  int profile = 0;
  // tuning
  int gram_variant = 1;        // 1: dual-tile kernel when eligible, 0: always the generic one
  int wgrad_variant = 2;       // 2: 256x256 fast kernel when eligible; 1/0: 128x128 kernel (LDS transpose reads / gathers)
  int stream_blocks_per_cu = 0;   // resident workgroups per CU of the streaming kernels; 0: automatic
  int stream_variant = 0;
};

namespace adloco {

inline int fail(adloco_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  return code;
}

#define ADLOCO_HIP_CHECK(ctx, expr)                                                      \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return adloco::fail((ctx), ADLOCO_EHIP, "%s failed: %s (%s:%d)", #expr,            \
                          hipGetErrorString(e_), __FILE__, __LINE__);                    \
  } while (0)

// Event timing of one kernel launch when ctx->profile is set (no-ops otherwise).
enum ProfKernel { kProfGram = 0, kProfWgrad, kProfFinalize, kProfSqnorm, kProfOuter, kProfMerge,
                  kProfVecTab, kProfInner, kProfIp, kProfTileStats, kProfCount };
hipEvent_t prof_begin(adloco_ctx* ctx, hipStream_t st);
void prof_end(adloco_ctx* ctx, int kernel, hipEvent_t start, hipStream_t st);

// Grow-only scratch buffer.  Growing frees the old block, which waits for the device.
int ensure_scratch(adloco_ctx* ctx, Scratch& s, size_t bytes);

// Kernel launchers (defined next to their kernels).  All return a hipError_t from the launch.
struct GramLaunch {
  const LayerDev* layers;   // device table
  const int* order;         // device: launch order of layer indices, heaviest first
  int n_layers, B, T;
  float* partials;          // [n_layers][B][n_pairs]
  int n_pairs;              // tile pairs per (layer, sample)
  int tile;                 // T-tile edge used by the kernel
  int dtype = ADLOCO_BF16;  // element type of a and delta
};
// Linear layers that read the same activation tensor (q / k / v, gate / up of a transformer block):
// their A A^T is one and the same, so the dual-tile Gram kernel forms it once per group and runs the
// members' delta delta^T contractions against it one after the other.
constexpr int kGramGroupMax = 4;
struct GramGroup {
  int n;                      // members, 1 .. kGramGroupMax
  int layer[kGramGroupMax];   // indices into the layer table; all share a, d_in, d_out and the strides
};
// One workgroup of the dual-tile Gram kernel: up to two 128x128 tile pairs (A-block, B-block)
// drawn from at most three distinct 128-row blocks.
struct GramJob {
  int blk[3];      // distinct row blocks to stage (unused entries repeat blk[0])
  int nblk;        // 2 or 3 (1 when T fits one block)
  int sa[2], sb[2];  // per tile pair: which staged block supplies the rows / the columns
  float w[2];      // 1 on the diagonal, 2 off it (symmetry), 0 for an absent second pair
};
std::vector<GramJob> make_gram_jobs(int nt, int order);
int gram_tile_edge(int dtype, int variant);
// g.order: launch order of GROUP indices; g.n_layers: number of groups; g.n_pairs: partial sums per
// (layer, sample) = gram_dual_parts(n_jobs)
hipError_t launch_gram_bf16_dual(const GramLaunch& g, const GramGroup* groups, const GramJob* jobs,
                                 int n_jobs, int variant, hipStream_t st);
int gram_dual_parts(int n_jobs);
hipError_t launch_gram_bf16(const GramLaunch& g, int variant, hipStream_t st);
hipError_t launch_gram_f32(const GramLaunch& g, hipStream_t st);
int wgrad_tile_edge(int dtype);
int make_wgrad_x_tiles(const std::vector<LayerDev>& layers, std::vector<int4>& out,
                       std::vector<int4>& split_tiles, int& n_pieces);
hipError_t launch_wgrad_x(const LayerDev* layers, const void* tiles, int slots,
                          const void* split_tiles, int n_split, float* partials, long long rows,
                          int accumulate, int dtype, hipStream_t st);
hipError_t launch_wgrad(const LayerDev* layers, int n_layers, int n_blocks, long long rows,
                        int dtype, int accumulate, int variant, hipStream_t st);
hipError_t launch_finalize_stats(const float* partials, int n_layers, int B, int n_pairs,
                                 float* per_sample, float* per_layer_sample, double* sample_f64,
                                 adloco_stats_acc* acc, int accumulate, hipStream_t st);
int vector_table_slab();
int embed_table_slab();
hipError_t launch_vector_stats(const LayerDev* layers, const AuxDesc* tab, int n_tab,
                               int blocks_rowsum, int blocks_colsum, int B, int T, int dtype,
                               float* vec, float* partials, int n_pairs, int accumulate,
                               bool write_grad_sum, hipStream_t st);
int make_ip_tiles(const std::vector<LayerDev>& layers, const std::vector<char>& use, int B, int T,
                  int forced_group, std::vector<int4>& out, int& group);
hipError_t launch_ip_tiles(const LayerDev* layers, const void* tiles, int slots, int T, int group,
                           int dtype, bool want_sq, float* ip_out, hipStream_t st);
int make_stats_tiles(const std::vector<LayerDev>& layers, const std::vector<char>& use, int B,
                     std::vector<int4>& out, std::vector<int>& part, std::vector<int4>& split,
                     std::vector<int>& lay, std::vector<int>& ptr, std::vector<int>& idx,
                     int& n_pieces);
hipError_t launch_stats_tiles(const LayerDev* layers, const void* tiles, const int* part, int slots,
                              const void* split, int n_split, float* partial_tiles, int B, int T,
                              int dtype, int accumulate, float* tile_out, const int* lay, const int* ptr,
                              const int* idx, int n_listed, float* partials, int n_pairs,
                              hipStream_t st);
hipError_t launch_ip_generic(const LayerDev& L, int layer, int B, int T, int dtype, double* part,
                             float* dot, float* sq, hipStream_t st);
size_t ip_generic_part_doubles(const LayerDev& L, int B);
hipError_t launch_ip_vector_table(const LayerDev* layers, const AuxDesc* vec_tab, int n_vec,
                                  const AuxDesc* emb_tab, int n_emb, int B, int T, int dtype,
                                  const float* vec, float* dot, hipStream_t st);
hipError_t launch_ip_finalize(const void* tiles, const float* tile_out, long long n_tiles, int group,
                              const float* dot, const float* sq, const unsigned char* in_tiles,
                              int n_layers, int B, float* per_sample_ip, float* per_sample_sq,
                              double* sample_f64, adloco_ip_acc* acc, int accumulate, hipStream_t st);
hipError_t launch_embed_stats(const LayerDev* layers, const AuxDesc* tab, int n_tab, int blocks_rows,
                              int B, int T, int dtype, int* perm, double* part, float* partials,
                              int n_pairs, hipStream_t st);
// sum_l ||grad_sum_l||^2 -> *out (device double); partial buffer sized by sqnorm_partials().
int sqnorm_chunk();
size_t sqnorm_partials(const std::vector<LayerDev>& host_layers);
hipError_t launch_sqnorm(const LayerDev* layers, const std::vector<LayerDev>& host_layers,
                         double* partial, double* out, hipStream_t st);
// The same on a device table of n_layers blocks whose sq_blk_start fields add up to nblk workgroups.
hipError_t launch_sqnorm_table(const LayerDev* layers, int n_layers, size_t nblk, double* partial,
                               double* out, hipStream_t st);
// Looks up, for the context's device, the address of the file-scope device array that serves
// adloco_norm_test_noalloc (called once per context by adloco_create, with the device current).
int no_alloc_init(adloco_ctx* ctx);

}  // namespace adloco
