// Per-sample gradient squared norms by the Gram identity
//   || sum_t delta_t a_t^T ||_F^2  =  sum_{t,t'} (a_t . a_t') (delta_t . delta_t')
// i.e. n_i = < A_i A_i^T , D_i D_i^T >_F with A_i [T, d_in], D_i [T, d_out] the token rows of
// sample i.  It gives ||g_i||^2 of the per-sample gradients that eq. 1 averages (needed by the
// variance of Section 3.3.1) without forming any d_out x d_in matrix.
//
// Work decomposition: the T x T Gram matrices are symmetric, so only tile pairs (p <= q) of
// T-tiles are computed; off-diagonal pairs count twice.  One workgroup handles one
// (layer, sample, tile pair): it accumulates the (p,q) tile of A A^T over d_in and the same
// tile of D D^T over d_out in two sets of MFMA accumulators that share one register layout,
// multiplies them element-wise in registers and reduces to one float.
#include "common.h"
#include <algorithm>
#include <cstdlib>
#include <type_traits>

namespace adloco {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct GramArgs {
  const LayerDev* layers;
  const int* order;
  float* partials;
  int n_layers, B, T, n_pairs, nt, units_padded;
};

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Workgroup id -> (layer, sample, tile pair).  Consecutive workgroup ids go to different XCDs,
// so the id is split as (slot, xcd): all tile pairs of one sample run on one XCD, next to each
// other in launch order, and re-read that sample's rows from the XCD's L2.
__device__ __forceinline__ bool decode_block(const GramArgs& g, int& layer, int& sample, int& p,
                                             int& q, int& pair) {
  const int bid = blockIdx.x;
  const int xcd = bid % kNumXcd;
  const int slot = bid / kNumXcd;
  pair = slot % g.n_pairs;
  const int u = (slot / g.n_pairs) * kNumXcd + xcd;
  if (u >= g.n_layers * g.B) return false;
  layer = g.order[u / g.B];
  sample = u % g.B;
  // triangular decode: pairs are listed row by row, (0,0),(0,1)..(0,nt-1),(1,1)...
  int rem = pair, row = 0, len = g.nt;
  while (rem >= len) { rem -= len; ++row; --len; }
  p = row;
  q = row + rem;
  return true;
}

// ---------------------------------------------------------------------------------------
// bf16 inputs, MFMA 32x32x16, fp32 accumulation.
//   workgroup: 256 threads = 4 waves in a 2x2 arrangement over a 128x128 tile of the Gram
//   matrices; each wave owns 64x64 = 2x2 MFMA blocks for A A^T and again for D D^T.
//   LDS: two stages of [p rows | q rows] x 64 bf16 (128-byte rows), 16-byte chunks XOR-swizzled
//   by the row so that both the row-wise writes and the fragment reads spread over the banks.
// ---------------------------------------------------------------------------------------
constexpr int kTile = 128;
constexpr int kKc = 64;                               // bf16 elements per staged row
constexpr int kStageBytes = 2 * kTile * kKc * 2;      // p and q rows: 32 KiB
constexpr int kGramLds = 2 * kStageBytes;             // two stages: 64 KiB

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row ^ (row >> 3)) & 7); }

struct ChunkRegs { u32x4 v[8]; };

// Load the 16-byte pieces this thread stages for k-chunk `c` of the concatenated operand
// sequence [a chunks | delta chunks].  Piece e = tid + 256*it: tile (e>>10), row ((e&1023)>>3),
// 16-byte chunk (e&7).  Rows beyond T and columns beyond d read as zero.
__device__ __forceinline__ void load_chunk(const LayerDev& L, int T, long long samp_row0, int p,
                                           int q, int c, int nka, ChunkRegs& r) {
  const bool is_a = c < nka;
  const unsigned short* base = reinterpret_cast<const unsigned short*>(is_a ? L.a : L.delta);
  const long long stride = is_a ? L.a_stride : L.delta_stride;
  const int d = is_a ? L.d_in : L.d_out;
  const int k0 = (is_a ? c : c - nka) * kKc;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int e = threadIdx.x + 256 * it;
    const int tile = e >> 10;
    const int row = (e & 1023) >> 3;
    const int ch = e & 7;
    const int t = (tile ? q : p) * kTile + row;
    const int k = k0 + ch * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (t < T && k < d) {
      const unsigned short* src = base + (samp_row0 + t) * stride + k;
      if (L.fast) {
        v = *reinterpret_cast<const u32x4*>(src);
      } else {
        unsigned short h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = (k + j < d) ? src[j] : (unsigned short)0;
        v[0] = h[0] | (unsigned(h[1]) << 16);
        v[1] = h[2] | (unsigned(h[3]) << 16);
        v[2] = h[4] | (unsigned(h[5]) << 16);
        v[3] = h[6] | (unsigned(h[7]) << 16);
      }
    }
    r.v[it] = v;
  }
}

__device__ __forceinline__ void store_chunk(unsigned char* stage, const ChunkRegs& r) {
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int e = threadIdx.x + 256 * it;
    const int tile = e >> 10;
    const int row = (e & 1023) >> 3;
    const int ch = e & 7;
    *reinterpret_cast<u32x4*>(stage + tile * (kTile * kKc * 2) + row * (kKc * 2) + swz(row, ch) * 16) =
        r.v[it];
  }
}

__device__ __forceinline__ bf16x8 read_frag(const unsigned char* tile_base, int row, int chunk) {
  u32x4 v = *reinterpret_cast<const u32x4*>(tile_base + row * (kKc * 2) + swz(row, chunk) * 16);
  return __builtin_bit_cast(bf16x8, v);
}

template <bool F16>
__device__ __forceinline__ void mma_stage(const unsigned char* stage, int wm, int wn, int lane,
                                          f32x16 (&acc)[2][2]) {
  const unsigned char* ptile = stage;
  const unsigned char* qtile = stage + kTile * kKc * 2;
  const int r32 = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < kKc / 16; ++ks) {
    bf16x8 fa[2], fb[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) fa[m] = read_frag(ptile, wm * 64 + m * 32 + r32, ks * 2 + kg);
#pragma unroll
    for (int n = 0; n < 2; ++n) fb[n] = read_frag(qtile, wn * 64 + n * 32 + r32, ks * 2 + kg);
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int n = 0; n < 2; ++n)
        acc[m][n] = mfma_32x32x16<F16>(fa[m], fb[n], acc[m][n]);
  }
}

template <bool F16>
__global__ __launch_bounds__(256, 2) void gram_bf16_kernel(GramArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  int layer, sample, p, q, pair;
  if (!decode_block(g, layer, sample, p, q, pair)) return;
  const LayerDev L = g.layers[layer];
  const int T = g.T;
  const long long samp_row0 = (long long)sample * T;
  const int nka = (L.d_in + kKc - 1) / kKc;
  const int nkd = (L.d_out + kKc - 1) / kKc;
  const int nk = nka + nkd;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16 acc_a[2][2], acc_d[2][2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) { acc_a[m][n][j] = 0.f; acc_d[m][n][j] = 0.f; }

  ChunkRegs regs;
  load_chunk(L, T, samp_row0, p, q, 0, nka, regs);
  store_chunk(lds, regs);
  __syncthreads();
  // One pipeline over the concatenated k-chunks of a and delta: while the MFMAs consume stage
  // c&1, the next chunk travels global -> registers -> the other stage.
  auto step = [&](int c, f32x16 (&acc)[2][2]) {
    unsigned char* cur = lds + (c & 1) * kStageBytes;
    unsigned char* nxt = lds + ((c + 1) & 1) * kStageBytes;
    const bool more = c + 1 < nk;
    if (more) load_chunk(L, T, samp_row0, p, q, c + 1, nka, regs);
    mma_stage<F16>(cur, wm, wn, lane, acc);
    if (more) store_chunk(nxt, regs);
    __syncthreads();
  };
  int c = 0;
  for (; c < nka; ++c) step(c, acc_a);
  for (; c < nk; ++c) step(c, acc_d);

  float s = 0.f;
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) s += acc_a[m][n][j] * acc_d[m][n][j];
  s = wave_sum_f32(s);
  float* red = reinterpret_cast<float*>(lds);   // staging is idle after the last barrier
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    g.partials[(size_t(layer) * g.B + sample) * g.n_pairs + pair] = (p == q) ? tot : 2.f * tot;
  }
}

// ---------------------------------------------------------------------------------------
// bf16 fast path ("dual-tile" kernel), used when every operand row is 16-byte aligned and every
// width is a multiple of 64.
//   workgroup: 512 threads = 8 waves = two groups of four; each group owns one 128x128 tile pair
//   of one job.  A job is a pair of tile pairs that share a row block, so that at most three
//   distinct 128-row blocks have to be staged: less L2 and LDS-write traffic per MFMA than one
//   tile pair per workgroup, with the same executed flops.
//   Staging: global -> LDS directly (16 bytes per lane, no registers in between), three stages
//   of (3 blocks x 128 rows x 64 bf16), or four stages of 36 KiB for a job that has only two
//   distinct blocks (most jobs of a short sequence: 4 of the 5 at T = 512), which then has one
//   more chunk in flight.  One workgroup barrier per k-chunk, placed in the middle
//   of the chunk: by then every wave's loads of the next chunk have landed and every wave has
//   finished with the previous chunk's stage, so the chunk after next is requested right there
//   and the fragment reads never drain across a chunk boundary.
//   Fragments for the next k-step are read from LDS while the MFMAs of the current one run.
//   A tile pair on the diagonal is symmetric: three of its four 64x64 wave tiles are computed,
//   and the two of them that lie on the diagonal three of their four 32x32 blocks.
// ---------------------------------------------------------------------------------------
constexpr int kDualStageRows = 3 * kTile;
constexpr int kDualStage = kDualStageRows * kKc * 2;          // 48 KiB
constexpr int kDualStages = 3;
constexpr int kDualLds = kDualStages * kDualStage;            // 144 KiB

struct GramDualArgs {
  const LayerDev* layers;
  const GramGroup* groups;
  const int* order;         // launch order of group indices
  const GramJob* jobs;
  float* partials;          // [layer][sample][n_jobs * 8]: one partial sum per job and wave
  int n_groups, B, T, n_jobs, units_padded;
};

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 0xf) | ((N >> 4) << 14));
}

__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// What one wave of a group of four does on a 128 x 128 tile pair: the 32-row fragments it reads per
// k-step (frag_block: which 32-row block of the tile; from_b: of the pair's column side) and the
// 32 x 32 blocks it accumulates, block b = fragment fa(b) (rows) x fragment fb(b) (columns).
struct GramShapeOff {        // off-diagonal pair: wave (wq / 2, wq % 2) owns 2 x 2 blocks
  static constexpr int NF = 4, NB = 4;
  __device__ static constexpr bool from_b(int f) { return f >= 2; }
  __device__ static constexpr int frag_block(int f, int wq) { return f < 2 ? (wq >> 1) * 2 + f : (wq & 1) * 2 + (f - 2); }
  __device__ static constexpr int fa(int b) { return b >> 1; }
  __device__ static constexpr int fb(int b) { return 2 + (b & 1); }
  __device__ static constexpr int row_block(int b, int wq) { return (wq >> 1) * 2 + (b >> 1); }
  __device__ static constexpr int col_block(int b, int wq) { return (wq & 1) * 2 + (b & 1); }
  __device__ static constexpr float weight(int) { return 1.f; }
};
// Pair on the diagonal, upper blocks (i <= j) of the 4 x 4 block grid:
//   wave 0: (0,0) (0,1) (1,1)   wave 1: (0,2) (1,2) (2,2)   wave 2: (0,3) (1,3) (2,3)   wave 3: (3,3)
template <int W> struct GramShapeDiag {
  static constexpr int NF = W == 0 ? 2 : W == 1 ? 3 : W == 2 ? 4 : 1;
  static constexpr int NB = W == 3 ? 1 : 3;
  __device__ static constexpr bool from_b(int) { return false; }
  __device__ static constexpr int frag_block(int f, int) { return W == 3 ? 3 : f; }
  __device__ static constexpr int row_block(int b, int) { return W == 0 ? (b == 2 ? 1 : 0) : W == 3 ? 3 : b; }
  __device__ static constexpr int col_block(int b, int) { return W == 0 ? (b == 0 ? 0 : 1) : W == 3 ? 3 : W + 1; }
  __device__ static constexpr int fa(int b) { return W == 3 ? 0 : row_block(b, 0); }
  __device__ static constexpr int fb(int b) { return W == 3 ? 0 : col_block(b, 0); }
  __device__ static constexpr float weight(int b) { return row_block(b, 0) == col_block(b, 0) ? 1.f : 2.f; }
};

// MAXM: the largest group of layers sharing their activation tensor in the launch (1: none share)
template <bool F16, int MAXM>
__global__ __launch_bounds__(512, 1) void gram_bf16_dual_kernel(GramDualArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int bid = blockIdx.x;
  const int xcd = bid % kNumXcd;
  const int slot = bid / kNumXcd;
  const int job = slot % g.n_jobs;
  const int u = (slot / g.n_jobs) * kNumXcd + xcd;
  if (u >= g.n_groups * g.B) return;
  // the unit: one sample of a group of layers that share their activation tensor (mostly a group of one)
  const int gi = __builtin_amdgcn_readfirstlane(g.order[u / g.B]);
  const GramGroup G = g.groups[gi];
  const int n_mem = MAXM == 1 ? 1 : __builtin_amdgcn_readfirstlane(G.n);
  const int sample = u % g.B;
  const LayerDev L = g.layers[__builtin_amdgcn_readfirstlane(G.layer[0])];   // a, widths and strides are the group's
  const GramJob J = g.jobs[job];
  const int nblk = __builtin_amdgcn_readfirstlane(J.nblk);
  const int T = g.T;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int grp = wave >> 2;                         // which tile pair of the job
  const int slot_a = grp ? J.sa[1] : J.sa[0];
  const int slot_b = grp ? J.sb[1] : J.sb[0];
  const int nka = L.d_in / kKc, nkd = L.d_out / kKc, nk = nka + n_mem * nkd;
  constexpr int ROWB = kKc * 2;

  // ---- direct global->LDS loads.  One wave instruction fills 8 rows (1 KiB): lane -> row lane/8,
  // 16-byte position lane%8, which receives chunk position ^ f(row) of that row.  Wave w covers
  // row groups w and w+8 of each staged block.  Rows beyond T re-read row T-1 (their products
  // are masked in the epilogue).
  const int ld_row = wave * 8 + (lane >> 3);         // row within the block for i = 0; +64 for i = 1
  const int ld_col = swz(ld_row, lane & 7) * 8;      // element offset within the 64-wide chunk
  // Address = (sample's first row + chunk's first column: wave-uniform, scalar registers) + (row
  // within the sample, position within the chunk: a 32-bit byte offset per lane, computed once for
  // each operand; the host keeps T * row stride below 2^31 elements).
  int t_row[3][2];
#pragma unroll
  for (int s = 0; s < 3; ++s)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int t = J.blk[s < nblk ? s : 0] * kTile + ld_row + 64 * i;
      t_row[s][i] = t < T ? t : T - 1;
    }
  unsigned off_pa[3][2], off_pd[3][2];
#pragma unroll
  for (int s = 0; s < 3; ++s)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      off_pa[s][i] = unsigned((long long)t_row[s][i] * L.a_stride + ld_col) * 2u;
      off_pd[s][i] = unsigned((long long)t_row[s][i] * L.delta_stride + ld_col) * 2u;
    }
  const unsigned short* const samp_a =
      reinterpret_cast<const unsigned short*>(L.a) + (long long)sample * T * L.a_stride;
  // delta of the member whose chunks are being requested (the members' chunks follow each other; the
  // next member's tensor is looked up when the requests cross over: once per member, not per chunk)
  const long long samp_off_d = (long long)sample * T * L.delta_stride;
  const unsigned short* cur_d = reinterpret_cast<const unsigned short*>(L.delta) + samp_off_d;
  int seg_m = 0, seg_end = nka + nkd;
  const unsigned lds_base = lds_address(lds);
  // A job with three row blocks runs three stages of 48 KiB, one with at most two blocks four stages
  // of 36 KiB (32 used): one more chunk in flight out of the same 144 KiB.
  const int n_st = nblk == 3 ? 3 : 4;
  const unsigned st_bytes = nblk == 3 ? unsigned(kDualStage) : unsigned(kDualLds / 4);
  // stage indices are carried along (no division in the loop): chunk c lives in stage c mod n_st
  auto issue_loads = [&](int c, int st) {
    const unsigned stage = lds_base + unsigned(st) * st_bytes;
    if (c < nka) {
      const unsigned short* base = uniform_ptr(samp_a + c * kKc);
#pragma unroll
      for (int s = 0; s < 3; ++s)
        if (s < nblk) {
#pragma unroll
          for (int i = 0; i < 2; ++i)
            direct_load_lds16_s(off_pa[s][i], base, stage + (s * kTile + (wave + 8 * i) * 8) * ROWB);
        }
    } else {
      if (MAXM > 1 && c >= seg_end) {          // (requests come in the order of the chunks)
        ++seg_m;
        seg_end += nkd;
        const int lm = __builtin_amdgcn_readfirstlane(g.groups[gi].layer[seg_m]);
        cur_d = reinterpret_cast<const unsigned short*>(g.layers[lm].delta) + samp_off_d;
      }
      const unsigned short* base = uniform_ptr(cur_d + (c - (seg_end - nkd)) * kKc);
#pragma unroll
      for (int s = 0; s < 3; ++s)
        if (s < nblk) {
#pragma unroll
          for (int i = 0; i < 2; ++i)
            direct_load_lds16_s(off_pd[s][i], base, stage + (s * kTile + (wave + 8 * i) * 8) * ROWB);
        }
    }
  };

  // ---- fragment addressing
  const int r32 = lane & 31, kg = lane >> 5;
  const bool diag = slot_a == slot_b;       // both sides of the tile pair are the same row block
  const int wq = wave & 3;                  // this wave's place in its group of four
  typedef __attribute__((address_space(3))) const u32x4* lds_v4;

  f32x16 acc_a[4], acc_d[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) { acc_a[b][j] = 0.f; acc_d[b][j] = 0.f; }

  // ---- prologue: chunks 0 .. n_st-2 in flight, chunk 0 landed for everybody (a wave issues
  // 2 * nblk loads per chunk)
  issue_loads(0, 0);
  if (nk > 1) issue_loads(1, 1);
  if (n_st == 4 && nk > 2) issue_loads(2, 2);
  if (nblk == 3) {
    if (nk > 1) wait_vmcnt<6>(); else wait_vmcnt<0>();
  } else if (nblk == 2) {
    if (nk > 2) wait_vmcnt<8>(); else if (nk > 1) wait_vmcnt<4>(); else wait_vmcnt<0>();
  } else {
    if (nk > 2) wait_vmcnt<4>(); else if (nk > 1) wait_vmcnt<2>(); else wait_vmcnt<0>();
  }
  wg_barrier();

  const int blk_a = J.blk[slot_a], blk_b = J.blk[slot_b];
  // (the grouped form is launched only for T a multiple of the tile edge: no ragged block there; with the
  // masked epilogue inside its member loop the kernel runs out of scalar registers)
  const bool whole = MAXM > 1 ? true : ((blk_a + 1) * kTile <= T && (blk_b + 1) * kTile <= T);
  // One wave's share of a tile pair.  `shape` (a GramShape) lists the 32-row fragments the wave reads
  // per k-step and the 32 x 32 blocks it accumulates from them; every wave of the workgroup passes
  // the same waits, barriers and loads whatever its shape.
  auto run = [&](auto shape) {
    typedef decltype(shape) S;
    constexpr int NF = S::NF, NB = S::NB;
    // byte offset within a stage of this lane's 16 bytes for every (k-step, fragment): computed
    // once, so that a k-step spends no vector instruction on addresses
    unsigned pre[4][NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const int row = (S::from_b(f) ? slot_b : slot_a) * kTile + S::frag_block(f, wq) * 32 + r32;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) pre[ks][f] = unsigned(row * ROWB + ((ks * 2 + kg) ^ swz(row, 0)) * 16);
    }
    auto read_frags = [&](int st, int ks, bf16x8 (&f)[NF]) {
      const unsigned stage = lds_base + unsigned(st) * st_bytes;
#pragma unroll
      for (int i = 0; i < NF; ++i) f[i] = __builtin_bit_cast(bf16x8, *(lds_v4)(size_t)(stage + pre[ks][i]));
    };
    auto mfmas = [&](const bf16x8 (&f)[NF], f32x16 (&acc)[4]) {
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[b] = mfma_32x32x16<F16>(f[S::fa(b)], f[S::fb(b)], acc[b]);
      // issue order: MFMA, LDS read, MFMA, LDS read, ...
#pragma unroll
      for (int i = 0; i < (NB < NF ? NB : NF); ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if (NF > NB) __builtin_amdgcn_sched_group_barrier(0x100, NF - NB, 0);
      if (NB > NF) __builtin_amdgcn_sched_group_barrier(0x008, NB - NF, 0);
    };
    bf16x8 fr[2][NF];
    read_frags(0, 0, fr[0]);
    int st_cur = 0, st_prev = n_st - 1;            // stages of chunk c and of chunk c-1
    const int ahead = n_st - 1;                    // the chunk requested at chunk c's barrier is c + ahead
    auto chunk_step = [&](int c, f32x16 (&acc)[4]) {
      const int st_next = st_cur + 1 == n_st ? 0 : st_cur + 1;
      // k-step 0
      read_frags(st_cur, 1, fr[1]);
      mfmas(fr[0], acc);
      // k-step 1, with the barrier of this chunk in front of it
      if (c + 1 < nk) {
        // my share of chunk c+1 has landed (with four stages chunk c+2 may still be in flight) ...
        if (n_st == 4 && c + 2 < nk) {
          if (nblk == 2) wait_vmcnt<4>(); else wait_vmcnt<2>();
        } else {
          wait_vmcnt<0>();
        }
        wg_barrier();           // ... and so has everybody's; the stage of chunk c-1 is free
        if (c + ahead < nk) issue_loads(c + ahead, st_prev);
      }
      read_frags(st_cur, 2, fr[0]);
      mfmas(fr[1], acc);
      // k-step 2
      read_frags(st_cur, 3, fr[1]);
      mfmas(fr[0], acc);
      // k-step 3: fragments of the next chunk's first k-step (after the last chunk: a harmless
      // re-read of this chunk, so that the reads stay interleaved with the MFMAs)
      read_frags(c + 1 < nk ? st_next : st_cur, 0, fr[0]);
      mfmas(fr[1], acc);
      st_prev = st_cur;
      st_cur = st_next;
    };
    int c = 0;
    for (; c < nka; ++c) chunk_step(c, acc_a);
    // A A^T of this wave's blocks is complete; the members' D D^T follow one after the other
    const float w_pair = grp ? J.w[1] : J.w[0];
    for (int m = 0; m < n_mem; ++m) {
      for (const int cend = nka + (m + 1) * nkd; c < cend; ++c) chunk_step(c, acc_d);
      // ---- < A A^T , D D^T > over this wave's blocks, masked beyond T
      float s = 0.f;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float sb = 0.f;
        if (whole) {
#pragma unroll
          for (int j = 0; j < 16; ++j) sb += acc_a[b][j] * acc_d[b][j];
        } else {
          const int col = blk_b * kTile + S::col_block(b, wq) * 32 + r32;
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int row = blk_a * kTile + S::row_block(b, wq) * 32 + (j >> 2) * 8 + kg * 4 + (j & 3);
            if (row < T && col < T) sb += acc_a[b][j] * acc_d[b][j];
          }
        }
        s += sb * S::weight(b);
#pragma unroll
        for (int j = 0; j < 16; ++j) acc_d[b][j] = 0.f;
      }
      s = wave_sum_f32(s) * w_pair;
      const int layer = __builtin_amdgcn_readfirstlane(g.groups[gi].layer[m]);
      if (lane == 0)
        g.partials[((size_t(layer) * g.B + sample) * g.n_jobs + job) * 8 + wave] = s;
    }
  };
  // An off-diagonal tile pair: 2 x 2 waves of 64 x 64.  A tile pair on the diagonal is symmetric: its
  // ten upper 32 x 32 blocks (i <= j) are dealt 3, 3, 3, 1 to the four waves, blocks off the diagonal
  // count twice.
  if (!diag) {
    run(GramShapeOff{});
  } else {
    switch (wq) {
      case 0: run(GramShapeDiag<0>{}); break;
      case 1: run(GramShapeDiag<1>{}); break;
      case 2: run(GramShapeDiag<2>{}); break;
      default: run(GramShapeDiag<3>{}); break;
    }
  }
}

// ---------------------------------------------------------------------------------------
// fp32 inputs: plain FMA path (correctness path for fp32 activations; not MFMA).
//   workgroup: 256 threads over a 32x32 tile pair, 2x2 entries per thread.
// ---------------------------------------------------------------------------------------
constexpr int kTileF = 32;
constexpr int kKcF = 32;

__global__ __launch_bounds__(256) void gram_f32_kernel(GramArgs g) {
  __shared__ float sp[kTileF][kKcF + 1];
  __shared__ float sq[kTileF][kKcF + 1];
  __shared__ float red[4];
  int layer, sample, p, q, pair;
  if (!decode_block(g, layer, sample, p, q, pair)) return;
  const LayerDev L = g.layers[layer];
  const int T = g.T;
  const long long samp_row0 = (long long)sample * T;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;   // entries (ty*2+{0,1}, tx*2+{0,1})
  float prod[2][2][2];   // [operand][i][j]
#pragma unroll
  for (int o = 0; o < 2; ++o)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) prod[o][i][j] = 0.f;
#pragma unroll
  for (int o = 0; o < 2; ++o) {
    const float* base = reinterpret_cast<const float*>(o == 0 ? L.a : L.delta);
    const long long stride = o == 0 ? L.a_stride : L.delta_stride;
    const int d = o == 0 ? L.d_in : L.d_out;
    for (int k0 = 0; k0 < d; k0 += kKcF) {
      for (int e = threadIdx.x; e < kTileF * kKcF; e += 256) {
        const int row = e / kKcF, k = e % kKcF;
        const int tp = p * kTileF + row, tq = q * kTileF + row;
        const bool kin = k0 + k < d;
        sp[row][k] = (tp < T && kin) ? base[(samp_row0 + tp) * stride + k0 + k] : 0.f;
        sq[row][k] = (tq < T && kin) ? base[(samp_row0 + tq) * stride + k0 + k] : 0.f;
      }
      __syncthreads();
#pragma unroll 8
      for (int k = 0; k < kKcF; ++k) {
        const float x0 = sp[ty * 2][k], x1 = sp[ty * 2 + 1][k];
        const float y0 = sq[tx * 2][k], y1 = sq[tx * 2 + 1][k];
        prod[o][0][0] = fmaf(x0, y0, prod[o][0][0]);
        prod[o][0][1] = fmaf(x0, y1, prod[o][0][1]);
        prod[o][1][0] = fmaf(x1, y0, prod[o][1][0]);
        prod[o][1][1] = fmaf(x1, y1, prod[o][1][1]);
      }
      __syncthreads();
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) s += prod[0][i][j] * prod[1][i][j];
  s = wave_sum_f32(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    g.partials[(size_t(layer) * g.B + sample) * g.n_pairs + pair] = (p == q) ? tot : 2.f * tot;
  }
}

int gram_tile_edge(int dtype, int /*variant*/) { return is_16bit(dtype) ? kTile : kTileF; }

static GramArgs make_args(const GramLaunch& l) {
  GramArgs a;
  a.layers = l.layers;
  a.order = l.order;
  a.partials = l.partials;
  a.n_layers = l.n_layers;
  a.B = l.B;
  a.T = l.T;
  a.n_pairs = l.n_pairs;
  a.nt = (l.T + l.tile - 1) / l.tile;
  const int units = l.n_layers * l.B;
  a.units_padded = (units + kNumXcd - 1) / kNumXcd * kNumXcd;
  return a;
}

hipError_t launch_gram_bf16(const GramLaunch& l, int /*variant*/, hipStream_t st) {
  auto kern = l.dtype == ADLOCO_F16 ? gram_bf16_kernel<true> : gram_bf16_kernel<false>;
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kGramLds);
    if (e != hipSuccess) return e;
  }
  GramArgs a = make_args(l);
  const long long grid = (long long)a.units_padded * a.n_pairs;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3(unsigned(grid)), dim3(256), kGramLds, st, a);
  return hipGetLastError();
}

// Jobs of the dual-tile kernel for nt row blocks: tile pairs (p,q), p <= q, taken two at a time.
// A pair on the diagonal costs three MFMAs per wave and k-step, any other four, and a job lasts as
// long as its slower pair: so diagonal pairs go together, (p,p) with (p+1,p+1) (two blocks to
// stage).  Off the diagonal, consecutive pairs (p,q),(p,q+1) of a row share block p; a row's
// leftover (p, nt-1) is combined with another row's leftover, which shares block nt-1.
std::vector<GramJob> make_gram_jobs(int nt, int order) {
  std::vector<GramJob> jobs, diag_jobs;
  auto make = [&](int p0, int q0, int p1, int q1) {
    GramJob j{};
    int blocks[4] = {p0, q0, p1 < 0 ? p0 : p1, q1 < 0 ? q0 : q1};
    int n = 0;
    int idx[4];
    for (int i = 0; i < 4; ++i) {
      int f = -1;
      for (int k = 0; k < n; ++k)
        if (j.blk[k] == blocks[i]) f = k;
      if (f < 0) { j.blk[n] = blocks[i]; f = n++; }
      idx[i] = f;
    }
    j.nblk = n;
    for (int k = n; k < 3; ++k) j.blk[k] = j.blk[0];
    j.sa[0] = idx[0]; j.sb[0] = idx[1]; j.sa[1] = idx[2]; j.sb[1] = idx[3];
    j.w[0] = p0 == q0 ? 1.f : 2.f;
    j.w[1] = p1 < 0 ? 0.f : (p1 == q1 ? 1.f : 2.f);
    jobs.push_back(j);
  };
  for (int d0 = 0; d0 + 1 < nt; d0 += 2) make(d0, d0, d0 + 1, d0 + 1);
  diag_jobs.swap(jobs);
  std::vector<int> left;
  for (int p = 0; p < nt; ++p) {
    int q = p + 1;
    for (; q + 1 < nt; q += 2) make(p, q, p, q + 1);
    if (q == nt - 1) left.push_back(p);
  }
  size_t i = 0;
  for (; i + 1 < left.size(); i += 2) make(left[i], nt - 1, left[i + 1], nt - 1);
  if (i < left.size()) {
    // one off-diagonal pair is left: it takes the last diagonal pair along when their number is odd
    if (nt % 2) make(left[i], nt - 1, nt - 1, nt - 1); else make(left[i], nt - 1, -1, -1);
  } else if (nt % 2) {
    make(nt - 1, nt - 1, -1, -1);
  }
  // Where the (shorter) jobs of two diagonal pairs go among the others.  First: they run a little
  // ahead of the unit's other jobs and touch all of its row blocks, which the others then find in
  // the cache (the order of the off-diagonal jobs among themselves made no difference).
  std::vector<GramJob> out;
  if (order == 1) {                       // last
    out = jobs;
    out.insert(out.end(), diag_jobs.begin(), diag_jobs.end());
  } else if (order == 2) {                // spread evenly
    const size_t n = jobs.size(), m = diag_jobs.size();
    size_t di = 0;
    for (size_t i = 0; i < n; ++i) {
      while (di < m && di * n <= i * m) out.push_back(diag_jobs[di++]);
      out.push_back(jobs[i]);
    }
    while (di < m) out.push_back(diag_jobs[di++]);
  } else {                                // first
    out = diag_jobs;
    out.insert(out.end(), jobs.begin(), jobs.end());
  }
  return out;
}

int gram_dual_parts(int n_jobs) { return n_jobs * 8; }

// variant: 1 = no layers share their activations (every group has one member), else groups of up to four
hipError_t launch_gram_bf16_dual(const GramLaunch& l, const GramGroup* groups, const GramJob* jobs,
                                 int n_jobs, int variant, hipStream_t st) {
  const bool f16 = l.dtype == ADLOCO_F16;
  auto kern = variant == 1 ? (f16 ? gram_bf16_dual_kernel<true, 1> : gram_bf16_dual_kernel<false, 1>)
                           : (f16 ? gram_bf16_dual_kernel<true, kGramGroupMax> : gram_bf16_dual_kernel<false, kGramGroupMax>);
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kDualLds);
    if (e != hipSuccess) return e;
  }
  GramDualArgs a;
  a.layers = l.layers;
  a.groups = groups;
  a.order = l.order;
  a.jobs = jobs;
  a.partials = l.partials;
  a.n_groups = l.n_layers;
  a.B = l.B;
  a.T = l.T;
  a.n_jobs = n_jobs;
  const int units = l.n_layers * l.B;
  a.units_padded = (units + kNumXcd - 1) / kNumXcd * kNumXcd;
  const long long grid = (long long)a.units_padded * n_jobs;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3(unsigned(grid)), dim3(512), kDualLds, st, a);
  return hipGetLastError();
}

hipError_t launch_gram_f32(const GramLaunch& l, hipStream_t st) {
  GramArgs a = make_args(l);
  const long long grid = (long long)a.units_padded * a.n_pairs;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gram_f32_kernel, dim3(unsigned(grid)), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace adloco
