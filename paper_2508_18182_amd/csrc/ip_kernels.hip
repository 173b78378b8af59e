// Kernels that form the per-sample gradients g_i = delta_i^T a_i of the linear layers tile by tile
// in registers (never in memory) and reduce each tile on the spot:
//   * inner products c_i = <g_i, G> with the batch gradient sum G, whose variance the
//     inner-product test and the augmented inner-product test of Section 3.3.2 need;
//   * the statistics of the norm test (eq. 4, Section 3.3.1): ||g_i||^2 from the squares of the
//     tiles while they are being added up to G -- the route of adloco_grad_stats where G is
//     formed by the library.
// Aligned bf16 layers take the MFMA tile kernel (ip_tile_kernel); a plain path covers every other
// layer for the inner products, and the dot kernels of the vector / table blocks and the
// reductions follow.  The inner-product paths also return the explicit ||g_i||^2, a second
// route to the Gram kernel's result.
#include "common.h"

namespace adloco {

constexpr int kIpThreads = 256;

__device__ __forceinline__ float ip_elem(unsigned short h) { return __uint_as_float(unsigned(h) << 16); }
__device__ __forceinline__ float ip_elem(_Float16 h) { return float(h); }
__device__ __forceinline__ float ip_elem(float f) { return f; }

__device__ __forceinline__ double ip_wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double ip_block_sum(double v, double* lds4) {
  v = ip_wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

// ---------------------------------------------------------------------------------------
// Tile path (aligned bf16 linear layers, T a multiple of 32).
// Work item = one 256 (d_out) x 128 (d_in) tile of one layer for a run of consecutive samples.
// The workgroup (8 waves as 4 x 2, wave tile 64 x 64) streams the token rows of its samples
// through one uninterrupted load pipeline: the rows of consecutive samples are consecutive in
// memory.  Every T rows the accumulators hold that sample's gradient tile.  A second set of 64
// registers per lane, in the MFMA accumulator layout, holds
//   MODE 0 (inner products): the tile of G; the finished sample tile is multiplied element-wise
//     with it, summed over the wave and cleared; two floats per (tile, sample, wave) leave the chip;
//   MODE 1 (statistics): the running sum of the sample tiles; each finished tile is squared and
//     summed (its share of ||g_i||^2), added to the running sum and cleared; the sum is stored as
//     the tile of G at the end.
// A 256 x 256 tile would need 128 accumulators + 128 registers of the second set per lane, the
// whole register file at two waves per SIMD.
//   Staging: global -> LDS directly, four stages of 32 token rows x (256 + 128) columns.  A load
//   instruction moves 1 KiB: token rows j, j+16 of delta (2 x 512 B) or rows j, j+8, j+16, j+24 of
//   a (4 x 256 B); the 1 KiB blocks are 1088 bytes apart so that the four consecutive rows of an
//   LDS transpose read fall into different banks.  One barrier per chunk, loads two chunks ahead.
// ---------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 ip_bf16x8;
typedef __attribute__((ext_vector_type(16))) float ip_f32x16;
typedef __attribute__((ext_vector_type(4))) short ip_s16x4;
typedef __attribute__((ext_vector_type(8))) short ip_s16x8;

constexpr int kIpE = 256;                         // tile rows (d_out side)
constexpr int kIpC = 128;                         // tile columns (d_in side)
constexpr int kIpK = 32;                          // token rows per stage
constexpr int kIpBlk = 1024 + 64;                 // one load instruction + 64 B skew
constexpr int kIpOpE = 16 * kIpBlk;               // delta side of a stage
constexpr int kIpOpC = 8 * kIpBlk;                // a side of a stage
constexpr int kIpStage = kIpOpE + kIpOpC;         // 25.5 KiB
#ifndef IP_WM
#define IP_WM 4
#endif
constexpr int kIpWM = IP_WM, kIpWN = 2;           // waves along d_out and d_in
constexpr int kIpWaves = kIpWM * kIpWN;
constexpr int kIpFM = kIpE / (32 * kIpWM);        // 32x32 MFMA blocks per wave along d_out
constexpr int kIpFN = kIpC / (32 * kIpWN);        // ... along d_in
constexpr int kIpLdE = 16 / kIpWaves, kIpLdC = 8 / kIpWaves, kIpLd = kIpLdE + kIpLdC;   // loads per wave
constexpr int kIpStages = 4;
constexpr int kIpLds = kIpStages * kIpStage;      // 102 KiB

struct IpTileArgs {
  const LayerDev* layers;
  const int4* tiles;      // [8][slots]: (layer, e0, c0, first sample | samples << 16); layer < 0: none
  float* out;             // [8 * slots][group][kIpWaves][2]: <tile_i, G tile>, sum of squares of tile_i
                          // (statistics form: sum of squares, unused)
  int slots, T, group;
  // statistics form only
  const int* part;        // [8][slots]: -1: the entry covers all samples and owns its tile of G;
                          // else index of the partial tile that receives its share of the sum
  float* partials;        // [pieces][256][128] fp32
  int accumulate;         // G += sum instead of G = sum
};

// Sum over the 64 lanes without the LDS round trips of a shuffle chain: four DPP steps leave the
// total of each row of 16 lanes in all of its lanes, the four row totals are then read as scalars.
__device__ __forceinline__ float ip_wave_sum_f32(float v) {
#define IP_DPP(x, ctrl) \
  __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (x)), (ctrl), 0xf, 0xf, true))
  v += IP_DPP(v, 0xB1);    // quad_perm [1,0,3,2]
  v += IP_DPP(v, 0x4E);    // quad_perm [2,3,0,1]
  v += IP_DPP(v, 0x141);   // row_half_mirror
  v += IP_DPP(v, 0x140);   // row_mirror
#undef IP_DPP
  const int b = __builtin_bit_cast(int, v);
  return (__builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)) +
          __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16))) +
         (__builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)) +
          __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48)));
}

template <int N> __device__ __forceinline__ void ip_wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 0xf) | ((N >> 4) << 14));
}
__device__ __forceinline__ int ip_row_off_e(int row) { return (row & 15) * kIpBlk + (row >> 4) * 512; }
__device__ __forceinline__ int ip_row_off_c(int row) { return (row & 7) * kIpBlk + (row >> 3) * 256; }

// MODE 1 is the explicit form of the per-sample norms: when G has to be formed here anyway, its
// per-sample terms pass through the registers and the Gram contraction is not needed.
// SQ: also return the tile's sum of squares (always in MODE 1).
template <int MODE, bool SQ, bool F16>
__global__ __launch_bounds__(64 * kIpWaves, 1) void ip_tile_kernel(IpTileArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int xcd = blockIdx.x % kNumXcd, slot = blockIdx.x / kNumXcd;
  const int4 tile = g.tiles[xcd * g.slots + slot];
  if (tile.x < 0) return;
  const LayerDev L = g.layers[tile.x];
  const int e0 = tile.y, c0 = tile.z;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / kIpWN, wn = wave % kIpWN;  // kIpWM x kIpWN waves
  const int nk_sample = g.T / kIpK;               // chunks per sample
  const long long ck0 = (long long)(tile.w & 0xffff) * nk_sample;
  const int nk = (tile.w >> 16) * nk_sample;       // chunks of this entry: the host keeps it below 2^31

  // ---- second register set.  Accumulator element j of a 32x32 block: row
  // (j/4)*8 + (lane/32)*4 + j%4, column lane%32.  MODE 0: this lane's entries of the G tile
  // (zero past the edge); MODE 1: running sum of the sample tiles.
  float gt[kIpFM][kIpFN][16];
#pragma unroll
  for (int m = 0; m < kIpFM; ++m)
#pragma unroll
    for (int n = 0; n < kIpFN; ++n) {
      const int tc = c0 + wn * (32 * kIpFN) + n * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int tr = e0 + wm * (32 * kIpFM) + m * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if (MODE == 0) {
          const bool ok = tr < L.d_out && tc < L.d_in;
          const float v = L.grad_sum[ok ? (size_t)tr * L.d_in + tc : 0];
          gt[m][n][j] = ok ? v : 0.f;
        } else {
          gt[m][n][j] = 0.f;                       // running sum of the per-sample tiles
        }
      }
    }
  const bool ragged = e0 + kIpE > L.d_out || c0 + kIpC > L.d_in;

  // ---- direct loads, kIpLd per wave and chunk: delta instructions j = wave, wave + kIpWaves, ..
  // (rows j and j + 16, 16-byte piece lane % 32), then a instructions j = wave, .. (rows
  // j + 8 * (lane / 16), piece lane % 16).  Columns past the edge re-read the last valid piece.
  // Address = (first row of the chunk: wave-uniform, scalar registers) + (row within the chunk and
  // column: a 32-bit byte offset per lane, computed once; the host keeps row strides below 2^25).
  unsigned lane_off[kIpLd];
  int lds_off[kIpLd];
#pragma unroll
  for (int i = 0; i < kIpLd; ++i) {
    const bool is_a = i >= kIpLdE;
    const int j = wave + kIpWaves * (is_a ? i - kIpLdE : i);
    const int row = is_a ? j + 8 * (lane >> 4) : j + 16 * (lane >> 5);
    const int piece = is_a ? (lane & 15) : (lane & 31);
    const int d = is_a ? L.d_in : L.d_out;
    int col = (is_a ? c0 : e0) + piece * 8;
    col = col < d ? col : d - 8;
    lane_off[i] = unsigned(row * (is_a ? L.a_stride : L.delta_stride) + col) * 2u;
    lds_off[i] = (is_a ? kIpOpE : 0) + j * kIpBlk;
  }
  const unsigned short* const run_e = reinterpret_cast<const unsigned short*>(L.delta) + ck0 * kIpK * L.delta_stride;
  const unsigned short* const run_c = reinterpret_cast<const unsigned short*>(L.a) + ck0 * kIpK * L.a_stride;
  const unsigned lds_base = lds_address(lds);       // LDS byte addresses are handled as integers
  // stage indices are carried along (no modulo in the loop: kIpStages need not be a power of two)
  auto issue_loads = [&](int c, int st) {
    const unsigned stage = lds_base + unsigned(st) * kIpStage;
    const unsigned short* const pe = run_e + (long long)c * kIpK * L.delta_stride;
    const unsigned short* const pc = run_c + (long long)c * kIpK * L.a_stride;
#pragma unroll
    for (int i = 0; i < kIpLd; ++i)
      direct_load_lds16_s(lane_off[i], i >= kIpLdE ? pc : pe, stage + lds_off[i]);
  };

  // ---- fragments by LDS transpose reads.  Within a group of 16 lanes, lane s points at the 4
  // columns 4*(s%4).. of token row kbase + s/4; the read hands lane i column i of the group's
  // 16 at the four token rows.  Lane l ends up with column m0 + l%32, token rows
  // ks*16 + (l/32)*8 + 0..7.
  const int i16 = lane & 15;
  const int krow = (lane >> 5) * 8 + (i16 >> 2);              // + ks*16 (+4 for the upper half)
  const int ccol = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;    // column within a 32-wide block
  // Every read address of a k-step is stage + (a part that depends on the lane) + (a constant of the
  // fragment): three lane parts -- delta side; a side, rows r and r + 4, which wrap differently in
  // its 8-row blocks -- are kept in registers, the constants ride in the offset field of the read.
  typedef __attribute__((address_space(3))) ip_s16x4* lds_ptr;
  const unsigned lane_e = unsigned(ip_row_off_e(krow) + (wm * (32 * kIpFM) + ccol) * 2);
  const unsigned lane_c0 = unsigned(kIpOpE + ip_row_off_c(krow) + (wn * (32 * kIpFN) + ccol) * 2);
  const unsigned lane_c1 = unsigned(kIpOpE + ip_row_off_c(krow + 4) + (wn * (32 * kIpFN) + ccol) * 2);
  auto frag = [&](lds_ptr p0, lds_ptr p1) -> ip_bf16x8 {
    ip_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(p0);
    ip_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(p1);
    ip_s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(ip_bf16x8, v);
  };
  // token rows ks*16 + krow (+4) of the stage: row blocks of 16 (delta) and 8 (a) rows make ks * 512
  // bytes on both sides; 32 columns are 64 bytes; offsets in units of the 8-byte read
  auto read_frags = [&](int st, int ks, ip_bf16x8 (&fa)[kIpFM], ip_bf16x8 (&fb)[kIpFN]) {
    const unsigned stage = lds_base + unsigned(st) * kIpStage;
    const lds_ptr be = (lds_ptr)(size_t)(stage + lane_e);
    const lds_ptr bc0 = (lds_ptr)(size_t)(stage + lane_c0), bc1 = (lds_ptr)(size_t)(stage + lane_c1);
#pragma unroll
    for (int m = 0; m < kIpFM; ++m)
      fa[m] = frag(be + (ks * 512 + m * 64) / 8, be + (ks * 512 + m * 64 + 4 * kIpBlk) / 8);
#pragma unroll
    for (int n = 0; n < kIpFN; ++n)
      fb[n] = frag(bc0 + (ks * 512 + n * 64) / 8, bc1 + (ks * 512 + n * 64) / 8);
  };

  ip_f32x16 acc[kIpFM][kIpFN];
#pragma unroll
  for (int m = 0; m < kIpFM; ++m)
#pragma unroll
    for (int n = 0; n < kIpFN; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0.f;

  auto mfma4 = [&](const ip_bf16x8 (&a)[kIpFM], const ip_bf16x8 (&b)[kIpFN]) {
#pragma unroll
    for (int m = 0; m < kIpFM; ++m)
#pragma unroll
      for (int n = 0; n < kIpFN; ++n)
        acc[m][n] = mfma_32x32x16<F16>(a[m], b[n], acc[m][n]);
    // the LDS reads of the next k-step go out two at a time behind the first MFMAs
#pragma unroll
    for (int i = 0; i < kIpFM + kIpFN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    if (kIpFM * kIpFN > kIpFM + kIpFN)
      __builtin_amdgcn_sched_group_barrier(0x008, kIpFM * kIpFN - kIpFM - kIpFN, 0);
  };

  // prologue: chunks 0 .. kIpStages-2 in flight
#pragma unroll
  for (int s = 0; s < kIpStages - 1; ++s)
    if (s < nk) issue_loads(s, s);
  // The G registers are needed only at the end of the first sample, but a wait placed there by the
  // compiler would drain the load pipeline at every sample; pin them down here, once.
  if (MODE == 0) {
#pragma unroll
    for (int m = 0; m < kIpFM; ++m)
#pragma unroll
      for (int n = 0; n < kIpFN; ++n)
#pragma unroll
        for (int j = 0; j < 16; ++j) asm volatile("" : "+v"(gt[m][n][j]));
  }
  if (nk >= kIpStages - 1) ip_wait_vmcnt<kIpLd * (kIpStages - 2)>(); else ip_wait_vmcnt<0>();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  int left = nk_sample, sample_out = 0;
  float* dst = g.out + ((size_t(xcd) * g.slots + slot) * g.group * kIpWaves + wave) * 2;
  ip_bf16x8 fa[2][kIpFM], fb[2][kIpFN];
  read_frags(0, 0, fa[0], fb[0]);
  int st_cur = 0, st_load = kIpStages - 1;        // stage of chunk c; stage that chunk c-1 frees
  for (int c = 0; c < nk; ++c) {
    const int st_next = st_cur + 1 == kIpStages ? 0 : st_cur + 1;
    read_frags(st_cur, 1, fa[1], fb[1]);
    mfma4(fa[0], fb[0]);
    if (c + 1 < nk) {
      // chunk c+1 has landed for me (the chunks behind it may still be in flight), then for
      // everybody; every wave is done with chunk c-1, whose stage takes chunk c-1+kIpStages
      if (c + kIpStages - 2 < nk) ip_wait_vmcnt<kIpLd * (kIpStages - 3)>(); else ip_wait_vmcnt<0>();
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (c + kIpStages - 1 < nk) issue_loads(c + kIpStages - 1, st_load);
    }
    read_frags(c + 1 < nk ? st_next : st_cur, 0, fa[0], fb[0]);
    mfma4(fa[1], fb[1]);
    st_load = st_cur;
    st_cur = st_next;
    if (--left == 0) {
      // the sample's tile is complete: reduce it against the G tile, clear it
      float dot = 0.f, sq = 0.f;
      if (!ragged) {
#pragma unroll
        for (int m = 0; m < kIpFM; ++m)
#pragma unroll
          for (int n = 0; n < kIpFN; ++n)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const float v = acc[m][n][j];
              if (MODE == 0) dot = fmaf(v, gt[m][n][j], dot);
              else gt[m][n][j] += v;
              if (SQ) sq = fmaf(v, v, sq);
              acc[m][n][j] = 0.f;
            }
      } else {
        // tile on the edge of the layer: entries past the edge hold products of re-read columns;
        // they meet zeros in the G registers (MODE 0) or are never stored (MODE 1), but must not
        // enter the sum of squares
#pragma unroll
        for (int m = 0; m < kIpFM; ++m)
#pragma unroll
          for (int n = 0; n < kIpFN; ++n) {
            const bool col_ok = c0 + wn * (32 * kIpFN) + n * 32 + (lane & 31) < L.d_in;
            const int tr0 = e0 + wm * (32 * kIpFM) + m * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const float v = acc[m][n][j];
              if (MODE == 0) dot = fmaf(v, gt[m][n][j], dot);
              else gt[m][n][j] += v;
              if (SQ) {
                const float vm = (col_ok && tr0 + (j >> 2) * 8 + (j & 3) < L.d_out) ? v : 0.f;
                sq = fmaf(vm, vm, sq);
              }
              acc[m][n][j] = 0.f;
            }
          }
      }
      if (MODE == 0) dot = ip_wave_sum_f32(dot);
      if (SQ) sq = ip_wave_sum_f32(sq);
      if (lane == 0) {
        if (MODE == 0) {
          dst[size_t(sample_out) * (2 * kIpWaves)] = dot;
          dst[size_t(sample_out) * (2 * kIpWaves) + 1] = sq;
        } else {
          dst[size_t(sample_out) * (2 * kIpWaves)] = sq;
        }
      }
      ++sample_out;
      left = nk_sample;
    }
  }
  if (MODE == 1) {
    const int part = g.part[xcd * g.slots + slot];
    float* pt = part >= 0 ? g.partials + (size_t)part * (kIpE * kIpC) : nullptr;
#pragma unroll
    for (int m = 0; m < kIpFM; ++m)
#pragma unroll
      for (int n = 0; n < kIpFN; ++n) {
        const int tc = wn * (32 * kIpFN) + n * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int tr = wm * (32 * kIpFM) + m * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
          if (pt) {
            pt[tr * kIpC + tc] = gt[m][n][j];
          } else if (e0 + tr < L.d_out && c0 + tc < L.d_in) {
            float* d = L.grad_sum + (size_t)(e0 + tr) * L.d_in + c0 + tc;
            *d = g.accumulate ? *d + gt[m][n][j] : gt[m][n][j];
          }
        }
      }
  }
}

// Statistics form: sums the partial tiles of the entries that were split along the samples, in
// piece order (fixed order: repeatable), into grad_sum.  One workgroup per 4 rows of a split tile,
// one thread per column, rows unrolled so that their loads are in flight together;
// split[t] = (layer, e0, c0, pieces << 16 | first partial tile).
constexpr int kIpRedRows = 4;
__global__ __launch_bounds__(kIpC) void stats_tile_reduce_kernel(const LayerDev* layers, const int4* split,
                                                                const float* partials, int accumulate) {
  const int t = blockIdx.x / (kIpE / kIpRedRows), r0 = (blockIdx.x % (kIpE / kIpRedRows)) * kIpRedRows;
  const int4 S = split[t];
  const LayerDev L = layers[S.x];
  const int pieces = S.w >> 16;
  const float* base = partials + (size_t)(S.w & 0xffff) * (kIpE * kIpC) + threadIdx.x;
  const int col = S.z + threadIdx.x;
  float v[kIpRedRows];
#pragma unroll
  for (int r = 0; r < kIpRedRows; ++r) v[r] = 0.f;
  for (int p = 0; p < pieces; ++p)
#pragma unroll
    for (int r = 0; r < kIpRedRows; ++r) v[r] += base[(size_t)p * (kIpE * kIpC) + (r0 + r) * kIpC];
#pragma unroll
  for (int r = 0; r < kIpRedRows; ++r) {
    const int row = S.y + r0 + r;
    if (row >= L.d_out || col >= L.d_in) continue;
    float* d = L.grad_sum + (size_t)row * L.d_in + col;
    *d = accumulate ? *d + v[r] : v[r];
  }
}

// Statistics form: ||g_i^l||^2 = sum over the layer's tile entries and waves of the tile's sum of
// squares -> slot 0 of the layer's partial sums (the other slots are cleared), from where the
// common reduction picks it up.  One workgroup per (listed layer, sample); the entries of layer
// `lay[q]` are idx[ptr[q] .. ptr[q+1]).
__global__ __launch_bounds__(64) void stats_tile_finalize_kernel(const int4* tiles, const float* out, int group,
                                                                const int* lay, const int* ptr, const int* idx,
                                                                int B, float* partials, int n_pairs) {
  const int q = blockIdx.x / B, i = blockIdx.x % B;
  const int l = lay[q];
  double s = 0.0;
  for (int k = ptr[q] + threadIdx.x; k < ptr[q + 1]; k += 64) {
    const int e = idx[k];
    const int4 t = tiles[e];
    const int s0 = t.w & 0xffff, cnt = t.w >> 16;
    if (i >= s0 && i < s0 + cnt) {
      const float* o = out + ((size_t)e * group + (i - s0)) * (2 * kIpWaves);
#pragma unroll
      for (int w = 0; w < kIpWaves; ++w) s += double(o[2 * w]);
    }
  }
  s = ip_wave_sum(s);
  float* p = partials + (size_t(l) * B + i) * n_pairs;
  if (threadIdx.x == 0) p[0] = float(s);
  for (int k = 1 + threadIdx.x; k < n_pairs; k += 64) p[k] = 0.f;
}

// Tile table.  All tiles of one (layer, run of samples) stream the same rows, so such a set
// goes to one XCD (one L2); sets are dealt to the least loaded XCD, largest first.  The run
// length trades the once-per-entry costs (G tile, pipeline fill) against the balance of the last
// round of workgroups.
int make_ip_tiles(const std::vector<LayerDev>& layers, const std::vector<char>& use, int B, int T,
                  int forced_group, std::vector<int4>& out, int& group) {
  auto tiles_of = [&](const LayerDev& L) {
    return (long long)((L.d_out + kIpE - 1) / kIpE) * ((L.d_in + kIpC - 1) / kIpC);
  };
  long long tiles_all = 0;
  for (size_t l = 0; l < layers.size(); ++l)
    if (use[l]) tiles_all += tiles_of(layers[l]);
  // cost in chunks of 32 token rows: an entry of s samples costs s * T/32 + 8; 32 workgroups run
  // at a time on each of the 8 XCDs
  const double per_sample = double(T) / kIpK, fixed = 8.0;
  double best = 0.0;
  group = 1;
  for (int gsz = 1; gsz <= std::min(B, 0x7fff); ++gsz) {
    const long long runs = (B + gsz - 1) / gsz;
    const double rounds = std::ceil(double(tiles_all * runs) / (32.0 * kNumXcd));
    const double cost = rounds * (gsz * per_sample + fixed);
    if (gsz == 1 || cost < best * 0.999) {
      best = cost;
      group = gsz;
    }
  }
  if (forced_group > 0) group = std::min(std::min(forced_group, B), 0x7fff);
  struct Set { int layer, s0, cnt; long long n; };
  std::vector<Set> sets;
  for (size_t l = 0; l < layers.size(); ++l) {
    if (!use[l]) continue;
    for (int s0 = 0; s0 < B; s0 += group)
      sets.push_back({int(l), s0, std::min(group, B - s0), tiles_of(layers[l])});
  }
  std::stable_sort(sets.begin(), sets.end(), [](const Set& x, const Set& y) {
    return x.n * x.cnt > y.n * y.cnt;
  });
  std::vector<std::vector<int4>> per(kNumXcd);
  std::vector<long long> load(kNumXcd, 0);
  for (const Set& S : sets) {
    int bx = 0;
    for (int x = 1; x < kNumXcd; ++x)
      if (load[x] < load[bx]) bx = x;
    load[bx] += S.n * S.cnt;
    const LayerDev& L = layers[S.layer];
    for_tiles_blocked((L.d_out + kIpE - 1) / kIpE, (L.d_in + kIpC - 1) / kIpC, kIpE / kIpC, [&](int e, int c) {
      per[bx].push_back(int4{S.layer, e * kIpE, c * kIpC, S.s0 | (S.cnt << 16)});
    });
  }
  size_t slots = 0;
  for (auto& v : per) slots = std::max(slots, v.size());
  out.assign(size_t(kNumXcd) * slots, int4{-1, 0, 0, 0});
  for (int x = 0; x < kNumXcd; ++x)
    for (size_t i = 0; i < per[x].size(); ++i) out[x * slots + i] = per[x][i];
  return int(slots);
}

hipError_t launch_ip_tiles(const LayerDev* layers, const void* tiles, int slots, int T, int group,
                           int dtype, bool want_sq, float* ip_out, hipStream_t st) {
  if (slots <= 0) return hipSuccess;
  const bool h = dtype == ADLOCO_F16;
  auto kern = want_sq ? (h ? ip_tile_kernel<0, true, true> : ip_tile_kernel<0, true, false>)
                      : (h ? ip_tile_kernel<0, false, true> : ip_tile_kernel<0, false, false>);
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kIpLds);
    if (e != hipSuccess) return e;
  }
  IpTileArgs a{layers, static_cast<const int4*>(tiles), ip_out, slots, T, group, nullptr, nullptr, 0};
  hipLaunchKernelGGL(kern, dim3(unsigned(slots) * kNumXcd), dim3(64 * kIpWaves), kIpLds, st, a);
  return hipGetLastError();
}

// Tile table of the statistics form: one entry per 256 x 128 tile covering all B samples; the
// tiles of a layer go to one XCD where possible (they stream the same rows).  The entries of an XCD's incomplete last round of 32 are split along the samples
// into pieces whose partial sums a small kernel adds up in piece order.
// lay / ptr / idx: for every listed layer the indices (into `out`) of its entries.
int make_stats_tiles(const std::vector<LayerDev>& layers, const std::vector<char>& use, int B,
                     std::vector<int4>& out, std::vector<int>& part, std::vector<int4>& split,
                     std::vector<int>& lay, std::vector<int>& ptr, std::vector<int>& idx,
                     int& n_pieces) {
  constexpr int kCuPerXcd = kNumCu / kNumXcd;
  // all tiles in layer order (within a layer: blocks of tiles that share rows), cut into eight
  // equal runs: a layer stays on one XCD unless it straddles a cut, and the XCDs get the same
  // number of tiles
  std::vector<int4> all;
  for (size_t l = 0; l < layers.size(); ++l) {
    if (!use[l]) continue;
    for_tiles_blocked((layers[l].d_out + kIpE - 1) / kIpE, (layers[l].d_in + kIpC - 1) / kIpC, kIpE / kIpC,
                      [&](int e, int c) { all.push_back(int4{int(l), e * kIpE, c * kIpC, B << 16}); });
  }
  std::vector<std::vector<int4>> per(kNumXcd);
  for (int x = 0; x < kNumXcd; ++x)
    for (size_t i = all.size() * x / kNumXcd; i < all.size() * (x + 1) / kNumXcd; ++i)
      per[x].push_back(all[i]);
  split.clear();
  n_pieces = 0;
  std::vector<std::vector<int4>> fin(kNumXcd);
  std::vector<std::vector<int>> finp(kNumXcd);
  for (int x = 0; x < kNumXcd; ++x) {
    const int n = int(per[x].size());
    const int full = n / kCuPerXcd * kCuPerXcd, left = n - full;
    const int S = left > 0 ? std::min(kCuPerXcd / left, B) : 1;
    for (int i = 0; i < n; ++i) {
      if (i < full || S < 2 || n_pieces + S > 0xffff) {
        fin[x].push_back(per[x][i]);
        finp[x].push_back(-1);
        continue;
      }
      split.push_back(int4{per[x][i].x, per[x][i].y, per[x][i].z, (S << 16) | n_pieces});
      for (int p = 0; p < S; ++p) {
        const int s0 = int((long long)B * p / S), s1 = int((long long)B * (p + 1) / S);
        int4 e = per[x][i];
        e.w = s0 | ((s1 - s0) << 16);
        fin[x].push_back(e);
        finp[x].push_back(n_pieces + p);
      }
      n_pieces += S;
    }
  }
  size_t slots = 0;
  for (auto& v : fin) slots = std::max(slots, v.size());
  out.assign(size_t(kNumXcd) * slots, int4{-1, 0, 0, 0});
  part.assign(size_t(kNumXcd) * slots, -1);
  for (int x = 0; x < kNumXcd; ++x)
    for (size_t i = 0; i < fin[x].size(); ++i) {
      out[x * slots + i] = fin[x][i];
      part[x * slots + i] = finp[x][i];
    }
  std::vector<std::vector<int>> by_layer(layers.size());
  for (size_t k = 0; k < out.size(); ++k)
    if (out[k].x >= 0) by_layer[out[k].x].push_back(int(k));
  lay.clear();
  ptr.assign(1, 0);
  idx.clear();
  for (size_t l = 0; l < layers.size(); ++l) {
    if (!use[l]) continue;
    lay.push_back(int(l));
    idx.insert(idx.end(), by_layer[l].begin(), by_layer[l].end());
    ptr.push_back(int(idx.size()));
  }
  return int(slots);
}

hipError_t launch_stats_tiles(const LayerDev* layers, const void* tiles, const int* part, int slots,
                              const void* split, int n_split, float* partial_tiles, int B, int T,
                              int dtype, int accumulate, float* tile_out, const int* lay, const int* ptr,
                              const int* idx, int n_listed, float* partials, int n_pairs,
                              hipStream_t st) {
  if (slots <= 0) return hipSuccess;
  auto kern = dtype == ADLOCO_F16 ? ip_tile_kernel<1, true, true> : ip_tile_kernel<1, true, false>;
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kIpLds);
    if (e != hipSuccess) return e;
  }
  IpTileArgs a{layers, static_cast<const int4*>(tiles), tile_out, slots, T, B, part, partial_tiles, accumulate};
  hipLaunchKernelGGL(kern, dim3(unsigned(slots) * kNumXcd), dim3(64 * kIpWaves), kIpLds, st, a);
  if (n_split > 0)
    hipLaunchKernelGGL(stats_tile_reduce_kernel, dim3(unsigned(n_split) * (kIpE / kIpRedRows)), dim3(kIpC), 0, st,
                       layers, static_cast<const int4*>(split), partial_tiles, accumulate);
  hipLaunchKernelGGL(stats_tile_finalize_kernel, dim3(unsigned(n_listed) * B), dim3(64), 0, st,
                     static_cast<const int4*>(tiles), tile_out, B, lay, ptr, idx, B, partials, n_pairs);
  return hipGetLastError();
}

// Plain path for one linear layer: workgroup = (sample, 256 rows e of the gradient); a thread owns
// one row e and walks the columns c: g_ec = sum_t delta[t,e] a[t,c] (fp32), then adds
// g_ec * G[e,c] and g_ec^2 in fp64.  Slab totals go to part[(sample * slabs + slab) * 2 + {0,1}].
template <typename E>
__global__ __launch_bounds__(kIpThreads) void ip_generic_kernel(LayerDev L, int T, int slabs,
                                                               double* part) {
  __shared__ double lds4[4];
  const int sample = blockIdx.x / slabs, slab = blockIdx.x % slabs;
  const int e = slab * kIpThreads + threadIdx.x;
  const E* D = reinterpret_cast<const E*>(L.delta) + (long long)sample * T * L.delta_stride;
  const E* A = reinterpret_cast<const E*>(L.a) + (long long)sample * T * L.a_stride;
  double dot = 0.0, sq = 0.0;
  if (e < L.d_out) {
    for (int c = 0; c < L.d_in; ++c) {
      float gec = 0.f;
      for (int t = 0; t < T; ++t)
        gec = fmaf(ip_elem(D[(long long)t * L.delta_stride + e]), ip_elem(A[(long long)t * L.a_stride + c]), gec);
      dot += double(gec) * double(L.grad_sum[(size_t)e * L.d_in + c]);
      sq += double(gec) * double(gec);
    }
  }
  const double s0 = ip_block_sum(dot, lds4);
  const double s1 = ip_block_sum(sq, lds4);
  if (threadIdx.x == 0) {
    part[((size_t)sample * slabs + slab) * 2] = s0;
    part[((size_t)sample * slabs + slab) * 2 + 1] = s1;
  }
}

// Slab totals of the plain path -> dot[layer, sample], sq[layer, sample].
__global__ __launch_bounds__(64) void ip_generic_finish_kernel(const double* part, int slabs, int B,
                                                               float* dot, float* sq) {
  const int i = blockIdx.x * 64 + threadIdx.x;
  if (i >= B) return;
  double s0 = 0.0, s1 = 0.0;
  for (int k = 0; k < slabs; ++k) {
    s0 += part[((size_t)i * slabs + k) * 2];
    s1 += part[((size_t)i * slabs + k) * 2 + 1];
  }
  dot[i] = float(s0);
  sq[i] = float(s1);
}

// Vector blocks: v_i [d] is in `vec` (vector_rowsum_kernel); <v_i, G> -> dot[layer, sample].
__global__ __launch_bounds__(kIpThreads) void vector_ip_kernel(const LayerDev* layers, const AuxDesc* tab,
                                                              int B, const float* vec, float* dot) {
  __shared__ double lds4[4];
  const AuxDesc A = tab[blockIdx.x / B];
  const int sample = blockIdx.x % B;
  const LayerDev L = layers[A.layer];
  const float* v = vec + A.vec_off + (long long)sample * L.d_out;
  double acc = 0.0;
  for (int c = threadIdx.x; c < L.d_out; c += kIpThreads) acc += double(v[c]) * double(L.grad_sum[c]);
  const double s = ip_block_sum(acc, lds4);
  if (threadIdx.x == 0) dot[size_t(A.layer) * B + sample] = float(s);
}

// Embedding tables: <g_i, G> = sum_t <delta_t, G[id_t, :]>; ids outside [0, V) own no row of the
// table and contribute nothing.
template <typename E>
__global__ __launch_bounds__(kIpThreads) void embed_ip_kernel(const LayerDev* layers, const AuxDesc* tab,
                                                             int B, int T, float* dot) {
  __shared__ double lds4[4];
  const AuxDesc A = tab[blockIdx.x / B];
  const int sample = blockIdx.x % B;
  const LayerDev L = layers[A.layer];
  const int* ids = reinterpret_cast<const int*>(L.a) + (long long)sample * T;
  const E* D = reinterpret_cast<const E*>(L.delta) + (long long)sample * T * L.delta_stride;
  double acc = 0.0;
  for (int t = 0; t < T; ++t) {
    const int id = ids[t];
    if (id < 0 || id >= L.d_in) continue;
    const float* row = L.grad_sum + (size_t)id * L.d_out;
    float s = 0.f;
    for (int c = threadIdx.x; c < L.d_out; c += kIpThreads)
      s = fmaf(ip_elem(D[(long long)t * L.delta_stride + c]), row[c], s);
    acc += double(s);
  }
  const double s = ip_block_sum(acc, lds4);
  if (threadIdx.x == 0) dot[size_t(A.layer) * B + sample] = float(s);
}

// One workgroup per sample i: c_i = sum of its tile results + sum over the other blocks;
// likewise the explicit ||g_i||^2.  A tile entry covers samples [w & 0xffff, + (w >> 16)) and
// leaves, per sample and wave, a pair at tile_out[((k * group + sample - first) * 8 + wave) * 2].
__global__ __launch_bounds__(kIpThreads) void ip_finalize_samples_kernel(
    const int4* tiles, const float* tile_out, long long n_tiles, int group, const float* dot, const float* sq,
    const unsigned char* in_tiles, int n_layers, int B, float* per_sample_ip, float* per_sample_sq,
    double* sample_f64) {
  __shared__ double lds4[4];
  const int i = blockIdx.x;
  double c = 0.0, q = 0.0;
  for (long long k = threadIdx.x; k < n_tiles; k += kIpThreads) {
    const int4 t = tiles[k];
    const int s0 = t.w & 0xffff, cnt = t.w >> 16;
    if (t.x >= 0 && i >= s0 && i < s0 + cnt) {
      const float* o = tile_out + ((size_t)k * group + (i - s0)) * (2 * kIpWaves);
#pragma unroll
      for (int w = 0; w < kIpWaves; ++w) {
        c += double(o[2 * w]);
        q += double(o[2 * w + 1]);
      }
    }
  }
  for (int l = threadIdx.x; l < n_layers; l += kIpThreads)
    if (!in_tiles[l]) {
      c += double(dot[size_t(l) * B + i]);
      q += double(sq[size_t(l) * B + i]);
    }
  const double cs = ip_block_sum(c, lds4);
  const double qs = ip_block_sum(q, lds4);
  if (threadIdx.x == 0) {
    per_sample_ip[i] = float(cs);
    if (per_sample_sq) per_sample_sq[i] = float(qs);
    sample_f64[i] = cs;
  }
}

// One workgroup: sum_ip (+)= sum_i c_i, sum_ip_sq (+)= sum_i c_i^2, n_samples (+)= B.
__global__ __launch_bounds__(1024) void ip_finalize_batch_kernel(const double* sample_f64, int B,
                                                                 adloco_ip_acc* acc, int accumulate) {
  __shared__ double lds[16];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < B; i += blockDim.x) {
    a += sample_f64[i];
    b += sample_f64[i] * sample_f64[i];
  }
  a = ip_wave_sum(a);
  b = ip_wave_sum(b);
  if ((threadIdx.x & 63) == 0) { lds[threadIdx.x >> 6] = a; }
  __syncthreads();
  double sa = 0.0;
  if (threadIdx.x == 0) for (int w = 0; w < 16; ++w) sa += lds[w];
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { lds[threadIdx.x >> 6] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sb = 0.0;
    for (int w = 0; w < 16; ++w) sb += lds[w];
    if (accumulate) {
      acc->sum_ip += sa;
      acc->sum_ip_sq += sb;
      acc->n_samples += B;
    } else {
      acc->sum_ip = sa;
      acc->sum_ip_sq = sb;
      acc->n_samples = B;
    }
    acc->reserved = 0;
  }
}

hipError_t launch_ip_generic(const LayerDev& L, int layer, int B, int T, int dtype, double* part,
                             float* dot, float* sq, hipStream_t st) {
  const int slabs = (L.d_out + kIpThreads - 1) / kIpThreads;
  if (dtype == ADLOCO_BF16)
    hipLaunchKernelGGL(ip_generic_kernel<unsigned short>, dim3(unsigned(B) * slabs), dim3(kIpThreads), 0,
                       st, L, T, slabs, part);
  else if (dtype == ADLOCO_F16)
    hipLaunchKernelGGL(ip_generic_kernel<_Float16>, dim3(unsigned(B) * slabs), dim3(kIpThreads), 0,
                       st, L, T, slabs, part);
  else
    hipLaunchKernelGGL(ip_generic_kernel<float>, dim3(unsigned(B) * slabs), dim3(kIpThreads), 0, st, L, T,
                       slabs, part);
  hipLaunchKernelGGL(ip_generic_finish_kernel, dim3((B + 63) / 64), dim3(64), 0, st, part, slabs, B,
                     dot + size_t(layer) * B, sq + size_t(layer) * B);
  return hipGetLastError();
}
size_t ip_generic_part_doubles(const LayerDev& L, int B) {
  return size_t(B) * ((L.d_out + kIpThreads - 1) / kIpThreads) * 2;
}

hipError_t launch_ip_vector_table(const LayerDev* layers, const AuxDesc* vec_tab, int n_vec,
                                  const AuxDesc* emb_tab, int n_emb, int B, int T, int dtype,
                                  const float* vec, float* dot, hipStream_t st) {
  if (n_vec > 0)
    hipLaunchKernelGGL(vector_ip_kernel, dim3(unsigned(n_vec) * B), dim3(kIpThreads), 0, st, layers,
                       vec_tab, B, vec, dot);
  if (n_emb > 0) {
    if (dtype == ADLOCO_BF16)
      hipLaunchKernelGGL(embed_ip_kernel<unsigned short>, dim3(unsigned(n_emb) * B), dim3(kIpThreads), 0,
                         st, layers, emb_tab, B, T, dot);
    else if (dtype == ADLOCO_F16)
      hipLaunchKernelGGL(embed_ip_kernel<_Float16>, dim3(unsigned(n_emb) * B), dim3(kIpThreads), 0,
                         st, layers, emb_tab, B, T, dot);
    else
      hipLaunchKernelGGL(embed_ip_kernel<float>, dim3(unsigned(n_emb) * B), dim3(kIpThreads), 0, st,
                         layers, emb_tab, B, T, dot);
  }
  return hipGetLastError();
}

hipError_t launch_ip_finalize(const void* tiles, const float* tile_out, long long n_tiles, int group,
                              const float* dot, const float* sq, const unsigned char* in_tiles,
                              int n_layers, int B, float* per_sample_ip, float* per_sample_sq,
                              double* sample_f64, adloco_ip_acc* acc, int accumulate, hipStream_t st) {
  hipLaunchKernelGGL(ip_finalize_samples_kernel, dim3(B), dim3(kIpThreads), 0, st,
                     static_cast<const int4*>(tiles), tile_out, n_tiles, group, dot, sq, in_tiles, n_layers, B,
                     per_sample_ip, per_sample_sq, sample_f64);
  hipLaunchKernelGGL(ip_finalize_batch_kernel, dim3(1), dim3(1024), 0, st, sample_f64, B, acc,
                     accumulate);
  return hipGetLastError();
}

}  // namespace adloco
