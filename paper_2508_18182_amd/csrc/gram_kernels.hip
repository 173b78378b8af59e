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
        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m], fb[n], acc[m][n], 0, 0, 0);
  }
}

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
    mma_stage(cur, wm, wn, lane, acc);
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

int gram_tile_edge(int dtype, int /*variant*/) { return dtype == ADLOCO_BF16 ? kTile : kTileF; }

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
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gram_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kGramLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  GramArgs a = make_args(l);
  const long long grid = (long long)a.units_padded * a.n_pairs;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gram_bf16_kernel, dim3(unsigned(grid)), dim3(256), kGramLds, st, a);
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
