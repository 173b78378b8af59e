// Gradient sum of a linear layer over the batch: G^l (+)= sum_i delta_i^T a_i, i.e. B times
// the mini-batch gradient of eq. 1 (and Algorithm 3's "g <- g + grad L" across micro-batches).
// A GEMM [d_out, d_in] with the contraction over all B*T token rows.  Both operands are stored
// token-major (the contraction index is the slow one), so tiles are staged in LDS as they are
// and handed to the MFMA through the LDS transpose read of gfx950.
#include <algorithm>

#include "common.h"

namespace adloco {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

struct WgradArgs {
  const LayerDev* layers;
  int n_layers;
  long long rows;      // B*T
  int accumulate;
};

__device__ __forceinline__ int find_layer_wg(const LayerDev* layers, int n_layers, int b) {
  int lo = 0, hi = n_layers - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (layers[mid].wg_blk_start <= b) lo = mid; else hi = mid - 1;
  }
  // layers with ADLOCO_GRAD_PROVIDED own no workgroup and share a start with their successor;
  // the search lands on the last layer with that start, which is the one that owns workgroups.
  return lo;
}

// ---------------------------------------------------------------------------------------
// bf16: 128 (d_out) x 128 (d_in) output tile per workgroup, 4 waves 2x2, MFMA 32x32x16.
// LDS stage: 32 token rows of delta[.,128] and of a[.,128], row pitch 144 elements.
// ---------------------------------------------------------------------------------------
constexpr int kWt = 128;
constexpr int kWk = 32;
constexpr int kWpitch = 144;                      // elements; 288 bytes
constexpr int kWopBytes = kWk * kWpitch * 2;      // one operand of one stage
constexpr int kWstage = 2 * kWopBytes;
constexpr int kWlds = 2 * kWstage;

struct WChunk { u32x4 v[4]; };

__device__ __forceinline__ void wgrad_load(const LayerDev& L, long long rows, long long k0, int e0,
                                           int c0, WChunk& r) {
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int e = threadIdx.x + 256 * it;
    const int op = e >> 9;                 // 0: delta (d_out side), 1: a (d_in side)
    const int row = (e & 511) >> 4;
    const int ch = e & 15;
    const unsigned short* base = reinterpret_cast<const unsigned short*>(op ? L.a : L.delta);
    const long long stride = op ? L.a_stride : L.delta_stride;
    const int d = op ? L.d_in : L.d_out;
    const int col = (op ? c0 : e0) + ch * 8;
    const long long k = k0 + row;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (k < rows && col < d) {
      const unsigned short* src = base + k * stride + col;
      if (L.fast) {
        v = *reinterpret_cast<const u32x4*>(src);
      } else {
        unsigned short h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = (col + j < d) ? src[j] : (unsigned short)0;
        v[0] = h[0] | (unsigned(h[1]) << 16);
        v[1] = h[2] | (unsigned(h[3]) << 16);
        v[2] = h[4] | (unsigned(h[5]) << 16);
        v[3] = h[6] | (unsigned(h[7]) << 16);
      }
    }
    r.v[it] = v;
  }
}

__device__ __forceinline__ void wgrad_store(unsigned char* stage, const WChunk& r) {
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int e = threadIdx.x + 256 * it;
    const int op = e >> 9;
    const int row = (e & 511) >> 4;
    const int ch = e & 15;
    *reinterpret_cast<u32x4*>(stage + op * kWopBytes + row * (kWpitch * 2) + ch * 16) = r.v[it];
  }
}

// Fragment of the MFMA operand for output rows/cols m0..m0+31 and k-step ks (16 token rows):
// lane l holds column m0 + l%32 at the eight token rows ks*16 + (l/32)*8 + 0..7.
template <int VARIANT>
__device__ __forceinline__ bf16x8 wgrad_frag(const unsigned char* op_base, int m0, int ks,
                                             int lane) {
  const int kbase = ks * 16 + (lane >> 5) * 8;
  if (VARIANT == 0) {
    // gather: eight 2-byte reads down one column
    const unsigned short* p =
        reinterpret_cast<const unsigned short*>(op_base) + kbase * kWpitch + m0 + (lane & 31);
    s16x8 v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (short)p[j * kWpitch];
    return __builtin_bit_cast(bf16x8, v);
  } else {
    // LDS transpose read: within each group of 16 lanes, lane s points at 4 consecutive columns
    // of token row kbase + s/4 (columns 4*(s%4)..+3 of the group's 16); the instruction hands
    // lane i the four token rows of column i.
    const int i = lane & 15;
    const int colbase = m0 + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
    const unsigned short* p =
        reinterpret_cast<const unsigned short*>(op_base) + (kbase + (i >> 2)) * kWpitch + colbase;
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * kWpitch));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int VARIANT, bool F16>
__device__ __forceinline__ void wgrad_mma(const unsigned char* stage, int wm, int wn, int lane,
                                          f32x16 (&acc)[2][2]) {
  const unsigned char* dt = stage;               // delta tile: rows = tokens, cols = d_out
  const unsigned char* at = stage + kWopBytes;   // a tile
#pragma unroll
  for (int ks = 0; ks < kWk / 16; ++ks) {
    bf16x8 fa[2], fb[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) fa[m] = wgrad_frag<VARIANT>(dt, wm * 64 + m * 32, ks, lane);
#pragma unroll
    for (int n = 0; n < 2; ++n) fb[n] = wgrad_frag<VARIANT>(at, wn * 64 + n * 32, ks, lane);
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int n = 0; n < 2; ++n)
        acc[m][n] = mfma_32x32x16<F16>(fa[m], fb[n], acc[m][n]);
  }
}

template <int VARIANT, bool F16>
__global__ __launch_bounds__(256, 2) void wgrad_bf16_kernel(WgradArgs g) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWlds];
  const int layer = find_layer_wg(g.layers, g.n_layers, blockIdx.x);
  const LayerDev L = g.layers[layer];
  const int tiles_c = (L.d_in + kWt - 1) / kWt;
  const int tile = blockIdx.x - L.wg_blk_start;
  const int e0 = (tile / tiles_c) * kWt;
  const int c0 = (tile % tiles_c) * kWt;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0.f;

  const long long nk = (g.rows + kWk - 1) / kWk;
  WChunk regs;
  wgrad_load(L, g.rows, 0, e0, c0, regs);
  wgrad_store(lds, regs);
  __syncthreads();
  for (long long c = 0; c < nk; ++c) {
    unsigned char* cur = lds + (c & 1) * kWstage;
    unsigned char* nxt = lds + ((c + 1) & 1) * kWstage;
    const bool more = c + 1 < nk;
    if (more) wgrad_load(L, g.rows, (c + 1) * kWk, e0, c0, regs);
    wgrad_mma<VARIANT, F16>(cur, wm, wn, lane, acc);
    if (more) wgrad_store(nxt, regs);
    __syncthreads();
  }

  // accumulator element j of a 32x32 block: row (j/4)*8 + (lane/32)*4 + j%4, column lane%32
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int col = c0 + wn * 64 + n * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int row = e0 + wm * 64 + m * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if (row < L.d_out && col < L.d_in) {
          float* dst = L.grad_sum + (size_t)row * L.d_in + col;
          *dst = g.accumulate ? *dst + acc[m][n][j] : acc[m][n][j];
        }
      }
    }
}

// ---------------------------------------------------------------------------------------
// bf16 fast path: 256 (d_out) x 256 (d_in) output tile per workgroup of 8 waves (2 x 4, each
// 128 x 64), used when every row is 16-byte aligned, widths are multiples of 8 and the number
// of token rows is a multiple of 32.
//   Staging: global -> LDS directly, four stages of 32 token rows x (256 + 256) columns; one
//   wave instruction moves two token rows of one operand (2 x 512 contiguous bytes); the LDS
//   blocks are padded so that the transpose reads of four consecutive rows fall into different
//   banks.
//   One barrier per 32-row chunk, between its two k-steps; loads run two chunks ahead.
//   Tiles are dealt to the XCDs layer by layer (table built on the host): the tiles of one layer
//   run next to each other on one XCD and stream the same columns out of that XCD's L2.
//   Columns beyond d_out / d_in re-read the last valid 16-byte piece; those accumulators are
//   never stored.
// ---------------------------------------------------------------------------------------
constexpr int kXt = 256;                          // tile edge
constexpr int kXk = 32;                           // token rows per stage
constexpr int kXrowB = kXt * 2;                   // bytes per staged row of one operand
constexpr int kXblk = 2 * kXrowB + 64;            // one load instruction: rows j and j+16, + 64 B pad
constexpr int kXop = 16 * kXblk;                  // 17 KiB
constexpr int kXstage = 2 * kXop;                 // 34 KiB
constexpr int kXstages = 4;
constexpr int kXlds = kXstages * kXstage;         // 136 KiB

struct WgradXArgs {
  const LayerDev* layers;
  const int4* tiles;      // [8][slots]: (layer, e0, c0, split); layer < 0 = no tile.
                          // split = 0: whole contraction, result goes to grad_sum;
                          // else (S << 24) | (piece << 16) | slot: piece of S equal parts of
                          // the contraction, result goes to partial tile `slot` of `partials`
  float* partials;        // [pieces][256][256] fp32
  int slots;
  long long rows;
  int accumulate;
};

template <int N> __device__ __forceinline__ void wgx_wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 0xf) | ((N >> 4) << 14));
}

// LDS offset of staged token row `row` (0..31) of one operand: load instruction j brings rows j
// and j+16 into one 1 KiB block; blocks are 1088 bytes apart, so four consecutive rows start
// 64 bytes apart modulo 256 and a transpose read (per 32 lanes: 4 rows x 2 x 32 bytes) touches
// 256 distinct bytes.  Global addresses stay linear: 512 contiguous bytes per half wave.
__device__ __forceinline__ int wgx_row_off(int row) { return (row & 15) * kXblk + (row >> 4) * kXrowB; }

template <bool F16>
__global__ __launch_bounds__(512, 1) void wgrad_bf16_x_kernel(WgradXArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int xcd = blockIdx.x % kNumXcd, slot = blockIdx.x / kNumXcd;
  const int4 tile = g.tiles[xcd * g.slots + slot];
  if (tile.x < 0) return;
  const LayerDev L = g.layers[tile.x];
  const int e0 = tile.y, c0 = tile.z;
  const int split_s = (tile.w >> 24) & 0xff, split_p = (tile.w >> 16) & 0xff, split_id = tile.w & 0xffff;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 2, wn = wave & 3;        // 2 x 4 waves; wave tile 128 (e) x 64 (c)
  // chunk range of this workgroup: everything, or piece split_p of split_s equal parts
  // (32-bit counters keep the loop's compares on the scalar unit; the host keeps rows / 32 < 2^31)
  const long long nk_all = g.rows / kXk;
  const long long ck0 = split_s ? nk_all * split_p / split_s : 0;
  const int nk = int((split_s ? nk_all * (split_p + 1) / split_s : nk_all) - ck0);

  // ---- direct loads: instruction j = wave + 8*i (i = 0..3): operand j/16, rows j%16 (lanes 0-31)
  // and j%16 + 16 (lanes 32-63), 16-byte piece lane%32
  // Address = (first row of the chunk: wave-uniform, scalar registers) + (row within the chunk and
  // column: a 32-bit byte offset per lane, computed once; the host keeps row strides below 2^25).
  // j = wave + 8*i < 16 for i = 0, 1 (delta) and >= 16 for i = 2, 3 (a).
  unsigned lane_off[4];
  int lds_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = wave + 8 * i;
    const int op = i >> 1;                        // 0: delta (d_out side), 1: a (d_in side)
    const int row = (j & 15) + 16 * (lane >> 5);
    const int piece = lane & 31;
    const int d = op ? L.d_in : L.d_out;
    int col = (op ? c0 : e0) + piece * 8;
    col = col < d ? col : d - 8;
    lane_off[i] = unsigned(row * (op ? L.a_stride : L.delta_stride) + col) * 2u;
    lds_off[i] = op * kXop + (j & 15) * kXblk;
  }
  const unsigned short* const run_e = reinterpret_cast<const unsigned short*>(L.delta) + ck0 * kXk * L.delta_stride;
  const unsigned short* const run_c = reinterpret_cast<const unsigned short*>(L.a) + ck0 * kXk * L.a_stride;
  const unsigned lds_base = lds_address(lds);       // LDS byte addresses are handled as integers
  auto issue_loads = [&](int c, int st) {
    const unsigned stage = lds_base + unsigned(st) * kXstage;
    const unsigned short* const pe = run_e + (long long)c * kXk * L.delta_stride;
    const unsigned short* const pc = run_c + (long long)c * kXk * L.a_stride;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      direct_load_lds16_s(lane_off[i], i >= 2 ? pc : pe, stage + lds_off[i]);
  };

  // ---- fragments by LDS transpose reads.  Within a group of 16 lanes, lane s points at the 4
  // columns 4*(s%4).. of token row kbase + s/4; the read hands lane i column i of the group's
  // 16 at the four token rows.  Lane l ends up with column m0 + l%32, token rows
  // ks*16 + (l/32)*8 + 0..7.
  const int i16 = lane & 15;
  const int krow = (lane >> 5) * 8 + (i16 >> 2);              // + ks*16 (+4 for the upper half)
  const int ccol = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;    // column within a 32-wide block
  // Every read address of a k-step is stage + (a part that depends on the lane) + (a constant of
  // the fragment): one lane part per operand is kept in a register, the constants ride in the
  // offset field of the read.  Token rows ks*16 + krow and + 4 stay inside one 16-row block.
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  const unsigned lane_e = unsigned(wgx_row_off(krow) + (wm * 128 + ccol) * 2);
  const unsigned lane_c = unsigned(kXop + wgx_row_off(krow) + (wn * 64 + ccol) * 2);
  auto frag = [&](lds_ptr base, int byte_off) -> bf16x8 {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(base + byte_off / 8);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(base + (byte_off + 4 * kXblk) / 8);
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  auto read_frags = [&](int st, int ks, bf16x8 (&fa)[4], bf16x8 (&fb)[2]) {
    const unsigned stage = lds_base + unsigned(st) * kXstage;
    const lds_ptr be = (lds_ptr)(size_t)(stage + lane_e), bc = (lds_ptr)(size_t)(stage + lane_c);
    // in the order the MFMAs need them; 32 columns are 64 bytes
    fa[0] = frag(be, ks * kXrowB);
    fb[0] = frag(bc, ks * kXrowB);
    fb[1] = frag(bc, ks * kXrowB + 64);
#pragma unroll
    for (int m = 1; m < 4; ++m) fa[m] = frag(be, ks * kXrowB + m * 64);
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0.f;

  auto mfma8 = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[2]) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int n = 0; n < 2; ++n)
        acc[m][n] = mfma_32x32x16<F16>(a[m], b[n], acc[m][n]);
    // issue order: the 12 LDS reads of the next k-step go out two at a time behind the first
    // six MFMAs, so that the last of them has two MFMAs to land before the next k-step starts
#pragma unroll
    for (int i = 0; i < 6; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
  };

  if (nk > 0) issue_loads(0, 0);
  if (nk > 1) issue_loads(1, 1);
  if (nk > 2) issue_loads(2, 2);
  if (nk > 2) wgx_wait_vmcnt<8>(); else if (nk > 1) wgx_wait_vmcnt<4>(); else wgx_wait_vmcnt<0>();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  bf16x8 fa[2][4], fb[2][2];
  read_frags(0, 0, fa[0], fb[0]);
  static_assert(kXstages == 4, "the stage of chunk c+3 is the stage of chunk c-1");
  int st_cur = 0, st_load = kXstages - 1;         // stage of chunk c; stage that chunk c-1 frees
  for (int c = 0; c < nk; ++c) {
    const int st_next = st_cur + 1 == kXstages ? 0 : st_cur + 1;
    read_frags(st_cur, 1, fa[1], fb[1]);
    mfma8(fa[0], fb[0]);
    if (c + 1 < nk) {
      // chunk c+1 has landed for me (chunk c+2 may still be in flight), then for everybody;
      // every wave is done with chunk c-1, whose stage takes chunk c+3
      if (c + 2 < nk) wgx_wait_vmcnt<4>(); else wgx_wait_vmcnt<0>();
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (c + 3 < nk) issue_loads(c + 3, st_load);
    }
    read_frags(c + 1 < nk ? st_next : st_cur, 0, fa[0], fb[0]);
    mfma8(fa[1], fb[1]);
    st_load = st_cur;
    st_cur = st_next;
  }

  // accumulator element j of a 32x32 block: row (j/4)*8 + (lane/32)*4 + j%4, column lane%32
  float* part = split_s ? g.partials + (size_t)split_id * (kXt * kXt) : nullptr;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int tc = wn * 64 + n * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int tr = wm * 128 + m * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if (split_s) {
          part[tr * kXt + tc] = acc[m][n][j];
        } else if (e0 + tr < L.d_out && c0 + tc < L.d_in) {
          float* dst = L.grad_sum + (size_t)(e0 + tr) * L.d_in + c0 + tc;
          *dst = g.accumulate ? *dst + acc[m][n][j] : acc[m][n][j];
        }
      }
    }
}

// Sums the partial tiles of a split contraction in piece order (fixed order: repeatable) and
// adds them to / stores them in grad_sum.  One workgroup per 4 rows of one split tile, one thread
// per column, rows unrolled so that their loads are in flight together.
struct WgradSplitTile { int layer, e0, c0, w; };   // w = (pieces << 16) | first partial tile
constexpr int kXredRows = 4;
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const LayerDev* layers,
                                                           const WgradSplitTile* tiles,
                                                           const float* partials, int accumulate) {
  const int t = blockIdx.x / (kXt / kXredRows), r0 = (blockIdx.x % (kXt / kXredRows)) * kXredRows;
  const WgradSplitTile S = tiles[t];
  const LayerDev L = layers[S.layer];
  const int pieces = S.w >> 16;
  const float* base = partials + (size_t)(S.w & 0xffff) * (kXt * kXt) + threadIdx.x;
  const int col = S.c0 + threadIdx.x;
  float v[kXredRows];
#pragma unroll
  for (int r = 0; r < kXredRows; ++r) v[r] = 0.f;
  for (int p = 0; p < pieces; ++p)
#pragma unroll
    for (int r = 0; r < kXredRows; ++r) v[r] += base[(size_t)p * (kXt * kXt) + (r0 + r) * kXt];
#pragma unroll
  for (int r = 0; r < kXredRows; ++r) {
    const int row = S.e0 + r0 + r;
    if (row >= L.d_out || col >= L.d_in) continue;
    float* dst = L.grad_sum + (size_t)row * L.d_in + col;
    *dst = accumulate ? *dst + v[r] : v[r];
  }
}

// ---------------------------------------------------------------------------------------
// fp32 inputs: plain FMA path, 32x32 output tile, 2x2 entries per thread.
// ---------------------------------------------------------------------------------------
constexpr int kWtF = 32;
constexpr int kWkF = 16;

__global__ __launch_bounds__(256) void wgrad_f32_kernel(WgradArgs g) {
  __shared__ float sd[kWkF][kWtF + 1];
  __shared__ float sa[kWkF][kWtF + 1];
  const int layer = find_layer_wg(g.layers, g.n_layers, blockIdx.x);
  const LayerDev L = g.layers[layer];
  const int tiles_c = (L.d_in + kWtF - 1) / kWtF;
  const int tile = blockIdx.x - L.wg_blk_start;
  const int e0 = (tile / tiles_c) * kWtF;
  const int c0 = (tile % tiles_c) * kWtF;
  const float* D = reinterpret_cast<const float*>(L.delta);
  const float* A = reinterpret_cast<const float*>(L.a);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  for (long long k0 = 0; k0 < g.rows; k0 += kWkF) {
    for (int e = threadIdx.x; e < kWkF * kWtF; e += 256) {
      const int row = e / kWtF, col = e % kWtF;
      const long long k = k0 + row;
      sd[row][col] = (k < g.rows && e0 + col < L.d_out) ? D[k * L.delta_stride + e0 + col] : 0.f;
      sa[row][col] = (k < g.rows && c0 + col < L.d_in) ? A[k * L.a_stride + c0 + col] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kWkF; ++k) {
      const float d0 = sd[k][ty * 2], d1 = sd[k][ty * 2 + 1];
      const float a0 = sa[k][tx * 2], a1 = sa[k][tx * 2 + 1];
      acc[0][0] = fmaf(d0, a0, acc[0][0]);
      acc[0][1] = fmaf(d0, a1, acc[0][1]);
      acc[1][0] = fmaf(d1, a0, acc[1][0]);
      acc[1][1] = fmaf(d1, a1, acc[1][1]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = e0 + ty * 2 + i, col = c0 + tx * 2 + j;
      if (row < L.d_out && col < L.d_in) {
        float* dst = L.grad_sum + (size_t)row * L.d_in + col;
        *dst = g.accumulate ? *dst + acc[i][j] : acc[i][j];
      }
    }
}

int wgrad_tile_edge(int dtype) { return is_16bit(dtype) ? kWt : kWtF; }

// Tile table of the fast kernel: [8 XCDs][slots] entries (layer, e0, c0, split).  The tiles of
// all layers, in layer order, are cut into eight equal runs, one per XCD: the tiles of a layer
// stream the same rows out of one L2 (a layer that straddles a cut out of two), and no XCD has
// more work than another.
// All tiles cost the same, so an XCD's 32 CUs work in rounds; the tiles of an incomplete last
// round are split along the contraction into as many pieces as fill the round, written to
// partial tiles and summed afterwards by wgrad_reduce_kernel.
int make_wgrad_x_tiles(const std::vector<LayerDev>& layers, std::vector<int4>& out,
                       std::vector<int4>& split_tiles, int& n_pieces) {
  constexpr int kCuPerXcd = kNumCu / kNumXcd;
  // all tiles in layer order (within a layer: blocks of tiles that share rows), cut into eight
  // equal runs: a layer stays on one XCD unless it straddles a cut, and the XCDs get the same
  // number of tiles
  std::vector<int4> all;
  for (size_t l = 0; l < layers.size(); ++l) {
    if (layers[l].provided || layers[l].kind != ADLOCO_KIND_LINEAR) continue;
    for_tiles_blocked((layers[l].d_out + kXt - 1) / kXt, (layers[l].d_in + kXt - 1) / kXt, 1,
                      [&](int e, int c) { all.push_back(int4{int(l), e * kXt, c * kXt, 0}); });
  }
  std::vector<std::vector<int4>> per(kNumXcd);
  for (int x = 0; x < kNumXcd; ++x)
    for (size_t i = all.size() * x / kNumXcd; i < all.size() * (x + 1) / kNumXcd; ++i)
      per[x].push_back(all[i]);
  split_tiles.clear();
  n_pieces = 0;
  std::vector<std::vector<int4>> fin(kNumXcd);
  for (int x = 0; x < kNumXcd; ++x) {
    const int n = int(per[x].size());
    const int full = n / kCuPerXcd * kCuPerXcd, left = n - full;
    const int S = left > 0 ? kCuPerXcd / left : 1;
    for (int i = 0; i < full; ++i) fin[x].push_back(per[x][i]);
    for (int i = full; i < n; ++i) {
      if (S < 2 || n_pieces + S > 0xffff) {
        fin[x].push_back(per[x][i]);
        continue;
      }
      split_tiles.push_back(int4{per[x][i].x, per[x][i].y, per[x][i].z, (S << 16) | n_pieces});
      for (int p = 0; p < S; ++p) {
        int4 e = per[x][i];
        e.w = (S << 24) | (p << 16) | (n_pieces + p);
        fin[x].push_back(e);
      }
      n_pieces += S;
    }
  }
  size_t slots = 0;
  for (auto& v : fin) slots = std::max(slots, v.size());
  out.assign(size_t(kNumXcd) * slots, int4{-1, 0, 0, 0});
  for (int x = 0; x < kNumXcd; ++x)
    for (size_t i = 0; i < fin[x].size(); ++i) out[x * slots + i] = fin[x][i];
  return int(slots);
}

hipError_t launch_wgrad_x(const LayerDev* layers, const void* tiles, int slots,
                          const void* split_tiles, int n_split, float* partials, long long rows,
                          int accumulate, int dtype, hipStream_t st) {
  if (slots <= 0) return hipSuccess;
  auto kern = dtype == ADLOCO_F16 ? wgrad_bf16_x_kernel<true> : wgrad_bf16_x_kernel<false>;
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kXlds);
    if (e != hipSuccess) return e;
  }
  WgradXArgs a{layers, static_cast<const int4*>(tiles), partials, slots, rows, accumulate};
  hipLaunchKernelGGL(kern, dim3(unsigned(slots * kNumXcd)), dim3(512), kXlds, st, a);
  if (n_split > 0)
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(unsigned(n_split) * (kXt / kXredRows)), dim3(256), 0, st, layers,
                       static_cast<const WgradSplitTile*>(split_tiles), partials, accumulate);
  return hipGetLastError();
}

hipError_t launch_wgrad(const LayerDev* layers, int n_layers, int n_blocks, long long rows,
                        int dtype, int accumulate, int variant, hipStream_t st) {
  if (n_blocks <= 0) return hipSuccess;
  WgradArgs a{layers, n_layers, rows, accumulate};
  if (is_16bit(dtype)) {
    const bool h = dtype == ADLOCO_F16;
    auto kern = variant == 0 ? (h ? wgrad_bf16_kernel<0, true> : wgrad_bf16_kernel<0, false>)
                             : (h ? wgrad_bf16_kernel<1, true> : wgrad_bf16_kernel<1, false>);
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(wgrad_f32_kernel, dim3(n_blocks), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace adloco
