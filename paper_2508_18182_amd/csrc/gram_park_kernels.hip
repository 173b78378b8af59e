// Per-sample gradient squared norms by the Gram identity, region form:
//   n_i = < A_i A_i^T , D_i D_i^T >_F ,  A_i [T, d_in], D_i [T, d_out] the token rows of sample i
// (the norm of the per-sample gradient that eq. 1 averages and the variance of Section 3.3.1 needs).
//
// Work item ("job") = one 256 x 256 region (p, q), p <= q, of the two T x T Gram matrices of one
// (layer, sample).  The job runs the two contractions one after the other through ONE set of
// accumulators: first the region of A A^T over d_in, whose fp32 result is parked in a private
// piece of device memory (every lane stores exactly the registers it later reloads, so no
// synchronisation is involved), then the region of D D^T over d_out in the same registers; the
// epilogue reloads the parked values, multiplies element by element and reduces.  One live
// accumulator set lets a workgroup of eight waves (two per SIMD, 128 x 64 wave tiles = 128
// accumulator registers) own a region four times the area of a 128 x 128 tile pair: per MFMA it
// stages a third less from L2 into LDS and reads a quarter fewer fragments from LDS than a kernel
// that keeps both sets live in 64 x 64 wave tiles.
//
// A region on the diagonal is symmetric: only its 36 upper 32 x 32 blocks are computed.  Its eight
// wave tiles hold 8, 8, 7, 7, 3, 3, 0, 0 of them; the waves are dealt to the tiles so that the two
// waves of a SIMD have 8 + 0 or 7 + 3 blocks.
//
// Staging: "units" of 256 rows x 64 elements (32 KiB, 128-byte rows, 16-byte pieces XOR-swizzled
// by the row so that fragment reads are conflict-free), global -> LDS directly, in a ring of five
// slots (160 KiB).  An off-diagonal region consumes two units (its p rows and its q rows) per
// k-chunk, a diagonal one a single unit.  One workgroup barrier per k-chunk, placed in front of
// the chunk's last k-step: there every wave has its fragments of the chunk in registers, so the
// chunk's slots are refilled at once, the loads issued between the MFMAs of that k-step.
//
// Launch: one persistent workgroup per CU walks a job list fixed by the host (list scheduling of
// the jobs in queue order on a cost model; workgroup w serves XCD w % 8).  All regions of one
// (layer, sample) are neighbours in one XCD's queue, so the rows they share come from that
// XCD's L2.  The first units of a workgroup's next job are requested before the epilogue of the
// current one, which runs while they travel.
#include <algorithm>

#include "common.h"

namespace adloco {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kPkRows = 256;                    // rows of a unit = edge of a region
constexpr int kPkKc = 64;                       // elements per staged row: four k-steps
constexpr int kPkRowB = kPkKc * 2;              // 128 bytes
constexpr int kPkUnit = kPkRows * kPkRowB;      // 32 KiB
constexpr int kPkSlots = 5;
constexpr int kPkLds = kPkSlots * kPkUnit;      // 160 KiB
constexpr int kPkBlockB = 32 * kPkRowB;         // one 32-row block inside a unit: 4 KiB
constexpr int kPkWaves = 8;
constexpr int kPkLoads = kPkUnit / 1024 / kPkWaves;   // wave-wide loads per wave and unit: 4
constexpr int kPkNB = 8;                        // blocks of a wave tile: 4 (rows) x 2 (columns)
static_assert(kGramParkFloats == kPkNB * 16 * 64, "parking area of a wave");

struct ParkArgs {
  const LayerDev* layers;
  const int* order;       // linear layers, heaviest first
  const int2* jobs;       // x: unit = position in `order` * B + sample; y: region
  const int* wg_start;    // [gridDim.x + 1] first job of every workgroup
  float* partials;        // [layer][sample][n_parts]
  float* park;            // [gridDim.x][8 waves][kGramParkFloats]
#ifdef PK_TIMING
  long long* dbg;         // [gridDim.x][8 waves][16]
#endif
  int B, T, nst, n_parts;
};

// s_waitcnt with lgkmcnt(0) and vmcnt(N): this wave's LDS reads have returned and all but its N
// youngest vector-memory operations have completed
template <int N> __device__ __forceinline__ void wait_lds_and_vm() {
  __builtin_amdgcn_s_waitcnt(0x0070 | (N & 0xf) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lds_and_vm_n(int n) {   // n: wave-uniform, a multiple of 4
  switch (n) {
    case 0: wait_lds_and_vm<0>(); break;
    case 4: wait_lds_and_vm<4>(); break;
    case 8: wait_lds_and_vm<8>(); break;
    case 12: wait_lds_and_vm<12>(); break;
    default: wait_lds_and_vm<16>(); break;
  }
}
__device__ __forceinline__ void pk_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
// A wave-uniform pointer the compiler may hold in vector registers, moved to scalar registers.
__device__ __forceinline__ const unsigned short* pk_uniform(const unsigned short* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane(unsigned(v));
  const unsigned hi = __builtin_amdgcn_readfirstlane(unsigned(v >> 32));
  return reinterpret_cast<const unsigned short*>((unsigned long long)hi << 32 | lo);
}
__device__ __forceinline__ float pk_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ---- wave shapes ------------------------------------------------------------------------------
// A wave tile is 4 x 2 blocks of 32 x 32: block b = row block b / 2, column block b % 2.  A shape
// says which of them a wave computes and with which weight: 2 off the diagonal of the Gram matrix
// (the mirrored block is not computed), 1 on it.
struct PkFull {            // every block, all off the diagonal
  static constexpr bool use(int) { return true; }
  static constexpr float weight(int) { return 2.f; }
};
struct PkSeven {           // wave tile whose row blocks 2, 3 meet its column blocks 0, 1 on the diagonal
  static constexpr bool use(int b) { return b != 6; }                       // (3, 0) lies below it
  static constexpr float weight(int b) { return (b == 4 || b == 7) ? 1.f : 2.f; }   // (2,0), (3,1)
};
struct PkThree {           // wave tile whose row blocks 0, 1 meet its column blocks 0, 1 on the diagonal
  static constexpr bool use(int b) { return b == 0 || b == 1 || b == 3; }   // (0,0), (0,1), (1,1)
  static constexpr float weight(int b) { return b == 1 ? 2.f : 1.f; }
};
struct PkIdle {            // wave tile below the diagonal: loads and barriers only
  static constexpr bool use(int) { return false; }
  static constexpr float weight(int) { return 0.f; }
};

#ifdef PK_TIMING
#define PK_T0(v) const long long v = __builtin_readcyclecounter()
#define PK_T1(v, f) const_cast<PkWave&>(w).f += __builtin_readcyclecounter() - v
#else
#define PK_T0(v)
#define PK_T1(v, f)
#endif

// Everything a wave carries from job to job.
struct PkWave {
#ifdef PK_TIMING
  long long t_wait = 0, t_park = 0, t_epi = 0, t_entry = 0, t_bar = 0, t_main0 = 0, t_main1 = 0, n_chunks0 = 0, n_chunks1 = 0;
#endif
  unsigned lds_base;       // LDS byte address of slot 0
  unsigned frag_off[4];    // per k-step: this lane's byte offset inside a 32-row block of a unit
  int lane, wave;
  f32x4* park;             // this lane's first parked float4
};

// One job as a wave sees it (wave-uniform but for the lane offsets).
struct PkJob {
  const unsigned short *a_p, *a_q;   // first element of the region's p rows / q rows in a ...
  const unsigned short *d_p, *d_q;   // ... and in delta
  int nka, nk, n_units;              // k-chunks of a, k-chunks in all, units in all
  int two;                           // 1: off-diagonal region, two units (p rows, q rows) per k-chunk
  int next_u, next_slot;             // next unit to request and the ring slot it goes to
  float* out;                        // this wave's partial sum
  unsigned off_a[kPkLoads], off_d[kPkLoads];   // lane offsets (bytes) of the wave's loads of a unit
};

// Workgroup's job j: which (layer, sample, region), and the addressing that follows from it.
__device__ __forceinline__ void pk_decode(const ParkArgs& g, const PkWave& w, int j, int next_slot,
                                          PkJob& J) {
  const int2 jb = g.jobs[j];
  const int oi = jb.x / g.B, sample = jb.x - oi * g.B;
  const int layer = g.order[oi];
  // regions are listed row by row: (0,0), (0,1) .. (0,nst-1), (1,1), ...
  int rem = jb.y, p = 0, len = g.nst;
  while (rem >= len) { rem -= len; ++p; --len; }
  const LayerDev L = g.layers[layer];
#ifdef PK_SAMPLE0   // timing experiment: every workgroup streams sample 0 (all loads hit the L2)
  const long long row_p = (long long)p * kPkRows;
#else
  const long long row_p = (long long)sample * g.T + (long long)p * kPkRows;
#endif
  const long long row_q = row_p + (long long)rem * kPkRows;
  J.a_p = reinterpret_cast<const unsigned short*>(L.a) + row_p * L.a_stride;
  J.a_q = reinterpret_cast<const unsigned short*>(L.a) + row_q * L.a_stride;
  J.d_p = reinterpret_cast<const unsigned short*>(L.delta) + row_p * L.delta_stride;
  J.d_q = reinterpret_cast<const unsigned short*>(L.delta) + row_q * L.delta_stride;
  J.two = rem != 0;
  J.nka = L.d_in / kPkKc;
  J.nk = J.nka + L.d_out / kPkKc;
  J.n_units = J.nk << J.two;
  J.next_u = 0;
  J.next_slot = next_slot;
  J.out = g.partials + (size_t(layer) * g.B + sample) * g.n_parts + jb.y * kPkWaves + w.wave;
  // wave-wide load i of a unit covers rows wave*32 + 8 i .. + 7: lane / 8 picks the row, lane % 8
  // the 16-byte position, which receives the piece position ^ f(row) of that row (f looks at the
  // row's place in its 32-row block only: the fragment reads of a block undo it)
  const int r = w.lane >> 3, pos = w.lane & 7;
#pragma unroll
  for (int i = 0; i < kPkLoads; ++i) {
    const int r32 = i * 8 + r;
    const int row = w.wave * 32 + r32;                           // row inside the unit
    const int piece = pos ^ ((r32 ^ (r32 >> 3)) & 7);
    J.off_a[i] = unsigned((long long)row * L.a_stride + piece * 8) * 2u;
    J.off_d[i] = unsigned((long long)row * L.delta_stride + piece * 8) * 2u;
  }
}

__device__ __forceinline__ int pk_slot_plus(int s, int d) { s += d; return s >= kPkSlots ? s - kPkSlots : s; }

// Address of the job's next unit: first element of its first row (global), and where this wave's
// share of it goes in LDS.
__device__ __forceinline__ const unsigned short* pk_unit_base(const PkJob& J) {
  const int c = J.next_u >> J.two;
  const bool q_side = (J.next_u & J.two) != 0;
  return pk_uniform(c < J.nka ? (q_side ? J.a_q : J.a_p) + c * kPkKc
                              : (q_side ? J.d_q : J.d_p) + (c - J.nka) * kPkKc);
}
__device__ __forceinline__ unsigned pk_unit_dst(const PkWave& w, const PkJob& J) {
  return __builtin_amdgcn_readfirstlane(w.lds_base + unsigned(J.next_slot) * kPkUnit +
                                        unsigned(w.wave) * (32 * kPkRowB));
}
__device__ __forceinline__ void pk_unit_done(PkJob& J) {
  ++J.next_u;
  J.next_slot = pk_slot_plus(J.next_slot, 1);
}
// Fill the (empty) ring with the job's first units.
__device__ __forceinline__ void pk_fill_ring(const PkWave& w, PkJob& J) {
  for (int i = 0; i < kPkSlots && J.next_u < J.n_units; ++i) {
    const bool in_a = (J.next_u >> J.two) < J.nka;
    const unsigned short* base = pk_unit_base(J);
    const unsigned dst = pk_unit_dst(w, J);
    if (in_a) {
#pragma unroll
      for (int l = 0; l < kPkLoads; ++l) direct_load_lds16_s(J.off_a[l], base, dst + l * 1024);
    } else {
#pragma unroll
      for (int l = 0; l < kPkLoads; ++l) direct_load_lds16_s(J.off_d[l], base, dst + l * 1024);
    }
    pk_unit_done(J);
  }
}

// One job for one wave whose tile is (wm, wn): row blocks 4 wm .. 4 wm + 3 of the p unit, column
// blocks 2 wn, 2 wn + 1 of the q unit (the p unit again for a region on the diagonal).  On entry the
// first units of job J have been requested (the first in slot `slot0`); on exit the first units of
// the workgroup's next job, if there is one, have been requested and J describes that job.  Every
// wave of the workgroup passes the same barriers whatever its shape.
template <bool F16, typename S>
__device__ __forceinline__ void pk_run_job(const ParkArgs& g, const PkWave& w, PkJob& J, int& slot0,
                                           int wm, int wn, int j_next, int j_end) {
  constexpr int NB = kPkNB;
  constexpr bool kIdle = !(S::use(0) || S::use(1) || S::use(2) || S::use(3) || S::use(4) || S::use(5) ||
                           S::use(6) || S::use(7));
  const int upc = 1 + J.two;                         // units per k-chunk
  const int nka = J.nka, nk = J.nk;
  typedef __attribute__((address_space(3))) const u32x4* lds_v4;
  // fragments of a k-step: f[0..3] row blocks, f[4..5] column blocks
  auto read_frags = [&](int slot_p, int slot_q, int ks, bf16x8 (&f)[6]) {
    if (kIdle) return;
    const unsigned bp = w.lds_base + unsigned(slot_p) * kPkUnit + w.frag_off[ks] + unsigned(wm) * (4 * kPkBlockB);
    const unsigned bq = w.lds_base + unsigned(slot_q) * kPkUnit + w.frag_off[ks] + unsigned(wn) * (2 * kPkBlockB);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (S::use(2 * i) || S::use(2 * i + 1))
        f[i] = __builtin_bit_cast(bf16x8, *(lds_v4)(size_t)(bp + unsigned(i) * kPkBlockB));
#pragma unroll
    for (int i = 0; i < 2; ++i)
      if (S::use(i) || S::use(2 + i) || S::use(4 + i) || S::use(6 + i))
        f[4 + i] = __builtin_bit_cast(bf16x8, *(lds_v4)(size_t)(bq + unsigned(i) * kPkBlockB));
  };
  f32x16 acc[NB];
  auto mfma_one = [&](const bf16x8 (&f)[6], int b) {
    if (S::use(b)) acc[b] = mfma_32x32x16<F16>(f[b >> 1], f[4 + (b & 1)], acc[b]);
  };
  auto mfma_all = [&](const bf16x8 (&f)[6]) {
#pragma unroll
    for (int b = 0; b < NB; ++b) mfma_one(f, b);
    if (!kIdle) {
      // issue order: MFMA, LDS read, MFMA, LDS read, ...
#pragma unroll
      for (int i = 0; i < 6; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
  };
  // Request the job's next unit (four wave-wide loads of 1 KiB per wave) into a slot that has just
  // been released, two loads behind each of the MFMAs b0, b0 + 1 of fragment set f.
  auto refill_unit = [&](const bf16x8 (&f)[6], int b0) {
    const bool have = J.next_u < J.n_units;
    const bool in_a = (J.next_u >> J.two) < nka;
    const unsigned short* base = pk_unit_base(J);
    const unsigned dst = pk_unit_dst(w, J);
#pragma unroll
    for (int i = 0; i < kPkLoads; i += 2) {
      if (have) {
        if (in_a) {
          direct_load_lds16_s(J.off_a[i], base, dst + i * 1024);
          direct_load_lds16_s(J.off_a[i + 1], base, dst + (i + 1) * 1024);
        } else {
          direct_load_lds16_s(J.off_d[i], base, dst + i * 1024);
          direct_load_lds16_s(J.off_d[i + 1], base, dst + (i + 1) * 1024);
        }
      }
      mfma_one(f, b0 + i / 2);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (have) pk_unit_done(J);
  };

#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

  // chunk 0 has landed for everybody
  PK_T0(te);
  wait_lds_and_vm_n((J.next_u - upc) * kPkLoads);
  pk_barrier();
  PK_T1(te, t_entry);
  PK_T0(tm);
  int slot_c = slot0;                                 // slot of the first unit of chunk c
  bf16x8 fr[2][6];
  const int two = J.two;
  auto slot_q2 = [&](int sp) { return two ? pk_slot_plus(sp, 1) : sp; };
  read_frags(slot_c, slot_q2(slot_c), 0, fr[0]);

  auto chunk_step = [&](int c) {
    const int sp = slot_c, sq = slot_q2(slot_c);
    read_frags(sp, sq, 1, fr[1]);
    mfma_all(fr[0]);
    read_frags(sp, sq, 2, fr[0]);
    mfma_all(fr[1]);
    read_frags(sp, sq, 3, fr[1]);
    mfma_all(fr[0]);
    const int slot_n = pk_slot_plus(slot_c, upc);
    if (c + 1 < nk) {
      // my fragments of chunk c are in registers and my share of chunk c + 1 has landed ...
      PK_T0(tw);
      wait_lds_and_vm_n((J.next_u - (c + 2) * upc) * kPkLoads);
      PK_T1(tw, t_wait);
      PK_T0(tb);
      pk_barrier();            // ... and so for everybody: the slots of chunk c are free
      PK_T1(tb, t_bar);
      refill_unit(fr[1], 0);
      if (two) refill_unit(fr[1], 2); else { mfma_one(fr[1], 2); mfma_one(fr[1], 3); }
      __builtin_amdgcn_sched_barrier(0);
      read_frags(slot_n, slot_q2(slot_n), 0, fr[0]);
#pragma unroll
      for (int b = 4; b < NB; ++b) mfma_one(fr[1], b);
      if (!kIdle) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    } else {
      mfma_all(fr[1]);
    }
    slot_c = slot_n;
  };
  int c = 0;
  for (; c < nka; ++c) chunk_step(c);
  // the region of A A^T is complete: park it, and start the region of D D^T from zero
  PK_T0(tp);
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    if (!S::use(b)) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const f32x4 x = {acc[b][4 * v], acc[b][4 * v + 1], acc[b][4 * v + 2], acc[b][4 * v + 3]};
#ifndef PK_NOPARK
      w.park[(b * 4 + v) * 64] = x;
#else
      asm volatile("" :: "v"(x));
#endif
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
  }
  PK_T1(tp, t_park);
  for (; c < nk; ++c) chunk_step(c);
  PK_T0(tq);
#ifdef PK_TIMING
  if (two) { const_cast<PkWave&>(w).t_main1 += tq - tm; const_cast<PkWave&>(w).n_chunks1 += nk; }
  else { const_cast<PkWave&>(w).t_main0 += tq - tm; const_cast<PkWave&>(w).n_chunks0 += nk; }
#endif

  // ---- the next job's first units are requested before this job's epilogue, which runs while
  // they travel
  float* const out = J.out;
  slot0 = slot_c;
  if (j_next < j_end) {
    pk_decode(g, w, j_next, slot_c, J);
    pk_barrier();                                     // every wave has its last fragments
    pk_fill_ring(w, J);
  }

  // ---- epilogue: < A A^T , D D^T > over this wave's blocks
  float s = 0.f;
  if (!kIdle) {
    // the parked values come back four blocks at a time (64 registers)
#pragma unroll
    for (int b0 = 0; b0 < NB; b0 += 4) {
      f32x4 x[4][4];
#pragma unroll
      for (int b = b0; b < b0 + 4; ++b)
        if (S::use(b)) {
#pragma unroll
          for (int v = 0; v < 4; ++v)
#ifndef PK_NOPARK
            x[b - b0][v] = w.park[(b * 4 + v) * 64];
#else
            x[b - b0][v] = f32x4{1.f, 2.f, 3.f, float(v)};
#endif
        }
#pragma unroll
      for (int b = b0; b < b0 + 4; ++b)
        if (S::use(b)) {
          float sb = 0.f;
#pragma unroll
          for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e) sb += x[b - b0][v][e] * acc[b][4 * v + e];
          s += sb * S::weight(b);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    s = pk_wave_sum(s);
  }
  if (w.lane == 0) *out = s;
  PK_T1(tq, t_epi);
}

template <bool F16>
__global__ __launch_bounds__(512, 1) void gram_park_kernel(ParkArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  PkWave w;
  w.lane = threadIdx.x & 63;
  w.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  w.lds_base = lds_address(lds);
  {
    const int r32 = w.lane & 31, kg = w.lane >> 5;
    const int sw = (r32 ^ (r32 >> 3)) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) w.frag_off[ks] = unsigned(r32 * kPkRowB + (((ks * 2 + kg) ^ sw) * 16));
  }
  w.park = reinterpret_cast<f32x4*>(g.park + (size_t(blockIdx.x) * kPkWaves + w.wave) * kGramParkFloats) + w.lane;
  const int j0 = g.wg_start[blockIdx.x], j1 = g.wg_start[blockIdx.x + 1];
  if (j0 >= j1) return;
#ifdef PK_TIMING
  const long long t_begin = __builtin_readcyclecounter();
  const long long w_begin = wall_clock64();
#endif
  PkJob J;
  pk_decode(g, w, j0, 0, J);
  pk_fill_ring(w, J);
  int slot0 = 0;
  // Wave tiles of a region on the diagonal, by wave: the two waves of a SIMD (w and w + 4) take a
  // full tile and one below the diagonal, or a tile of seven blocks and one of three.
  //   wave:  0      1      2      3      4      5      6      7
  //   tile: (0,2)  (0,3)  (0,1)  (1,3)  (1,0)  (1,1)  (0,0)  (1,2)
  for (int j = j0; j < j1; ++j) {
    if (J.two) {
      pk_run_job<F16, PkFull>(g, w, J, slot0, w.wave >> 2, w.wave & 3, j + 1, j1);
    } else {
      switch (w.wave) {
        case 0: pk_run_job<F16, PkFull>(g, w, J, slot0, 0, 2, j + 1, j1); break;
        case 1: pk_run_job<F16, PkFull>(g, w, J, slot0, 0, 3, j + 1, j1); break;
        case 2: pk_run_job<F16, PkSeven>(g, w, J, slot0, 0, 1, j + 1, j1); break;
        case 3: pk_run_job<F16, PkSeven>(g, w, J, slot0, 1, 3, j + 1, j1); break;
        case 6: pk_run_job<F16, PkThree>(g, w, J, slot0, 0, 0, j + 1, j1); break;
        case 7: pk_run_job<F16, PkThree>(g, w, J, slot0, 1, 2, j + 1, j1); break;
        default: pk_run_job<F16, PkIdle>(g, w, J, slot0, 1, 0, j + 1, j1); break;
      }
    }
  }
#ifdef PK_TIMING
  if (w.lane == 0) {
    long long* d = g.dbg + (size_t(blockIdx.x) * kPkWaves + w.wave) * 16;
    d[0] = __builtin_readcyclecounter() - t_begin;
    d[1] = w.t_wait; d[2] = w.t_park; d[3] = w.t_epi; d[4] = w.t_entry; d[5] = wall_clock64() - w_begin; d[6] = j1 - j0; d[7] = w.t_bar; d[8] = w.t_main0; d[9] = w.t_main1; d[10] = w.n_chunks0; d[11] = w.n_chunks1;
  }
#endif
}

}  // namespace

// Cost of a job in MFMA issue slots of one SIMD (the unit of the host's list scheduling): blocks
// per wave and k-step times k-steps, plus what prologue, parking and epilogue take.
static long long park_job_cost(const LayerDev& L, bool diag) {
  const long long ksteps = (L.d_in + L.d_out) / 16;
  return (diag ? 10 : 16) * ksteps + 400;
}

int gram_park_grid() { return kNumCu; }
size_t gram_park_scratch_floats() { return size_t(kNumCu) * kPkWaves * kGramParkFloats; }
int gram_park_parts(int T) { const int nst = T / kPkRows; return nst * (nst + 1) / 2 * kPkWaves; }
bool gram_park_eligible(int T) { return T >= kPkRows && T % kPkRows == 0; }

// Job lists of the persistent workgroups.  Units (layer in `order`, sample) are dealt round-robin to
// the XCDs; inside an XCD's queue the regions of a unit are neighbours; a job goes to the workgroup
// of that XCD which the cost model sees free first.
void make_park_jobs(const std::vector<LayerDev>& layers, const std::vector<int>& order, int B, int T,
                    std::vector<int2>& jobs, std::vector<int>& wg_start) {
  const int nst = T / kPkRows, nreg = nst * (nst + 1) / 2;
  const int per_xcd = kNumCu / kNumXcd;
  std::vector<std::vector<int2>> lists(kNumCu);
  std::vector<char> reg_diag(nreg);
  {
    int r = 0;
    for (int p = 0; p < nst; ++p)
      for (int q = p; q < nst; ++q) reg_diag[r++] = p == q;
  }
  const long long units = (long long)order.size() * B;
  for (int x = 0; x < kNumXcd; ++x) {
    std::vector<long long> busy(per_xcd, 0);
    for (long long u = x; u < units; u += kNumXcd) {
      const LayerDev& L = layers[order[size_t(u / B)]];
      for (int r = 0; r < nreg; ++r) {
        const int i = int(std::min_element(busy.begin(), busy.end()) - busy.begin());
        busy[i] += park_job_cost(L, reg_diag[r]);
        lists[size_t(i) * kNumXcd + x].push_back(make_int2(int(u), r));
      }
    }
  }
  jobs.clear();
  wg_start.assign(kNumCu + 1, 0);
  for (int w = 0; w < kNumCu; ++w) {
    wg_start[w] = int(jobs.size());
    jobs.insert(jobs.end(), lists[w].begin(), lists[w].end());
  }
  wg_start[kNumCu] = int(jobs.size());
}

#ifdef PK_TIMING
long long* g_pk_dbg = nullptr;
#endif
hipError_t launch_gram_park(const GramLaunch& l, const int2* jobs, const int* wg_start, float* park,
                            hipStream_t st) {
  auto kern = l.dtype == ADLOCO_F16 ? gram_park_kernel<true> : gram_park_kernel<false>;
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kPkLds);
    if (e != hipSuccess) return e;
  }
  ParkArgs a;
  a.layers = l.layers;
  a.order = l.order;
  a.jobs = jobs;
  a.wg_start = wg_start;
  a.partials = l.partials;
  a.park = park;
  a.B = l.B;
  a.T = l.T;
  a.nst = l.T / kPkRows;
  a.n_parts = l.n_pairs;
#ifdef PK_TIMING
  a.dbg = g_pk_dbg;
#endif
  hipLaunchKernelGGL(kern, dim3(kNumCu), dim3(64 * kPkWaves), kPkLds, st, a);
  return hipGetLastError();
}

}  // namespace adloco
