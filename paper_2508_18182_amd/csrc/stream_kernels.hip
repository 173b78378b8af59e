// HBM-streaming kernels: the multi-instance outer step (Algorithm 3: pseudo-gradient,
// OuterOpt, worker reset) and the trainer merge (Algorithm 2).  Every parameter is read
// once from each input and written once to each output; arithmetic is fp64 in registers
// (free next to the memory traffic) and rounded to fp32 once.
#include <cmath>

#include "common.h"

namespace adloco {

struct OuterArgs {
  float* theta;
  float* mom;         // may be null (mu == 0)
  float* pg;          // may be null
  float* inst[ADLOCO_MAX_INSTANCES];
  size_t n_vec;       // number of float4 elements handled by the vector kernel
  size_t n;           // total number of floats
  double lr, mu, inv_m;
  int nesterov, broadcast;
};

struct MergeArgs {
  float* x[ADLOCO_MAX_INSTANCES];
  double w[ADLOCO_MAX_INSTANCES];   // b_j
  double inv_wsum;
  size_t n_vec, n;
  int rep;
};

typedef float __attribute__((ext_vector_type(4))) f32x4;

__device__ __forceinline__ f32x4 ld_stream(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}

template <int M>
__device__ __forceinline__ void outer_elem(const OuterArgs& a, double th, double buf,
                                           const double (&x)[M], double& th_new,
                                           double& buf_new, double& delta) {
  // Delta = (1/M) sum_m (theta_outer - theta_m): differences first, as Algorithm 3 writes it
  double s = 0.0;
#pragma unroll
  for (int m = 0; m < M; ++m) s += th - x[m];
  delta = s * a.inv_m;
  buf_new = a.mu * buf + delta;
  const double step = a.nesterov ? delta + a.mu * buf_new : buf_new;
  th_new = th - a.lr * step;
}

// One float4 of every stream per thread and one single-wave workgroup per 1 KiB of every stream:
// on MI355X a plain (non-persistent) grid of small workgroups measured faster than 256-thread
// workgroups (+3 %) and than a grid-stride loop over fewer workgroups (+15 %); marking every
// load non-temporal, also those of the vectors written back in place, gave another 6 %.
// Fewer resident waves gave the most: with about 8 waves per compute unit instead of the 32
// that fit, the requests reaching HBM stay closer together (79 % -> 86 % of 8 TB/s for M = 4).
// Residency is capped by giving each workgroup a dynamic LDS allocation it never touches.
constexpr int kStreamThreads = 64;
constexpr int kLdsPerCu = 160 * 1024;
// `blocks_per_cu` > 0 is the tuning knob; 0 picks the count that measured best: 48 / load_streams
// + 2 waves per compute unit (each wave requests 1 KiB from each of `load_streams` vectors), i.e.
// 56-70 KiB of loads in flight (14 waves for 4 streams, 10 for 6, 8 for 8, 7 for 10).
static inline unsigned stream_lds_bytes(int blocks_per_cu, int load_streams) {
  if (blocks_per_cu < 1) {
    blocks_per_cu = (48 + load_streams / 2) / load_streams + 2;
    if (blocks_per_cu < 4) blocks_per_cu = 4;
  }
  if (blocks_per_cu >= 32) return 0;            // no cap
  // a little less than an even share, so that allocation rounding cannot cost a workgroup
  unsigned b = unsigned(kLdsPerCu / blocks_per_cu - 512) / 256u * 256u;
  return b > 65536u ? 65536u : b;
}

template <int M>
__global__ __launch_bounds__(kStreamThreads) void outer_step_vec_kernel(OuterArgs a) {
  const size_t v = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (v < a.n_vec) {
    const size_t e = v * 4;
    f32x4 th = ld_stream(a.theta + e);
    f32x4 bf = {0.f, 0.f, 0.f, 0.f};
    if (a.mom) bf = ld_stream(a.mom + e);
    f32x4 xs[M];
#pragma unroll
    for (int m = 0; m < M; ++m) xs[m] = ld_stream(a.inst[m] + e);
    f32x4 th_o, bf_o, pg_o;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      double x[M];
#pragma unroll
      for (int m = 0; m < M; ++m) x[m] = double(xs[m][c]);
      double tn, bn, dl;
      outer_elem<M>(a, double(th[c]), double(bf[c]), x, tn, bn, dl);
      th_o[c] = float(tn);
      bf_o[c] = float(bn);
      pg_o[c] = float(dl);
    }
    __builtin_nontemporal_store(th_o, reinterpret_cast<f32x4*>(a.theta + e));
    if (a.mom) __builtin_nontemporal_store(bf_o, reinterpret_cast<f32x4*>(a.mom + e));
    if (a.pg) __builtin_nontemporal_store(pg_o, reinterpret_cast<f32x4*>(a.pg + e));
    if (a.broadcast) {
#pragma unroll
      for (int m = 0; m < M; ++m)
        __builtin_nontemporal_store(th_o, reinterpret_cast<f32x4*>(a.inst[m] + e));
    }
  }
}

// Scalar path: the tail after the last whole float4 (first = n_vec*4) or, for pointers that
// are not 16-byte aligned, the whole vector (first = 0).
template <int M>
__global__ __launch_bounds__(256) void outer_step_scalar_kernel(OuterArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride) {
    double x[M];
#pragma unroll
    for (int m = 0; m < M; ++m) x[m] = double(a.inst[m][e]);
    double tn, bn, dl;
    outer_elem<M>(a, double(a.theta[e]), a.mom ? double(a.mom[e]) : 0.0, x, tn, bn, dl);
    a.theta[e] = float(tn);
    if (a.mom) a.mom[e] = float(bn);
    if (a.pg) a.pg[e] = float(dl);
    if (a.broadcast) {
#pragma unroll
      for (int m = 0; m < M; ++m) a.inst[m][e] = float(tn);
    }
  }
}

template <int S>
__device__ __forceinline__ double merge_elem(const MergeArgs& a, const double (&x)[S]) {
  // x_merge = w_sum^{-1} sum_j b_j x_j
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < S; ++j) s += a.w[j] * x[j];
  return s * a.inv_wsum;
}

template <int S>
__global__ __launch_bounds__(kStreamThreads) void merge_vec_kernel(MergeArgs a) {
  const size_t v = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (v < a.n_vec) {
    const size_t e = v * 4;
    f32x4 xs[S];
#pragma unroll
    for (int j = 0; j < S; ++j) xs[j] = ld_stream(a.x[j] + e);
    f32x4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      double x[S];
#pragma unroll
      for (int j = 0; j < S; ++j) x[j] = double(xs[j][c]);
      o[c] = float(merge_elem<S>(a, x));
    }
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(a.x[a.rep] + e));
  }
}

template <int S>
__global__ __launch_bounds__(256) void merge_scalar_kernel(MergeArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride) {
    double x[S];
#pragma unroll
    for (int j = 0; j < S; ++j) x[j] = double(a.x[j][e]);
    a.x[a.rep][e] = float(merge_elem<S>(a, x));
  }
}

struct InnerArgs {
  float* theta;
  float* m;
  float* v;
  const float* grad;
  size_t n_vec, n;
  double grad_scale, decay_keep, beta1, beta2, omb1, omb2, step_size, inv_sqrt_bc2, eps;
};

// AdamW on one parameter: decay_keep = 1 - lr*weight_decay, step_size = lr / (1 - beta1^step),
// inv_sqrt_bc2 = 1 / sqrt(1 - beta2^step).
__device__ __forceinline__ void inner_elem(const InnerArgs& a, double x, double m, double v,
                                           double g0, double& xo, double& mo, double& vo) {
  const double g = a.grad_scale * g0;
  mo = a.beta1 * m + a.omb1 * g;
  vo = a.beta2 * v + a.omb2 * g * g;
  const double denom = sqrt(vo) * a.inv_sqrt_bc2 + a.eps;
  xo = x * a.decay_keep - a.step_size * mo / denom;
}

__global__ __launch_bounds__(kStreamThreads) void inner_step_vec_kernel(InnerArgs a) {
  const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < a.n_vec) {
    const size_t e = i * 4;
    const f32x4 x = ld_stream(a.theta + e), m = ld_stream(a.m + e), v = ld_stream(a.v + e),
                g = ld_stream(a.grad + e);
    f32x4 xo, mo, vo;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      double xn, mn, vn;
      inner_elem(a, double(x[c]), double(m[c]), double(v[c]), double(g[c]), xn, mn, vn);
      xo[c] = float(xn);
      mo[c] = float(mn);
      vo[c] = float(vn);
    }
    __builtin_nontemporal_store(xo, reinterpret_cast<f32x4*>(a.theta + e));
    __builtin_nontemporal_store(mo, reinterpret_cast<f32x4*>(a.m + e));
    __builtin_nontemporal_store(vo, reinterpret_cast<f32x4*>(a.v + e));
  }
}

__global__ __launch_bounds__(256) void inner_step_scalar_kernel(InnerArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride) {
    double xn, mn, vn;
    inner_elem(a, double(a.theta[e]), double(a.m[e]), double(a.v[e]), double(a.grad[e]), xn, mn, vn);
    a.theta[e] = float(xn);
    a.m[e] = float(mn);
    a.v[e] = float(vn);
  }
}

// ---------------------------------------------------------------------------------------
// Instance drifts stored in bf16.  What Algorithm 3 averages is d_m = x^{(t-1)} - x_m^{(t,H)}; stored
// in bf16 it costs 2 bytes per instance and parameter instead of 4 and carries a rounding error of
// at most 2^-8 of the drift itself (a bf16 copy of the parameters would lose the drift altogether).
// Outer model and momentum stay fp32.  Eight parameters per thread: two 16-byte loads of every fp32
// stream, one of every drift.
// ---------------------------------------------------------------------------------------
typedef unsigned short __attribute__((ext_vector_type(4))) u16x4;

// fp32 -> bf16, round to nearest, ties to even (NaN keeps a quiet bit)
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float x) {
  const unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ double bf16_to_f64(unsigned short h) {
  return double(__uint_as_float(unsigned(h) << 16));
}
// A wave handles 512 consecutive parameters as two halves of 256: lane l takes elements 4 l .. 4 l + 3
// of each half, so that every load and store instruction of the wave covers one contiguous run (1 KiB
// of an fp32 vector, 512 bytes of a bf16 one) and no cache line is written in pieces.
__device__ __forceinline__ size_t drift_elem0(size_t v, int half) {
  return (v >> 6) * 512 + size_t(half) * 256 + (v & 63) * 4;
}

struct PackArgs {
  const float* theta;
  const float* inst;
  unsigned short* out;
  size_t n_grp, n;      // groups of eight handled by the vector kernel (a multiple of 64); total elements
};

__global__ __launch_bounds__(kStreamThreads) void pack_drift_vec_kernel(PackArgs a) {
  const size_t v = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (v >= a.n_grp) return;
  f32x4 t[2], x[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    t[h] = ld_stream(a.theta + drift_elem0(v, h));
    x[h] = ld_stream(a.inst + drift_elem0(v, h));
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    u16x4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = f32_to_bf16_rne(t[h][c] - x[h][c]);   // fp32 difference, one rounding
    __builtin_nontemporal_store(o, reinterpret_cast<u16x4*>(a.out + drift_elem0(v, h)));
  }
}
__global__ __launch_bounds__(256) void pack_drift_scalar_kernel(PackArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride)
    a.out[e] = f32_to_bf16_rne(a.theta[e] - a.inst[e]);
}

struct OuterDriftArgs {
  float* theta;
  float* mom;         // may be null (mu == 0)
  float* pg;          // may be null
  unsigned short* drift[ADLOCO_MAX_INSTANCES];
  size_t n_grp, n;
  double lr, mu, inv_m;
  int nesterov, broadcast;
};

template <int M>
__device__ __forceinline__ void outer_drift_elem(const OuterDriftArgs& a, double th, double buf,
                                                 const double (&d)[M], double& th_new, double& buf_new,
                                                 double& delta) {
  double s = 0.0;
#pragma unroll
  for (int m = 0; m < M; ++m) s += d[m];
  delta = s * a.inv_m;
  buf_new = a.mu * buf + delta;
  const double step = a.nesterov ? delta + a.mu * buf_new : buf_new;
  th_new = th - a.lr * step;
}

template <int M>
__global__ __launch_bounds__(kStreamThreads) void outer_step_drift_vec_kernel(OuterDriftArgs a) {
  const size_t v = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (v >= a.n_grp) return;
  f32x4 th[2], bf[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  u16x4 ds[2][M];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const size_t e = drift_elem0(v, h);
    th[h] = ld_stream(a.theta + e);
    if (a.mom) bf[h] = ld_stream(a.mom + e);
#pragma unroll
    for (int m = 0; m < M; ++m) ds[h][m] = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(a.drift[m] + e));
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const size_t e = drift_elem0(v, h);
    f32x4 th_o, bf_o, pg_o;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      double d[M];
#pragma unroll
      for (int m = 0; m < M; ++m) d[m] = bf16_to_f64(ds[h][m][c]);
      double tn, bn, dl;
      outer_drift_elem<M>(a, double(th[h][c]), double(bf[h][c]), d, tn, bn, dl);
      th_o[c] = float(tn);
      bf_o[c] = float(bn);
      pg_o[c] = float(dl);
    }
    __builtin_nontemporal_store(th_o, reinterpret_cast<f32x4*>(a.theta + e));
    if (a.mom) __builtin_nontemporal_store(bf_o, reinterpret_cast<f32x4*>(a.mom + e));
    if (a.pg) __builtin_nontemporal_store(pg_o, reinterpret_cast<f32x4*>(a.pg + e));
    if (a.broadcast) {          // worker reset x_m <- x: every drift is zero again
      const u16x4 z = {0, 0, 0, 0};
#pragma unroll
      for (int m = 0; m < M; ++m) __builtin_nontemporal_store(z, reinterpret_cast<u16x4*>(a.drift[m] + e));
    }
  }
}

template <int M>
__global__ __launch_bounds__(256) void outer_step_drift_scalar_kernel(OuterDriftArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride) {
    double d[M];
#pragma unroll
    for (int m = 0; m < M; ++m) d[m] = bf16_to_f64(a.drift[m][e]);
    double tn, bn, dl;
    outer_drift_elem<M>(a, double(a.theta[e]), a.mom ? double(a.mom[e]) : 0.0, d, tn, bn, dl);
    a.theta[e] = float(tn);
    if (a.mom) a.mom[e] = float(bn);
    if (a.pg) a.pg[e] = float(dl);
    if (a.broadcast) {
#pragma unroll
      for (int m = 0; m < M; ++m) a.drift[m][e] = 0;
    }
  }
}

struct MergeDriftArgs {
  float* x_rep;
  const unsigned short* drift[ADLOCO_MAX_INSTANCES];
  double w[ADLOCO_MAX_INSTANCES];   // b_j of the others
  double inv_wsum;                  // 1 / (b_r + sum_j b_j)
  size_t n_grp, n;
};

template <int S>
__global__ __launch_bounds__(kStreamThreads) void merge_drift_vec_kernel(MergeDriftArgs a) {
  const size_t v = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (v >= a.n_grp) return;
  f32x4 x[2];
  u16x4 ds[2][S];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const size_t e = drift_elem0(v, h);
    x[h] = ld_stream(a.x_rep + e);
#pragma unroll
    for (int j = 0; j < S; ++j) ds[h][j] = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(a.drift[j] + e));
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    f32x4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      // x_merge = x_r - sum_{j != r} b_j d_j / sum_j b_j
      double s = 0.0;
#pragma unroll
      for (int j = 0; j < S; ++j) s += a.w[j] * bf16_to_f64(ds[h][j][c]);
      o[c] = float(double(x[h][c]) - s * a.inv_wsum);
    }
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(a.x_rep + drift_elem0(v, h)));
  }
}

template <int S>
__global__ __launch_bounds__(256) void merge_drift_scalar_kernel(MergeDriftArgs a, size_t first) {
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (size_t e = first + size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < a.n; e += stride) {
    double s = 0.0;
#pragma unroll
    for (int j = 0; j < S; ++j) s += a.w[j] * bf16_to_f64(a.drift[j][e]);
    a.x_rep[e] = float(double(a.x_rep[e]) - s * a.inv_wsum);
  }
}

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Scalar (tail / unaligned) kernels use a grid-stride loop over a bounded grid.
static inline unsigned grid_for(size_t work_items, int blocks_per_cu) {
  size_t need = (work_items + 255) / 256;
  size_t cap = size_t(kNumCu) * (blocks_per_cu > 0 ? blocks_per_cu : 8);
  if (need < 1) need = 1;
  return static_cast<unsigned>(need < cap ? need : cap);
}
constexpr size_t kMaxVecPerLaunch = size_t(0x7fffffff) * kStreamThreads;   // grid.x limit of one launch

template <int M>
static hipError_t launch_outer_m(const OuterArgs& a, bool vec, int bpc, hipStream_t st) {
  if (vec) {
    if (a.n_vec > 0)
      hipLaunchKernelGGL(outer_step_vec_kernel<M>,
                         dim3(unsigned((a.n_vec + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(bpc, M + (a.mom ? 2 : 1)), st, a);
    if (a.n_vec * 4 < a.n)
      hipLaunchKernelGGL(outer_step_scalar_kernel<M>, dim3(1), dim3(256), 0, st, a, a.n_vec * 4);
  } else {
    hipLaunchKernelGGL(outer_step_scalar_kernel<M>, dim3(grid_for(a.n, bpc)), dim3(256), 0, st, a,
                       size_t(0));
  }
  return hipGetLastError();
}

template <int S>
static hipError_t launch_merge_s(const MergeArgs& a, bool vec, int bpc, hipStream_t st) {
  if (vec) {
    if (a.n_vec > 0)
      hipLaunchKernelGGL(merge_vec_kernel<S>,
                         dim3(unsigned((a.n_vec + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(bpc, S), st, a);
    if (a.n_vec * 4 < a.n)
      hipLaunchKernelGGL(merge_scalar_kernel<S>, dim3(1), dim3(256), 0, st, a, a.n_vec * 4);
  } else {
    hipLaunchKernelGGL(merge_scalar_kernel<S>, dim3(grid_for(a.n, bpc)), dim3(256), 0, st, a,
                       size_t(0));
  }
  return hipGetLastError();
}

template <int M>
static hipError_t launch_outer_drift_m(const OuterDriftArgs& a, bool vec, int bpc, hipStream_t st) {
  if (vec) {
    if (a.n_grp > 0)
      hipLaunchKernelGGL(outer_step_drift_vec_kernel<M>,
                         dim3(unsigned((a.n_grp + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(bpc, M + (a.mom ? 2 : 1)), st, a);   // measured best: 7 per CU at M = 8
    if (a.n_grp * 8 < a.n)
      hipLaunchKernelGGL(outer_step_drift_scalar_kernel<M>, dim3(1), dim3(256), 0, st, a, a.n_grp * 8);
  } else {
    hipLaunchKernelGGL(outer_step_drift_scalar_kernel<M>, dim3(grid_for(a.n, bpc)), dim3(256), 0, st, a,
                       size_t(0));
  }
  return hipGetLastError();
}

template <int S>
static hipError_t launch_merge_drift_s(const MergeDriftArgs& a, bool vec, int bpc, hipStream_t st) {
  if (vec) {
    if (a.n_grp > 0)
      hipLaunchKernelGGL(merge_drift_vec_kernel<S>,
                         dim3(unsigned((a.n_grp + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(bpc, S + 4), st, a);   // measured best: 6 per CU at S = 8
    if (a.n_grp * 8 < a.n)
      hipLaunchKernelGGL(merge_drift_scalar_kernel<S>, dim3(1), dim3(256), 0, st, a, a.n_grp * 8);
  } else {
    hipLaunchKernelGGL(merge_drift_scalar_kernel<S>, dim3(grid_for(a.n, bpc)), dim3(256), 0, st, a,
                       size_t(0));
  }
  return hipGetLastError();
}

#define ADLOCO_DISPATCH_COUNT(n, FN, ...)                                                   \
  switch (n) {                                                                              \
    case 1: e = FN<1>(__VA_ARGS__); break;                                                  \
    case 2: e = FN<2>(__VA_ARGS__); break;                                                  \
    case 3: e = FN<3>(__VA_ARGS__); break;                                                  \
    case 4: e = FN<4>(__VA_ARGS__); break;                                                  \
    case 5: e = FN<5>(__VA_ARGS__); break;                                                  \
    case 6: e = FN<6>(__VA_ARGS__); break;                                                  \
    case 7: e = FN<7>(__VA_ARGS__); break;                                                  \
    case 8: e = FN<8>(__VA_ARGS__); break;                                                  \
    case 9: e = FN<9>(__VA_ARGS__); break;                                                  \
    case 10: e = FN<10>(__VA_ARGS__); break;                                                \
    case 11: e = FN<11>(__VA_ARGS__); break;                                                \
    case 12: e = FN<12>(__VA_ARGS__); break;                                                \
    case 13: e = FN<13>(__VA_ARGS__); break;                                                \
    case 14: e = FN<14>(__VA_ARGS__); break;                                                \
    case 15: e = FN<15>(__VA_ARGS__); break;                                                \
    case 16: e = FN<16>(__VA_ARGS__); break;                                                \
    default: e = hipErrorInvalidValue;                                                      \
  }

}  // namespace adloco

using namespace adloco;

// Two [N] float vectors overlap (either pointer may be NULL: no vector, no overlap).
static bool ranges_overlap(const void* p, const void* q, size_t N) {
  if (!p || !q) return false;
  const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
  const uintptr_t bytes = uintptr_t(N) * sizeof(float);
  return a < b + bytes && b < a + bytes;
}

extern "C" int adloco_outer_step(adloco_ctx* ctx, float* theta_outer, float* const* theta_inst,
                                 int M, size_t N, float* momentum, double lr, double mu,
                                 int nesterov, uint32_t flags, float* pseudo_grad_out,
                                 void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (M < 1) return fail(ctx, ADLOCO_EINVAL, "outer_step: M = %d, need M >= 1", M);
  if (M > ADLOCO_MAX_INSTANCES)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "outer_step: M = %d exceeds %d", M, ADLOCO_MAX_INSTANCES);
  if (flags & ~ADLOCO_BROADCAST) return fail(ctx, ADLOCO_EINVAL, "outer_step: unknown flags");
  if (!(lr == lr) || !(mu == mu)) return fail(ctx, ADLOCO_EINVAL, "outer_step: lr or mu is NaN");
  if (N == 0) return ADLOCO_OK;
  if (!theta_outer || !theta_inst) return fail(ctx, ADLOCO_EINVAL, "outer_step: NULL pointer");
  if (!momentum && mu != 0.0)
    return fail(ctx, ADLOCO_EINVAL, "outer_step: momentum is NULL but mu != 0");
  OuterArgs a{};
  a.theta = theta_outer;
  a.mom = momentum;
  a.pg = pseudo_grad_out;
  bool vec = aligned16(theta_outer) && aligned16(momentum) && aligned16(pseudo_grad_out);
  for (int m = 0; m < M; ++m) {
    float* p = theta_inst[m];
    if (!p) return fail(ctx, ADLOCO_EINVAL, "outer_step: theta_inst[%d] is NULL", m);
    if (ranges_overlap(p, theta_outer, N) || ranges_overlap(p, momentum, N) ||
        ranges_overlap(p, pseudo_grad_out, N))
      return fail(ctx, ADLOCO_EINVAL, "outer_step: theta_inst[%d] overlaps another argument", m);
    // (instances that are only read may be one and the same vector; written ones may not overlap)
    for (int j = 0; j < m; ++j)
      if ((flags & ADLOCO_BROADCAST) ? ranges_overlap(theta_inst[j], p, N)
                                     : (theta_inst[j] != p && ranges_overlap(theta_inst[j], p, N)))
        return fail(ctx, ADLOCO_EINVAL, "outer_step: theta_inst[%d] overlaps theta_inst[%d]", j, m);
    vec = vec && aligned16(p);
    a.inst[m] = p;
  }
  if (ranges_overlap(momentum, theta_outer, N) || ranges_overlap(momentum, pseudo_grad_out, N))
    return fail(ctx, ADLOCO_EINVAL, "outer_step: momentum overlaps another argument");
  if (ranges_overlap(pseudo_grad_out, theta_outer, N))
    return fail(ctx, ADLOCO_EINVAL, "outer_step: pseudo_grad_out overlaps theta_outer");
  if (N / 4 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "outer_step: N = %zu exceeds one launch", N);
  a.n = N;
  a.n_vec = vec ? N / 4 : 0;
  a.lr = lr;
  a.mu = mu;
  a.inv_m = 1.0 / double(M);
  a.nesterov = nesterov ? 1 : 0;
  a.broadcast = (flags & ADLOCO_BROADCAST) ? 1 : 0;
  hipError_t e;
  hipEvent_t ev = prof_begin(ctx, static_cast<hipStream_t>(stream));
  ADLOCO_DISPATCH_COUNT(M, launch_outer_m, a, vec, ctx->stream_blocks_per_cu,
                        static_cast<hipStream_t>(stream));
  prof_end(ctx, kProfOuter, ev, static_cast<hipStream_t>(stream));
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "outer_step launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_merge(adloco_ctx* ctx, float* const* x, const double* weights, int S,
                            size_t N, int rep, int* rep_out, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (S < 1) return fail(ctx, ADLOCO_EINVAL, "merge: S = %d, need S >= 1", S);
  if (S > ADLOCO_MAX_INSTANCES)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "merge: S = %d exceeds %d", S, ADLOCO_MAX_INSTANCES);
  if (!weights) return fail(ctx, ADLOCO_EINVAL, "merge: weights is NULL");
  if (rep < -1 || rep >= S) return fail(ctx, ADLOCO_EINVAL, "merge: rep = %d out of range", rep);
  MergeArgs a{};
  double wsum = 0.0;
  int arg = 0;
  for (int j = 0; j < S; ++j) {
    if (!(weights[j] > 0.0) || weights[j] > 1.0e300)
      return fail(ctx, ADLOCO_EINVAL, "merge: weights[%d] must be positive and finite", j);
    a.w[j] = weights[j];
    wsum += weights[j];
    if (weights[j] > weights[arg]) arg = j;   // first maximum
  }
  if (rep < 0) rep = arg;
  if (rep_out) *rep_out = rep;
  if (N == 0) return ADLOCO_OK;
  if (!x) return fail(ctx, ADLOCO_EINVAL, "merge: x is NULL");
  bool vec = true;
  for (int j = 0; j < S; ++j) {
    if (!x[j]) return fail(ctx, ADLOCO_EINVAL, "merge: x[%d] is NULL", j);
    for (int i = 0; i < j; ++i)
      if (ranges_overlap(x[i], x[j], N))
        return fail(ctx, ADLOCO_EINVAL, "merge: x[%d] overlaps x[%d]", i, j);
    vec = vec && aligned16(x[j]);
    a.x[j] = x[j];
  }
  if (N / 4 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "merge: N = %zu exceeds one launch", N);
  a.inv_wsum = 1.0 / wsum;
  a.n = N;
  a.n_vec = vec ? N / 4 : 0;
  a.rep = rep;
  if (S == 1) return ADLOCO_OK;   // a singleton merge leaves x_r as it is, bit for bit
  hipError_t e;
  hipEvent_t ev = prof_begin(ctx, static_cast<hipStream_t>(stream));
  ADLOCO_DISPATCH_COUNT(S, launch_merge_s, a, vec, ctx->stream_blocks_per_cu,
                        static_cast<hipStream_t>(stream));
  prof_end(ctx, kProfMerge, ev, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(ctx, ADLOCO_EHIP, "merge launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_inner_step(adloco_ctx* ctx, float* theta, float* exp_avg, float* exp_avg_sq,
                                 const float* grad, size_t N, double grad_scale, double lr,
                                 double beta1, double beta2, double eps, double weight_decay,
                                 int64_t step, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (step < 1) return fail(ctx, ADLOCO_EINVAL, "inner_step: step = %lld, need step >= 1", (long long)step);
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0))
    return fail(ctx, ADLOCO_EINVAL, "inner_step: beta1 and beta2 must lie in [0, 1)");
  if (!(lr == lr) || !(eps >= 0.0) || !(weight_decay == weight_decay) || !(grad_scale == grad_scale))
    return fail(ctx, ADLOCO_EINVAL, "inner_step: lr, eps, weight_decay or grad_scale is NaN (or eps < 0)");
  if (N == 0) return ADLOCO_OK;
  if (!theta || !exp_avg || !exp_avg_sq || !grad)
    return fail(ctx, ADLOCO_EINVAL, "inner_step: NULL pointer");
  const void* p[4] = {theta, exp_avg, exp_avg_sq, grad};
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < i; ++j)
      if (ranges_overlap(p[i], p[j], N))
        return fail(ctx, ADLOCO_EINVAL, "inner_step: two arguments overlap");
  if (N / 4 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "inner_step: N = %zu exceeds one launch", N);
  const bool vec = aligned16(theta) && aligned16(exp_avg) && aligned16(exp_avg_sq) && aligned16(grad);
  InnerArgs a{};
  a.theta = theta;
  a.m = exp_avg;
  a.v = exp_avg_sq;
  a.grad = grad;
  a.n = N;
  a.n_vec = vec ? N / 4 : 0;
  a.grad_scale = grad_scale;
  a.decay_keep = 1.0 - lr * weight_decay;
  a.beta1 = beta1;
  a.beta2 = beta2;
  a.omb1 = 1.0 - beta1;
  a.omb2 = 1.0 - beta2;
  a.step_size = lr / (1.0 - std::pow(beta1, double(step)));
  a.inv_sqrt_bc2 = 1.0 / std::sqrt(1.0 - std::pow(beta2, double(step)));
  a.eps = eps;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t ev = prof_begin(ctx, st);
  if (vec) {
    if (a.n_vec > 0)
      hipLaunchKernelGGL(inner_step_vec_kernel,
                         dim3(unsigned((a.n_vec + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(ctx->stream_blocks_per_cu, 5), st, a);   // measured best: 10-12 per CU
    if (a.n_vec * 4 < a.n)
      hipLaunchKernelGGL(inner_step_scalar_kernel, dim3(1), dim3(256), 0, st, a, a.n_vec * 4);
  } else {
    hipLaunchKernelGGL(inner_step_scalar_kernel, dim3(grid_for(a.n, ctx->stream_blocks_per_cu)),
                       dim3(256), 0, st, a, size_t(0));
  }
  hipError_t e = hipGetLastError();
  prof_end(ctx, kProfInner, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "inner_step launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

// ---------------------------------------------------------------------------------------------
// Entry points of the bf16-drift variants
// ---------------------------------------------------------------------------------------------
static bool ranges_overlap_b(const void* p, size_t pb, const void* q, size_t qb) {
  if (!p || !q) return false;
  const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
  return a < b + qb && b < a + pb;
}

extern "C" int adloco_pack_drift(adloco_ctx* ctx, const float* theta_outer, const float* theta_m,
                                 uint16_t* drift_out, size_t N, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (N == 0) return ADLOCO_OK;
  if (!theta_outer || !theta_m || !drift_out) return fail(ctx, ADLOCO_EINVAL, "pack_drift: NULL pointer");
  if (reinterpret_cast<uintptr_t>(drift_out) % 2)
    return fail(ctx, ADLOCO_EINVAL, "pack_drift: drift_out not 2-byte aligned");
  if (ranges_overlap_b(drift_out, 2 * N, theta_outer, 4 * N) || ranges_overlap_b(drift_out, 2 * N, theta_m, 4 * N))
    return fail(ctx, ADLOCO_EINVAL, "pack_drift: drift_out overlaps an input");
  if (N / 8 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "pack_drift: N = %zu exceeds one launch", N);
  const bool vec = aligned16(theta_outer) && aligned16(theta_m) && aligned16(drift_out);
  PackArgs a{theta_outer, theta_m, drift_out, vec ? N / 512 * 64 : 0, N};
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (vec) {
    if (a.n_grp > 0)
      hipLaunchKernelGGL(pack_drift_vec_kernel, dim3(unsigned((a.n_grp + kStreamThreads - 1) / kStreamThreads)),
                         dim3(kStreamThreads), stream_lds_bytes(ctx->stream_blocks_per_cu, 4), st, a);
    if (a.n_grp * 8 < N) hipLaunchKernelGGL(pack_drift_scalar_kernel, dim3(1), dim3(256), 0, st, a, a.n_grp * 8);
  } else {
    hipLaunchKernelGGL(pack_drift_scalar_kernel, dim3(grid_for(N, ctx->stream_blocks_per_cu)), dim3(256), 0,
                       st, a, size_t(0));
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, ADLOCO_EHIP, "pack_drift launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_outer_step_drift(adloco_ctx* ctx, float* theta_outer, uint16_t* const* drift, int M,
                                       size_t N, float* momentum, double lr, double mu, int nesterov,
                                       uint32_t flags, float* pseudo_grad_out, void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (M < 1) return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: M = %d, need M >= 1", M);
  if (M > ADLOCO_MAX_INSTANCES)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "outer_step_drift: M = %d exceeds %d", M, ADLOCO_MAX_INSTANCES);
  if (flags & ~ADLOCO_BROADCAST) return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: unknown flags");
  if (!(lr == lr) || !(mu == mu)) return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: lr or mu is NaN");
  if (N == 0) return ADLOCO_OK;
  if (!theta_outer || !drift) return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: NULL pointer");
  if (!momentum && mu != 0.0)
    return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: momentum is NULL but mu != 0");
  OuterDriftArgs a{};
  a.theta = theta_outer;
  a.mom = momentum;
  a.pg = pseudo_grad_out;
  bool vec = aligned16(theta_outer) && aligned16(momentum) && aligned16(pseudo_grad_out);
  for (int m = 0; m < M; ++m) {
    uint16_t* p = drift[m];
    if (!p || (reinterpret_cast<uintptr_t>(p) % 2))
      return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: drift[%d] is NULL or not 2-byte aligned", m);
    if (ranges_overlap_b(p, 2 * N, theta_outer, 4 * N) || ranges_overlap_b(p, 2 * N, momentum, 4 * N) ||
        ranges_overlap_b(p, 2 * N, pseudo_grad_out, 4 * N))
      return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: drift[%d] overlaps another argument", m);
    for (int j = 0; j < m; ++j)
      if ((flags & ADLOCO_BROADCAST) ? ranges_overlap_b(drift[j], 2 * N, p, 2 * N)
                                     : (drift[j] != p && ranges_overlap_b(drift[j], 2 * N, p, 2 * N)))
        return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: drift[%d] overlaps drift[%d]", j, m);
    vec = vec && aligned16(p);
    a.drift[m] = p;
  }
  if (ranges_overlap(momentum, theta_outer, N) || ranges_overlap(momentum, pseudo_grad_out, N) ||
      ranges_overlap(pseudo_grad_out, theta_outer, N))
    return fail(ctx, ADLOCO_EINVAL, "outer_step_drift: theta_outer, momentum and pseudo_grad_out overlap");
  if (N / 8 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "outer_step_drift: N = %zu exceeds one launch", N);
  a.n = N;
  a.n_grp = vec ? N / 512 * 64 : 0;     // whole waves of 512 parameters; the rest goes to the scalar kernel
  a.lr = lr;
  a.mu = mu;
  a.inv_m = 1.0 / double(M);
  a.nesterov = nesterov ? 1 : 0;
  a.broadcast = (flags & ADLOCO_BROADCAST) ? 1 : 0;
  hipError_t e;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t ev = prof_begin(ctx, st);
  ADLOCO_DISPATCH_COUNT(M, launch_outer_drift_m, a, vec, ctx->stream_blocks_per_cu, st);
  prof_end(ctx, kProfOuter, ev, st);
  if (e != hipSuccess)
    return fail(ctx, ADLOCO_EHIP, "outer_step_drift launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}

extern "C" int adloco_merge_drift(adloco_ctx* ctx, float* x_rep, const uint16_t* const* drift,
                                  double w_rep, const double* w_others, int n_others, size_t N,
                                  void* stream) {
  if (!ctx) return ADLOCO_EINVAL;
  if (n_others < 0) return fail(ctx, ADLOCO_EINVAL, "merge_drift: n_others = %d", n_others);
  if (n_others + 1 > ADLOCO_MAX_INSTANCES)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "merge_drift: %d trainers exceed %d", n_others + 1, ADLOCO_MAX_INSTANCES);
  if (!(w_rep > 0.0) || w_rep > 1.0e300) return fail(ctx, ADLOCO_EINVAL, "merge_drift: w_rep must be positive and finite");
  if (n_others > 0 && (!w_others || !drift)) return fail(ctx, ADLOCO_EINVAL, "merge_drift: NULL weights or drifts");
  MergeDriftArgs a{};
  double wsum = w_rep;
  for (int j = 0; j < n_others; ++j) {
    if (!(w_others[j] > 0.0) || w_others[j] > 1.0e300)
      return fail(ctx, ADLOCO_EINVAL, "merge_drift: w_others[%d] must be positive and finite", j);
    a.w[j] = w_others[j];
    wsum += w_others[j];
  }
  if (N == 0 || n_others == 0) return ADLOCO_OK;      // a singleton merge leaves x_r as it is
  if (!x_rep) return fail(ctx, ADLOCO_EINVAL, "merge_drift: x_rep is NULL");
  bool vec = aligned16(x_rep);
  for (int j = 0; j < n_others; ++j) {
    if (!drift[j] || (reinterpret_cast<uintptr_t>(drift[j]) % 2))
      return fail(ctx, ADLOCO_EINVAL, "merge_drift: drift[%d] is NULL or not 2-byte aligned", j);
    if (ranges_overlap_b(drift[j], 2 * N, x_rep, 4 * N))
      return fail(ctx, ADLOCO_EINVAL, "merge_drift: drift[%d] overlaps x_rep", j);
    vec = vec && aligned16(drift[j]);
    a.drift[j] = drift[j];
  }
  if (N / 8 > kMaxVecPerLaunch)
    return fail(ctx, ADLOCO_EUNSUPPORTED, "merge_drift: N = %zu exceeds one launch", N);
  a.x_rep = x_rep;
  a.inv_wsum = 1.0 / wsum;
  a.n = N;
  a.n_grp = vec ? N / 512 * 64 : 0;
  hipError_t e;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t ev = prof_begin(ctx, st);
  ADLOCO_DISPATCH_COUNT(n_others, launch_merge_drift_s, a, vec, ctx->stream_blocks_per_cu, st);
  prof_end(ctx, kProfMerge, ev, st);
  if (e != hipSuccess) return fail(ctx, ADLOCO_EHIP, "merge_drift launch failed: %s", hipGetErrorString(e));
  return ADLOCO_OK;
}
