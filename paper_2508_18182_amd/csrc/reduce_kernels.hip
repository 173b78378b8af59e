// Reductions: S2 = sum_l ||grad_sum_l||_F^2 (the batch-gradient norm of eq. 1 times B^2) and
// the per-sample / batch totals of the Gram partial sums (S1 of the variance, Section 3.3.1).
// Wave-shuffle + LDS tree, fp64 accumulation, fixed summation order (bitwise repeatable).
#include "common.h"

namespace adloco {

constexpr int kRedThreads = 256;
constexpr int kSqChunk = 16384;   // floats per workgroup of the squared-norm kernel

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over the workgroup; result valid in thread 0.  blockDim.x must be a multiple of 64.
__device__ __forceinline__ double block_sum_f64(double v, double* lds) {
  v = wave_sum_f64(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();   // lds may still be in use by an earlier call
  if (lane == 0) lds[wave] = v;
  __syncthreads();
  double s = 0.0;
  if (threadIdx.x == 0)
    for (int w = 0; w < nw; ++w) s += lds[w];
  return s;
}

typedef float __attribute__((ext_vector_type(4))) f32x4;

// One workgroup per kSqChunk floats of one layer's grad_sum.
__global__ __launch_bounds__(kRedThreads) void sqnorm_partial_kernel(const LayerDev* layers,
                                                                     int n_layers,
                                                                     double* partial) {
  __shared__ double lds[kRedThreads / 64];
  // binary search: last layer whose sq_blk_start <= blockIdx.x
  int lo = 0, hi = n_layers - 1;
  const int b = blockIdx.x;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (layers[mid].sq_blk_start <= b) lo = mid; else hi = mid - 1;
  }
  const LayerDev L = layers[lo];
  const long long numel = (long long)L.d_in * L.d_out;
  const long long begin = (long long)(b - L.sq_blk_start) * kSqChunk;
  long long end = begin + kSqChunk;
  if (end > numel) end = numel;
  const float* g = L.grad_sum;
  double acc = 0.0;
  if ((reinterpret_cast<uintptr_t>(g) & 15u) == 0) {
    const long long vend = begin + ((end - begin) & ~3LL);
    for (long long e = begin + threadIdx.x * 4; e < vend; e += kRedThreads * 4) {
      f32x4 v = *reinterpret_cast<const f32x4*>(g + e);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc += double(v[c]) * double(v[c]);
    }
    for (long long e = vend + threadIdx.x; e < end; e += kRedThreads)
      acc += double(g[e]) * double(g[e]);
  } else {
    for (long long e = begin + threadIdx.x; e < end; e += kRedThreads)
      acc += double(g[e]) * double(g[e]);
  }
  double s = block_sum_f64(acc, lds);
  if (threadIdx.x == 0) partial[b] = s;
}

// One workgroup: out[0] = sum of partial[0..n) in a fixed order.
__global__ __launch_bounds__(1024) void sum_f64_kernel(const double* partial, long long n,
                                                       double* out) {
  __shared__ double lds[16];
  double acc = 0.0;
  for (long long i = threadIdx.x; i < n; i += blockDim.x) acc += partial[i];
  double s = block_sum_f64(acc, lds);
  if (threadIdx.x == 0) out[0] = s;
}

// One workgroup per sample i: n_i^l = sum over tile pairs of the Gram partials, n_i = sum_l n_i^l.
__global__ __launch_bounds__(kRedThreads) void finalize_samples_kernel(
    const float* partials, int n_layers, int B, int n_pairs, float* per_sample,
    float* per_layer_sample, double* sample_f64) {
  __shared__ double lds[kRedThreads / 64];
  const int i = blockIdx.x;
  double tot = 0.0;
  for (int l = threadIdx.x; l < n_layers; l += kRedThreads) {
    const float* p = partials + (size_t(l) * B + i) * n_pairs;
    double s = 0.0;
    for (int k = 0; k < n_pairs; ++k) s += double(p[k]);
    if (per_layer_sample) per_layer_sample[size_t(l) * B + i] = float(s);
    tot += s;
  }
  double s = block_sum_f64(tot, lds);
  if (threadIdx.x == 0) {
    per_sample[i] = float(s);
    sample_f64[i] = s;
  }
}

// One workgroup: S1 (+)= sum_i n_i, n_samples (+)= B.
__global__ __launch_bounds__(1024) void finalize_batch_kernel(const double* sample_f64, int B,
                                                              adloco_stats_acc* acc,
                                                              int accumulate) {
  __shared__ double lds[16];
  double a = 0.0;
  for (int i = threadIdx.x; i < B; i += blockDim.x) a += sample_f64[i];
  double s = block_sum_f64(a, lds);
  if (threadIdx.x == 0) {
    if (accumulate) {
      acc->sum_sample_sqnorm += s;
      acc->n_samples += B;
    } else {
      acc->sum_sample_sqnorm = s;
      acc->n_samples = B;
    }
  }
}

size_t sqnorm_partials(const std::vector<LayerDev>& host_layers) {
  if (host_layers.empty()) return 0;
  const LayerDev& L = host_layers.back();
  const long long numel = (long long)L.d_in * L.d_out;
  return size_t(L.sq_blk_start) + size_t((numel + kSqChunk - 1) / kSqChunk);
}

int sqnorm_chunk() { return kSqChunk; }

hipError_t launch_sqnorm_table(const LayerDev* layers, int n_layers, size_t nblk, double* partial,
                               double* out, hipStream_t st) {
  hipLaunchKernelGGL(sqnorm_partial_kernel, dim3(unsigned(nblk)), dim3(kRedThreads), 0, st, layers,
                     n_layers, partial);
  hipLaunchKernelGGL(sum_f64_kernel, dim3(1), dim3(1024), 0, st, partial, (long long)nblk, out);
  return hipGetLastError();
}

hipError_t launch_sqnorm(const LayerDev* layers, const std::vector<LayerDev>& host_layers,
                         double* partial, double* out, hipStream_t st) {
  return launch_sqnorm_table(layers, int(host_layers.size()), sqnorm_partials(host_layers), partial,
                             out, st);
}

hipError_t launch_finalize_stats(const float* partials, int n_layers, int B, int n_pairs,
                                 float* per_sample, float* per_layer_sample, double* sample_f64,
                                 adloco_stats_acc* acc, int accumulate, hipStream_t st) {
  hipLaunchKernelGGL(finalize_samples_kernel, dim3(B), dim3(kRedThreads), 0, st, partials, n_layers,
                     B, n_pairs, per_sample, per_layer_sample, sample_f64);
  hipLaunchKernelGGL(finalize_batch_kernel, dim3(1), dim3(1024), 0, st, sample_f64, B, acc,
                     accumulate);
  return hipGetLastError();
}

}  // namespace adloco
