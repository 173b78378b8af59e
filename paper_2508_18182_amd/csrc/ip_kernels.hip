// Per-sample inner products c_i = <g_i, G> with the batch gradient sum G, the quantity whose
// variance the inner-product test and the augmented inner-product test of Section 3.3.2 need.
// For aligned bf16 linear layers the tiles of each per-sample gradient g_i = delta_i^T a_i are
// formed in registers by the tile GEMM kernel (csrc/wgrad_kernels.hip, inner-product form) and
// reduced against the fp32 tile of G on the spot; this file holds the plain path for everything
// else, the vector / table blocks and the reductions.  As a by-product every path also returns
// the explicit ||g_i||^2, a second route to the Gram kernel's result.
#include "common.h"

namespace adloco {

constexpr int kIpThreads = 256;

__device__ __forceinline__ float ip_elem(unsigned short h) { return __uint_as_float(unsigned(h) << 16); }
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
// likewise the explicit ||g_i||^2.  tile_out may be null (no tile launch).
__global__ __launch_bounds__(kIpThreads) void ip_finalize_samples_kernel(
    const int4* tiles, const float* tile_out, long long n_tiles, const float* dot, const float* sq,
    const unsigned char* in_tiles, int n_layers, int B, float* per_sample_ip, float* per_sample_sq,
    double* sample_f64) {
  __shared__ double lds4[4];
  const int i = blockIdx.x;
  double c = 0.0, q = 0.0;
  for (long long k = threadIdx.x; k < n_tiles; k += kIpThreads) {
    const int4 t = tiles[k];
    if (t.x >= 0 && t.w == i) {
      c += double(tile_out[2 * k]);
      q += double(tile_out[2 * k + 1]);
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
    else
      hipLaunchKernelGGL(embed_ip_kernel<float>, dim3(unsigned(n_emb) * B), dim3(kIpThreads), 0, st,
                         layers, emb_tab, B, T, dot);
  }
  return hipGetLastError();
}

hipError_t launch_ip_finalize(const void* tiles, const float* tile_out, long long n_tiles,
                              const float* dot, const float* sq, const unsigned char* in_tiles,
                              int n_layers, int B, float* per_sample_ip, float* per_sample_sq,
                              double* sample_f64, adloco_ip_acc* acc, int accumulate, hipStream_t st) {
  hipLaunchKernelGGL(ip_finalize_samples_kernel, dim3(B), dim3(kIpThreads), 0, st,
                     static_cast<const int4*>(tiles), tile_out, n_tiles, dot, sq, in_tiles, n_layers, B,
                     per_sample_ip, per_sample_sq, sample_f64);
  hipLaunchKernelGGL(ip_finalize_batch_kernel, dim3(1), dim3(1024), 0, st, sample_f64, B, acc,
                     accumulate);
  return hipGetLastError();
}

}  // namespace adloco
