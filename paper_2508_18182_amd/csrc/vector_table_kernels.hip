// Per-sample gradient norms of the parameter blocks that are not linear weights: vectors that
// enter a layer element-wise (biases, normalisation gains) and embedding tables.  Together with
// the linear weights they make g_i the full per-sample gradient grad f(x_k; xi_i) that eq. 1
// averages and whose variance Section 3.3.1 tests.
//   vector p [d]:  g_i = sum_t delta_{i,t} * x_{i,t}   (x = 1 for a bias)      -> ||g_i||^2
//   table  E [V,d]: row v of g_i = sum_{t: id_t = v} delta_{i,t}               -> ||g_i||^2
// All of it streams delta (and x) once: HBM-bound.  Sums run in a fixed order (repeatable).
#include <type_traits>

#include "common.h"

namespace adloco {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kSlab = 256;       // columns per workgroup
constexpr int kVtThreads = 256;

__device__ __forceinline__ float elem_to_f32(unsigned short h) { return __uint_as_float(unsigned(h) << 16); }
__device__ __forceinline__ float elem_to_f32(_Float16 h) { return float(h); }
__device__ __forceinline__ float elem_to_f32(float f) { return f; }

__device__ __forceinline__ double vt_wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Sum over a 256-thread workgroup, valid in thread 0 (fixed order).
__device__ __forceinline__ double vt_block_sum(double v, double* lds4) {
  v = vt_wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

// last descriptor whose blk_start <= b
__device__ __forceinline__ int find_aux(const AuxDesc* tab, int n, int b) {
  int lo = 0, hi = n - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (tab[mid].blk_start <= b) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Eight consecutive elements of a row starting at column c (columns >= d read as zero).
template <typename E>
__device__ __forceinline__ void load8(const E* row, int c, int d, bool fast, float (&v)[8]) {
  if (fast && c + 8 <= d) {
    if constexpr (std::is_same<E, _Float16>::value) {
      typedef __attribute__((ext_vector_type(8))) _Float16 h8;
      const h8 r = __builtin_nontemporal_load(reinterpret_cast<const h8*>(row + c));
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = float(r[j]);
    } else if constexpr (sizeof(E) == 2) {
      const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + c));   // read once
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[2 * j] = __uint_as_float(r[j] << 16);
        v[2 * j + 1] = __uint_as_float(r[j] & 0xffff0000u);
      }
    } else {
      const float4 r0 = *reinterpret_cast<const float4*>(row + c);
      const float4 r1 = *reinterpret_cast<const float4*>(row + c + 4);
      v[0] = r0.x; v[1] = r0.y; v[2] = r0.z; v[3] = r0.w;
      v[4] = r1.x; v[5] = r1.y; v[6] = r1.z; v[7] = r1.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (c + j < d) ? elem_to_f32(row[c + j]) : 0.f;
  }
}

// ---------------------------------------------------------------------------------------
// Vectors, step 1: v_i[c] = sum_t delta[i,t,c] * x[i,t,c] for one (layer, sample, 256-column
// slab) per workgroup.  Thread = (row group tid/32, 8 columns (tid%32)*8): a half wave reads
// 512 contiguous bytes of a bf16 row; the eight row groups are summed through LDS in order.
// ---------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(kVtThreads) void vector_rowsum_kernel(const LayerDev* layers,
                                                                   const AuxDesc* tab, int n_tab,
                                                                   int B, int T, float* vec) {
  __shared__ float red[8][kSlab];
  const AuxDesc A = tab[find_aux(tab, n_tab, blockIdx.x)];
  const LayerDev L = layers[A.layer];
  const int rel = blockIdx.x - A.blk_start;
  const int sample = rel / A.slabs, slab = rel % A.slabs;
  const int d = L.d_out;
  const int cs = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int c = slab * kSlab + cs * 8;
  const E* D = reinterpret_cast<const E*>(L.delta) + (long long)sample * T * L.delta_stride;
  const E* X = L.a ? reinterpret_cast<const E*>(L.a) + (long long)sample * T * L.a_stride : nullptr;
  const bool also_bias = A.vec_off_bias >= 0;     // the bias that reads the same delta: sum_t delta as well
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float acc1[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c < d) {
#pragma unroll 4
    for (int t = rg; t < T; t += 8) {
      float dv[8];
      load8<E>(D + (long long)t * L.delta_stride, c, d, L.fast, dv);
      if (X) {
        float xv[8];
        load8<E>(X + (long long)t * L.a_stride, c, d, L.fast, xv);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = fmaf(dv[j], xv[j], acc[j]);
        if (also_bias) {
#pragma unroll
          for (int j = 0; j < 8; ++j) acc1[j] += dv[j];
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += dv[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[rg][cs * 8 + j] = acc[j];
  __syncthreads();
  const int col = slab * kSlab + threadIdx.x;
  if (col < d) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) s += red[r][threadIdx.x];
    vec[A.vec_off + (long long)sample * d + col] = s;
  }
  if (also_bias) {           // same order of summation as a bias block of its own
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) red[rg][cs * 8 + j] = acc1[j];
    __syncthreads();
    if (col < d) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) s += red[r][threadIdx.x];
      vec[A.vec_off_bias + (long long)sample * d + col] = s;
    }
  }
}

// Vectors, step 2a: grad_sum[c] (+)= sum_i v_i[c], samples in order.  One thread per column.
__global__ __launch_bounds__(kVtThreads) void vector_colsum_kernel(const LayerDev* layers,
                                                                   const AuxDesc* tab, int n_tab,
                                                                   int B, const float* vec,
                                                                   int accumulate) {
  // this launch uses blk_start2 (one workgroup per slab and layer)
  int lo = 0, hi = n_tab - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (tab[mid].blk_start2 <= int(blockIdx.x)) lo = mid; else hi = mid - 1;
  }
  const AuxDesc A = tab[lo];
  const LayerDev L = layers[A.layer];
  if (L.provided) return;
  const int col = (blockIdx.x - A.blk_start2) * kSlab + threadIdx.x;
  if (col >= L.d_out) return;
  float s = 0.f;
  for (int i = 0; i < B; ++i) s += vec[A.vec_off + (long long)i * L.d_out + col];
  L.grad_sum[col] = accumulate ? L.grad_sum[col] + s : s;
}

// Vectors, step 2b: ||v_i||^2 -> slot 0 of the layer's partial sums of sample i (others zero).
__global__ __launch_bounds__(kVtThreads) void vector_sqnorm_kernel(const LayerDev* layers,
                                                                   const AuxDesc* tab, int B,
                                                                   const float* vec,
                                                                   float* partials, int n_pairs) {
  __shared__ double lds4[4];
  const AuxDesc A = tab[blockIdx.x / B];
  const int sample = blockIdx.x % B;
  const int d = layers[A.layer].d_out;
  const float* v = vec + A.vec_off + (long long)sample * d;
  double acc = 0.0;
  for (int c = threadIdx.x; c < d; c += kVtThreads) acc += double(v[c]) * double(v[c]);
  const double s = vt_block_sum(acc, lds4);
  float* p = partials + (size_t(A.layer) * B + sample) * n_pairs;
  if (threadIdx.x == 0) p[0] = float(s);
  for (int k = 1 + threadIdx.x; k < n_pairs; k += kVtThreads) p[k] = 0.f;
}

// ---------------------------------------------------------------------------------------
// Tables, step 1: sort the tokens of one (table, sample) by id (bitonic sort of the keys
// id * 2^32 + t in LDS) and write the token order; bit 31 marks the first token of an id.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kVtThreads) void embed_sort_kernel(const LayerDev* layers,
                                                                const AuxDesc* tab, int B, int T,
                                                                int P, int* perm) {
  extern __shared__ unsigned long long keys[];
  const AuxDesc A = tab[blockIdx.x / B];
  const int sample = blockIdx.x % B;
  const int* ids = reinterpret_cast<const int*>(layers[A.layer].a) + (long long)sample * T;
  for (int t = threadIdx.x; t < P; t += kVtThreads)
    keys[t] = t < T ? ((unsigned long long)(unsigned)ids[t] << 32) | unsigned(t) : ~0ull;
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < P; i += kVtThreads) {
        const int l = i ^ j;
        if (l > i) {
          const unsigned long long x = keys[i], y = keys[l];
          const bool up = (i & k) == 0;
          if ((x > y) == up) { keys[i] = y; keys[l] = x; }
        }
      }
      __syncthreads();
    }
  int* out = perm + A.perm_off + (long long)sample * T;
  for (int s = threadIdx.x; s < T; s += kVtThreads) {
    const unsigned long long key = keys[s];
    const bool first = s == 0 || (keys[s - 1] >> 32) != (key >> 32);
    out[s] = int(unsigned(key) | (first ? 0x80000000u : 0u));
  }
}

// Tables, step 2: one workgroup per (table, sample, 64-column slab).  Its four waves split the
// sample's tokens, taken in id order, into four consecutive pieces; in each piece a thread
// (one column) sums the delta rows of equal ids and adds up the squares of the sums that are
// complete inside the piece.  A run of equal ids that crosses a piece boundary is stitched
// together afterwards from the pieces' head and tail sums, in piece order.
constexpr int kEmbSlab = 64;

template <typename E>
__global__ __launch_bounds__(kVtThreads) void embed_rows_kernel(const LayerDev* layers,
                                                                const AuxDesc* tab, int n_tab,
                                                                int B, int T, const int* perm,
                                                                double* part) {
  __shared__ float head[4][kEmbSlab], tail[4][kEmbSlab];
  __shared__ double inner[4][kEmbSlab];
  __shared__ int has_start[4];
  __shared__ double lds4[4];
  const AuxDesc A = tab[find_aux(tab, n_tab, blockIdx.x)];
  const LayerDev L = layers[A.layer];
  const int rel = blockIdx.x - A.blk_start;
  const int sample = rel / A.slabs, slab = rel % A.slabs;
  const int lane = threadIdx.x & 63, piece = threadIdx.x >> 6;
  const int col = slab * kEmbSlab + lane;
  const bool live = col < L.d_out;
  const E* D = reinterpret_cast<const E*>(L.delta) + (long long)sample * T * L.delta_stride;
  const int* order = perm + A.perm_off + (long long)sample * T;
  const int len = (T + 3) / 4;
  const int s_begin = piece * len, s_end = (piece + 1) * len < T ? (piece + 1) * len : T;
  float run = 0.f, first_run = 0.f;
  double tot = 0.0;
  bool started = false;           // a run began inside this piece
  // eight tokens' rows are requested together, then consumed in order
  for (int s0 = s_begin; s0 < s_end; s0 += 8) {
    int e[8];
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = s0 + j < s_end ? order[s0 + j] : 0;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      v[j] = (live && s0 + j < s_end)
                 ? elem_to_f32(D[(long long)(e[j] & 0x7fffffff) * L.delta_stride + col]) : 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < s_end) {
        if (e[j] < 0) {           // first token of an id: the run before it is finished
          if (started) tot += double(run) * double(run); else first_run = run;
          started = true;
          run = 0.f;
        }
        run += v[j];
      }
  }
  // no run began here: the whole piece continues an earlier run (head = run, nothing else)
  head[piece][lane] = started ? first_run : run;
  tail[piece][lane] = started ? run : 0.f;
  inner[piece][lane] = tot;
  if (lane == 0) has_start[piece] = started ? 1 : 0;
  __syncthreads();
  double total = 0.0;
  if (piece == 0) {
    float carry = 0.f;            // open run handed from piece to piece
    for (int k = 0; k < 4; ++k) {
      carry += head[k][lane];
      if (has_start[k]) {
        total += double(carry) * double(carry) + inner[k][lane];
        carry = tail[k][lane];
      }
    }
    total += double(carry) * double(carry);
    if (!live) total = 0.0;
  }
  const double s = vt_block_sum(total, lds4);
  if (threadIdx.x == 0) part[A.part_off + (long long)sample * A.slabs + slab] = s;
}

// Tables, step 3: slab totals -> slot 0 of the layer's partial sums of sample i (others zero).
__global__ __launch_bounds__(64) void embed_finalize_kernel(const AuxDesc* tab, int B,
                                                            const double* part, float* partials,
                                                            int n_pairs) {
  const AuxDesc A = tab[blockIdx.x / B];
  const int sample = blockIdx.x % B;
  float* p = partials + (size_t(A.layer) * B + sample) * n_pairs;
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int k = 0; k < A.slabs; ++k) s += part[A.part_off + (long long)sample * A.slabs + k];
    p[0] = float(s);
  }
  for (int k = 1 + threadIdx.x; k < n_pairs; k += 64) p[k] = 0.f;
}

int vector_table_slab() { return kSlab; }
int embed_table_slab() { return kEmbSlab; }

hipError_t launch_vector_stats(const LayerDev* layers, const AuxDesc* tab, int n_tab,
                               int blocks_rowsum, int blocks_colsum, int B, int T, int dtype,
                               float* vec, float* partials, int n_pairs, int accumulate,
                               bool write_grad_sum, hipStream_t st) {
  if (n_tab <= 0) return hipSuccess;
  if (dtype == ADLOCO_BF16)
    hipLaunchKernelGGL(vector_rowsum_kernel<unsigned short>, dim3(blocks_rowsum), dim3(kVtThreads), 0,
                       st, layers, tab, n_tab, B, T, vec);
  else if (dtype == ADLOCO_F16)
    hipLaunchKernelGGL(vector_rowsum_kernel<_Float16>, dim3(blocks_rowsum), dim3(kVtThreads), 0,
                       st, layers, tab, n_tab, B, T, vec);
  else
    hipLaunchKernelGGL(vector_rowsum_kernel<float>, dim3(blocks_rowsum), dim3(kVtThreads), 0, st,
                       layers, tab, n_tab, B, T, vec);
  if (write_grad_sum)
    hipLaunchKernelGGL(vector_colsum_kernel, dim3(blocks_colsum), dim3(kVtThreads), 0, st, layers, tab,
                       n_tab, B, vec, accumulate);
  hipLaunchKernelGGL(vector_sqnorm_kernel, dim3(n_tab * B), dim3(kVtThreads), 0, st, layers, tab, B,
                     vec, partials, n_pairs);
  return hipGetLastError();
}

hipError_t launch_embed_stats(const LayerDev* layers, const AuxDesc* tab, int n_tab, int blocks_rows,
                              int B, int T, int dtype, int* perm, double* part, float* partials,
                              int n_pairs, hipStream_t st) {
  if (n_tab <= 0) return hipSuccess;
  int P = 1;
  while (P < T) P <<= 1;
  const size_t lds = size_t(P) * sizeof(unsigned long long);
  if (lds > 64 * 1024) return hipErrorInvalidValue;   // the caller limits T
  hipLaunchKernelGGL(embed_sort_kernel, dim3(n_tab * B), dim3(kVtThreads), lds, st, layers, tab, B, T,
                     P, perm);
  if (dtype == ADLOCO_BF16)
    hipLaunchKernelGGL(embed_rows_kernel<unsigned short>, dim3(blocks_rows), dim3(kVtThreads), 0, st,
                       layers, tab, n_tab, B, T, perm, part);
  else if (dtype == ADLOCO_F16)
    hipLaunchKernelGGL(embed_rows_kernel<_Float16>, dim3(blocks_rows), dim3(kVtThreads), 0, st,
                       layers, tab, n_tab, B, T, perm, part);
  else
    hipLaunchKernelGGL(embed_rows_kernel<float>, dim3(blocks_rows), dim3(kVtThreads), 0, st, layers,
                       tab, n_tab, B, T, perm, part);
  hipLaunchKernelGGL(embed_finalize_kernel, dim3(n_tab * B), dim3(64), 0, st, tab, B, part, partials,
                     n_pairs);
  return hipGetLastError();
}

}  // namespace adloco
