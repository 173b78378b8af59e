// Measurement aid: the rate at which a compute unit turns LDS-resident bf16 operands into MFMA
// results when nothing else happens -- no global loads, no barriers, no epilogue.  It is the
// ceiling against which the Gram and gradient-sum kernels are read: both feed their MFMAs from LDS
// with the same fragment reads (ds_read_b128 per 32 x 16 fragment, 32x32x16 MFMA), and the chip
// lowers its clock under that load, so the nominal MFMA peak is out of reach for any of them.
#include "common.h"

namespace adloco {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Wave tile of FM x FN blocks of 32 x 32: per k-step FM + FN fragment reads and FM * FN MFMAs,
// reads and MFMAs interleaved one to one as in the production kernels.
template <int FM, int FN>
__global__ __launch_bounds__(512, 1) void probe_mfma_lds_kernel(float* out, int ksteps) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  // 64 KiB of pseudo-random bf16 values of moderate size (sign, exponent near 0, random mantissa)
  for (int i = threadIdx.x; i < 65536 / 4; i += 512) {
    unsigned h = unsigned(i) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const unsigned lo = 0x3e80u + (h & 0xffu) + ((h & 0x100u) << 7);
    const unsigned hi = 0x3e80u + ((h >> 9) & 0xffu) + ((h & 0x20000u) >> 2);
    reinterpret_cast<unsigned*>(lds)[i] = lo | (hi << 16);
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, kg = lane >> 5;
  f32x16 acc[FM][FN];
#pragma unroll
  for (int m = 0; m < FM; ++m)
#pragma unroll
    for (int n = 0; n < FN; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0.f;
  // 128-byte rows, 16-byte pieces XOR-swizzled by the row: conflict-free fragment reads
  int off_a[FM], off_b[FN];
#pragma unroll
  for (int m = 0; m < FM; ++m) {
    const int row = ((wave >> 2) * 128 + m * 32 + r32) & 255;
    off_a[m] = row * 128 + ((row ^ (row >> 3)) & 7) * 16;
  }
#pragma unroll
  for (int n = 0; n < FN; ++n) {
    const int row = 256 + (((wave & 3) * 64 + n * 32 + r32) & 255);
    off_b[n] = row * 128 + ((row ^ (row >> 3)) & 7) * 16;
  }
  bf16x8 fa[2][FM], fb[2][FN];
  auto rd = [&](int ks, bf16x8 (&A)[FM], bf16x8 (&B)[FN]) {
    const int x = ((ks & 3) * 2 + kg) * 16;
#pragma unroll
    for (int m = 0; m < FM; ++m) A[m] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lds + (off_a[m] ^ x)));
#pragma unroll
    for (int n = 0; n < FN; ++n) B[n] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lds + (off_b[n] ^ x)));
  };
  rd(0, fa[0], fb[0]);
  for (int it = 0; it < ksteps; it += 2) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      rd(it + h + 1, fa[h ^ 1], fb[h ^ 1]);
#pragma unroll
      for (int m = 0; m < FM; ++m)
#pragma unroll
        for (int n = 0; n < FN; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[h][m], fb[h][n], acc[m][n], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < FM * FN; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < FM + FN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
  }
  float r = 0.f;
#pragma unroll
  for (int m = 0; m < FM; ++m)
#pragma unroll
    for (int n = 0; n < FN; ++n) r += acc[m][n][0] + acc[m][n][9];
  out[blockIdx.x * 512 + threadIdx.x] = r;
}

}  // namespace
}  // namespace adloco

using namespace adloco;

// variant 0: 64 x 64 wave tiles (two accumulator sets of that size are what the tile-pair Gram
// kernel holds), 1: 128 x 64 wave tiles (gradient-sum and tile-statistics kernels).  One workgroup
// of eight waves per CU, `ksteps` k-steps of 16 each (rounded up to even).  Returns the kernel time
// of the second of two launches and the flops it executed.
extern "C" int adloco_probe_mfma_lds(adloco_ctx* ctx, int variant, int ksteps, double* ms,
                                     double* flops) {
  if (!ctx || !ms || !flops || ksteps < 2 || ksteps > (1 << 20) || (variant != 0 && variant != 1))
    return ctx ? fail(ctx, ADLOCO_EINVAL, "probe_mfma_lds: bad argument") : ADLOCO_EINVAL;
  ksteps += ksteps & 1;
  const size_t out_bytes = size_t(kNumCu) * 512 * sizeof(float);
  int rc = ensure_scratch(ctx, ctx->red_f64, out_bytes);
  if (rc) return rc;
  float* out = static_cast<float*>(ctx->red_f64.ptr);
  auto kern = variant ? probe_mfma_lds_kernel<4, 2> : probe_mfma_lds_kernel<2, 2>;
  ADLOCO_HIP_CHECK(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ADLOCO_HIP_CHECK(ctx, hipEventCreate(&e0));
  ADLOCO_HIP_CHECK(ctx, hipEventCreate(&e1));
  hipLaunchKernelGGL(kern, dim3(kNumCu), dim3(512), 128 * 1024, nullptr, out, ksteps);
  (void)hipEventRecord(e0, nullptr);
  hipLaunchKernelGGL(kern, dim3(kNumCu), dim3(512), 128 * 1024, nullptr, out, ksteps);
  (void)hipEventRecord(e1, nullptr);
  hipError_t e = hipEventSynchronize(e1);
  float t = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return fail(ctx, ADLOCO_EHIP, "probe_mfma_lds: %s", hipGetErrorString(e));
  *ms = double(t);
  *flops = double(kNumCu) * 8.0 * (variant ? 8.0 : 4.0) * double(ksteps) * 32768.0;
  return ADLOCO_OK;
}
