// Reference rate of the matrix cores on this device: a loop of 16x16x32 bf16 MFMAs (the form the grouped GEMMs use) whose operands stay in
// registers, on operand values the caller supplies.  The shader clock under matrix load depends on the data (power),
// so the figure that the grouped GEMMs can be priced against is this one measured on data like theirs, not the
// nominal peak.  Benchmark aid only; nothing on the training path calls it.
#include "kernels.h"

namespace spes {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 ref_bf16x8;
typedef __attribute__((ext_vector_type(4))) float ref_f32x4;

constexpr int kRefTiles = 8;                 // a wavefront holds an 8 x 8 grid of 16 x 16 accumulator tiles
constexpr int kRefMfmaPerIter = kRefTiles * kRefTiles;

__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(const uint4* __restrict__ data, int iters, float* __restrict__ sink) {
  const int tid = threadIdx.x;
  ref_bf16x8 fa[kRefTiles], fb[kRefTiles];
#pragma unroll
  for (int i = 0; i < kRefTiles; ++i) {
    fa[i] = __builtin_bit_cast(ref_bf16x8, data[(i * 256 + tid) & 4095]);
    fb[i] = __builtin_bit_cast(ref_bf16x8, data[((i + kRefTiles) * 256 + tid + blockIdx.x) & 4095]);
  }
  ref_f32x4 acc[kRefTiles][kRefTiles];
#pragma unroll
  for (int j = 0; j < kRefTiles; ++j)
#pragma unroll
    for (int i = 0; i < kRefTiles; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[j][i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kRefTiles; ++j)
#pragma unroll
      for (int i = 0; i < kRefTiles; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[j][i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kRefTiles; ++j)
#pragma unroll
    for (int i = 0; i < kRefTiles; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += acc[j][i][r];
  if (tid == 0) sink[blockIdx.x] = s;      // keeps the loop alive; one float per block
}

}  // namespace

int launch_mfma_rate(const void* data, int blocks, int iters, float* sink, double* flop, hipStream_t s) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)data, iters, sink);
  if (flop) *flop = (double)blocks * 4.0 * iters * kRefMfmaPerIter * (2.0 * 16 * 16 * 32);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

}  // namespace spes
