// Upcycling initialiser (paper Sec. 4, upcycling settings): every expert starts as a copy of one
// dense FFN matrix and a share of its parameters receives Gaussian noise.  The draws come from the
// counter-based generator Philox-4x64-10 (Salmon et al., SC'11), one call per group of four
// consecutive elements, so the result is a pure function of (seed, stream id, element index).
// Also here: gather / scatter of the trained experts' rows between the full store and the
// contiguous buffer a node uploads at a synchronisation (Sec. 3.3, Eq. 4).
#include "kernels.h"

namespace spes {
namespace {

struct Words4 { unsigned long long w[4]; };

__device__ __forceinline__ Words4 philox4x64_10(unsigned long long c0, unsigned long long c1, unsigned long long k0) {
  constexpr unsigned long long M0 = 0xD2E7470EE14C6C93ull, M1 = 0xCA5A826395121157ull;
  constexpr unsigned long long W0 = 0x9E3779B97F4A7C15ull, W1 = 0xBB67AE8584CAA73Bull;
  unsigned long long c2 = 0, c3 = 0, k1 = 0;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned long long hi0 = __umul64hi(M0, c0), lo0 = M0 * c0;
    const unsigned long long hi1 = __umul64hi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
    k0 += W0; k1 += W1;
  }
  Words4 o;
  o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// noise[j] for the four elements of group g: 0 where the element is not selected
__device__ __forceinline__ void group_noise(unsigned long long g, unsigned long long seed, unsigned long long stream_id,
                                            unsigned thr, float sigma, float* noise) {
  const Words4 o = philox4x64_10(g, stream_id, seed);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const float u1 = ((float)(unsigned)(o.w[2 * q] >> 40) + 0.5f) * (1.f / 16777216.f);
    const float u2 = ((float)(unsigned)(o.w[2 * q + 1] >> 40) + 0.5f) * (1.f / 16777216.f);
    const float r = sqrtf(-2.f * logf(u1));
    float sn, cs;
    sincospif(2.f * u2, &sn, &cs);
    noise[2 * q] = ((unsigned)(o.w[2 * q] & 0xffu) < thr) ? sigma * r * cs : 0.f;
    noise[2 * q + 1] = ((unsigned)(o.w[2 * q + 1] & 0xffu) < thr) ? sigma * r * sn : 0.f;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void upcycle_kernel(const T* __restrict__ dense, T* __restrict__ out, long nvec, long elems,
                                                      unsigned long long seed, unsigned long long stream_id, unsigned thr,
                                                      float sigma) {
  constexpr int N = Vec16<T>::N;          // 4 (fp32) or 8 (bf16) elements per 16-byte vector: one or two groups
  const int e = blockIdx.y;
  const long stride = (long)gridDim.x * 256;
  for (long v = (long)blockIdx.x * 256 + threadIdx.x; v < nvec; v += stride) {
    Vec16<T> q;
    q.load(dense + v * N);
    float f[N];
    q.unpack(f);
    const unsigned long long g0 = ((unsigned long long)e * (unsigned long long)elems + (unsigned long long)v * N) / 4;
#pragma unroll
    for (int h = 0; h < N / 4; ++h) {
      float nz[4];
      group_noise(g0 + h, seed, stream_id, thr, sigma, nz);
#pragma unroll
      for (int j = 0; j < 4; ++j) f[4 * h + j] += nz[j];
    }
    q.pack(f);
    q.store_once(out + (long)e * elems + v * N);
  }
}

constexpr int kPackSlots = 64;
struct PackTable { long row_off[kPackSlots]; };   // element offset of the slot's expert in the full store

// gather (to_store = 0): packed[s] = store[expert of s]; scatter (to_store = 1): the other way
__global__ __launch_bounds__(256) void pack_kernel(const PackTable tb, uint4* __restrict__ store, uint4* __restrict__ packed,
                                                   long slot0, long nvec, long vec_per_row, int to_store) {
  const int s = blockIdx.y;
  uint4* full = store + tb.row_off[s];
  uint4* comp = packed + (slot0 + s) * vec_per_row;
  const long stride = (long)gridDim.x * 256;
  for (long v = (long)blockIdx.x * 256 + threadIdx.x; v < nvec; v += stride) {
    if (to_store) store_stream(full + v, load_stream(comp + v)); else store_stream(comp + v, load_stream(full + v));
  }
}

inline int grid_x(long nvec) {
  long b = (nvec + 255) / 256;            // one vector per thread where the grid allows it
  return (int)(b < 1 ? 1 : b > 8192 ? 8192 : b);
}

}  // namespace

int launch_upcycle_init(int dtype, int n_experts, long elems, const void* dense, unsigned thr, float sigma,
                        unsigned long long seed, unsigned long long stream_id, void* out, hipStream_t s) {
  for (int e0 = 0; e0 < n_experts; e0 += 32768) {          // grid.y limit
    const int ne = n_experts - e0 < 32768 ? n_experts - e0 : 32768;
    if (dtype == SPES_F32) {
      const long nvec = elems / 4;
      hipLaunchKernelGGL(upcycle_kernel<float>, dim3(grid_x(nvec), ne), dim3(256), 0, s, (const float*)dense,
                         (float*)out + (long)e0 * elems, nvec, elems, seed, stream_id, thr, sigma);
    } else {
      const long nvec = elems / 8;
      hipLaunchKernelGGL(upcycle_kernel<bf16_t>, dim3(grid_x(nvec), ne), dim3(256), 0, s, (const bf16_t*)dense,
                         (bf16_t*)out + (long)e0 * elems, nvec, elems, seed, stream_id, thr, sigma);
    }
  }
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

int launch_expert_pack(int dtype, int n_experts, long elems, void* store, const unsigned char* mask, void* packed, int to_store,
                       hipStream_t s) {
  const long vec_per_row = elems * (dtype == SPES_F32 ? 4 : 2) / 16;
  PackTable tb;
  int n = 0;
  long slot0 = 0;
  auto flush = [&]() -> int {
    if (n == 0) return SPES_OK;
    hipLaunchKernelGGL(pack_kernel, dim3(grid_x(vec_per_row), n), dim3(256), 0, s, tb, (uint4*)store, (uint4*)packed, slot0,
                       vec_per_row, vec_per_row, to_store);
    slot0 += n;
    n = 0;
    return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
  };
  for (int e = 0; e < n_experts; ++e) {
    if (!mask[e]) continue;
    tb.row_off[n] = (long)e * vec_per_row;
    if (++n == kPackSlots) {
      const int rc = flush();
      if (rc != SPES_OK) return rc;
    }
  }
  return flush();
}

}  // namespace spes
