// Shared device helpers for the SPES MoE kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/spes.h"
#include "../../include/spes_bench.h"

namespace spes {

constexpr int kWave = 64;
constexpr int kMaxExperts = 64;   // one router score per lane of a wavefront
constexpr int kAuxExtra = 2;      // floats after the per-expert factors of the auxiliary-loss gradient record
constexpr int kAuxBlocks = 256;   // upper bound on the partial sums of the auxiliary router losses

typedef uint16_t bf16_t;          // raw bf16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even through the hardware conversion (v_cvt_pk_bf16_f32 on gfx950)
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// 16-byte accesses with the non-temporal hint, for data that is touched once: a pure read stream reaches 7.0 TB/s
// with it against 6.3 TB/s without, a copy 6.0 against 5.2
typedef __attribute__((ext_vector_type(4))) float nt_f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int nt_u32x4_t;
__device__ __forceinline__ float4 load_stream(const float4* p) {
  const nt_f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const nt_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float4* p, const float4& q) {
  const nt_f32x4_t v = {q.x, q.y, q.z, q.w};
  __builtin_nontemporal_store(v, reinterpret_cast<nt_f32x4_t*>(p));
}
__device__ __forceinline__ void store_stream(uint2* p, const uint2& q) {
  typedef __attribute__((ext_vector_type(2))) unsigned int nt_u32x2_t;
  const nt_u32x2_t v = {q.x, q.y};
  __builtin_nontemporal_store(v, reinterpret_cast<nt_u32x2_t*>(p));
}
__device__ __forceinline__ void store_stream(uint4* p, const uint4& q) {
  const nt_u32x4_t v = {q.x, q.y, q.z, q.w};
  __builtin_nontemporal_store(v, reinterpret_cast<nt_u32x4_t*>(p));
}

// 16-byte vector of storage elements, unpacked to floats and back; load_once / store_once carry the non-temporal hint
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  __device__ __forceinline__ void load_once(const float* p) { raw = load_stream(reinterpret_cast<const float4*>(p)); }
  __device__ __forceinline__ void store_once(float* p) const { store_stream(reinterpret_cast<float4*>(p), raw); }
  __device__ __forceinline__ void unpack(float* f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
  __device__ __forceinline__ void pack(const float* f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void load_once(const bf16_t* p) { raw = load_stream(reinterpret_cast<const uint4*>(p)); }
  __device__ __forceinline__ void store_once(bf16_t* p) const { store_stream(reinterpret_cast<uint4*>(p), raw); }
  __device__ __forceinline__ void unpack(float* f) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void pack(const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
    raw = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// All-lanes reductions of a full wavefront (every lane active) without LDS traffic: four data-parallel-primitive
// steps inside each row of 16 lanes (neighbour, other pair, mirrored half row, mirrored row), then the four row
// results through scalar registers.  The order of the operations is fixed, so results are reproducible.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(v);     // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);     // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);    // row_half_mirror
  v += dpp_move<0x140>(v);    // row_mirror
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}


// block-wide sum for blockDim.x == 256; result valid in every thread
__device__ __forceinline__ float block_sum_256(float v, float* smem4) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem4[w] = v;
  __syncthreads();
  return smem4[0] + smem4[1] + smem4[2] + smem4[3];
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ __device__ inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

}  // namespace spes
