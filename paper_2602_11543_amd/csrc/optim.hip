// AdamW on the trainable subset (paper Sec. 3.3 "Efficiency Analysis": gradients and the two
// moments exist only for the assigned experts and the shared parameters; hyper-parameters
// App. B, Table A1).  One streaming pass: per element 16 bytes of fp32 state and gradient in,
// 12 bytes of state out, plus the storage-type copy of the weight in the full expert store.
#include <cmath>

#include "kernels.h"

namespace spes {
namespace {

constexpr int kSlotsPerLaunch = 64;

struct SlotTable {
  long param_off[kSlotsPerLaunch];   // element offset of the slot's expert in the full store
  long slot_off[kSlotsPerLaunch];    // element offset of the slot in the compact arrays
};

struct AdamHyper {
  float lr, beta1, beta2, eps, wd, inv_bc1, inv_bc2, grad_scale;
};

// T = storage type of the full store; with T = float and master == nullptr the store itself is the fp32 weight.
template <typename T>
__global__ __launch_bounds__(256) void masked_adamw_kernel(const SlotTable tb, T* __restrict__ param, float* __restrict__ master,
                                                           float* __restrict__ m, float* __restrict__ v,
                                                           const float* __restrict__ grad, long nvec, const AdamHyper h) {
  const int s = blockIdx.y;
  T* p = param + tb.param_off[s];
  const long so = tb.slot_off[s];
  float* w = master ? master + so : reinterpret_cast<float*>(p);
  const long stride = (long)gridDim.x * 256;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
    const float4 g4 = load_stream(reinterpret_cast<const float4*>(grad + so + i * 4));
    const float4 m4 = load_stream(reinterpret_cast<const float4*>(m + so + i * 4));
    const float4 v4 = load_stream(reinterpret_cast<const float4*>(v + so + i * 4));
    const float4 w4 = load_stream(reinterpret_cast<const float4*>(w + i * 4));
    const float g[4] = {g4.x, g4.y, g4.z, g4.w};
    float mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w}, ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ge = g[e] * h.grad_scale;
      mm[e] = h.beta1 * mm[e] + (1.f - h.beta1) * ge;
      vv[e] = h.beta2 * vv[e] + (1.f - h.beta2) * ge * ge;
      const float upd = (mm[e] * h.inv_bc1) / (sqrtf(vv[e] * h.inv_bc2) + h.eps) + h.wd * ww[e];
      ww[e] -= h.lr * upd;
    }
    store_stream(reinterpret_cast<float4*>(m + so + i * 4), make_float4(mm[0], mm[1], mm[2], mm[3]));
    store_stream(reinterpret_cast<float4*>(v + so + i * 4), make_float4(vv[0], vv[1], vv[2], vv[3]));
    store_stream(reinterpret_cast<float4*>(w + i * 4), make_float4(ww[0], ww[1], ww[2], ww[3]));
    if (master) {
      if (sizeof(T) == 2) {
        *reinterpret_cast<uint2*>(p + i * 4) = make_uint2(pack_bf16x2(ww[0], ww[1]), pack_bf16x2(ww[2], ww[3]));
      } else {
        *reinterpret_cast<float4*>(p + i * 4) = make_float4(ww[0], ww[1], ww[2], ww[3]);
      }
    }
  }
}

}  // namespace

int launch_masked_adamw(int dtype, int n_experts, long elems, void* param, const unsigned char* mask, float* master, float* m,
                        float* v, const float* grad, float lr, float beta1, float beta2, float eps, float wd, int step,
                        float grad_scale, hipStream_t s) {
  AdamHyper h;
  h.lr = lr; h.beta1 = beta1; h.beta2 = beta2; h.eps = eps; h.wd = wd; h.grad_scale = grad_scale;
  h.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  h.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  const long nvec = elems / 4;
  long gx = (nvec + 255) / 256;           // one vector per thread where the grid allows it
  gx = gx < 1 ? 1 : gx > 8192 ? 8192 : gx;
  SlotTable tb;
  int n = 0;
  long slot = 0;
  auto flush = [&]() -> int {
    if (n == 0) return SPES_OK;
    if (dtype == SPES_F32)
      hipLaunchKernelGGL(masked_adamw_kernel<float>, dim3((unsigned)gx, n), dim3(256), 0, s, tb, (float*)param, master, m, v, grad,
                         nvec, h);
    else
      hipLaunchKernelGGL(masked_adamw_kernel<bf16_t>, dim3((unsigned)gx, n), dim3(256), 0, s, tb, (bf16_t*)param, master, m, v,
                         grad, nvec, h);
    n = 0;
    return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
  };
  for (int e = 0; e < n_experts; ++e) {
    if (!mask[e]) continue;
    tb.param_off[n] = (long)e * elems;
    tb.slot_off[n] = slot * elems;
    ++slot;
    if (++n == kSlotsPerLaunch) {
      const int rc = flush();
      if (rc != SPES_OK) return rc;
    }
  }
  return flush();
}

}  // namespace spes
