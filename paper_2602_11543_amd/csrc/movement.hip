// Bandwidth-bound row movement around the expert GEMMs: gather into
// expert-contiguous order, gate-weighted combine (Eq. 2), and their backward
// counterparts.  All traffic is 16-byte vectors along the contiguous feature
// dimension; sums run in fp32 in a fixed slot order and are rounded once.
#include "kernels.h"

namespace spes {
namespace {

// xp[inv[t*k+j], :] = x[t, :] for j < k: every input row is read once and written to its k places
template <typename T>
__global__ __launch_bounds__(256) void permute_kernel(const T* __restrict__ x, const int* __restrict__ inv, int k,
                                                      T* __restrict__ xp, long total_vec, int nvec, int d) {
  constexpr int N = Vec16<T>::N;
  const long stride = (long)gridDim.x * 256;
  for (long v = (long)blockIdx.x * 256 + threadIdx.x; v < total_vec; v += stride) {
    const long t = v / nvec;
    const int c = (int)(v - t * nvec);
    Vec16<T> q;
    q.load_once(x + t * d + c * N);
    for (int j = 0; j < k; ++j) {
      const long r = inv[t * k + j];
      q.store_once(xp + r * d + c * N);
    }
  }
}

// y[t,:] = sum_j gate[t,j] * yp[inv[t*k+j], :]; KU > 0: k == KU, all k rows are requested before the first is used
template <typename T, int KU>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ yp, const int* __restrict__ inv,
                                                      const float* __restrict__ gate, T* __restrict__ y, long total_vec,
                                                      int nvec, int d, int k) {
  constexpr int N = Vec16<T>::N;
  const long stride = (long)gridDim.x * 256;
  for (long v = (long)blockIdx.x * 256 + threadIdx.x; v < total_vec; v += stride) {
    const long t = v / nvec;
    const int c = (int)(v - t * nvec);
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    if (KU > 0) {
      Vec16<T> q[KU > 0 ? KU : 1];
      float g[KU > 0 ? KU : 1];
#pragma unroll
      for (int j = 0; j < KU; ++j) {
        const long r = inv[t * KU + j];
        g[j] = gate[t * KU + j];
        q[j].load_once(yp + r * d + c * N);
      }
#pragma unroll
      for (int j = 0; j < KU; ++j) {
        float f[N];
        q[j].unpack(f);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(g[j], f[i], acc[i]);
      }
    } else {
      for (int j = 0; j < k; ++j) {
        const long r = inv[t * k + j];
        const float g = gate[t * k + j];
        Vec16<T> q;
        q.load_once(yp + r * d + c * N);
        float f[N];
        q.unpack(f);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(g, f[i], acc[i]);
      }
    }
    Vec16<T> o;
    o.pack(acc);
    o.store_once(y + t * d + c * N);
  }
}

// dx[t,:] = sum_j dxp[inv[t*k+j], :] + router part; one block per token.  The router part is either the row
// dxr[t,:] computed beforehand, or sum_e dlogits[t,e] * w_router[e,:] formed here.
template <typename T>
__global__ __launch_bounds__(256) void dx_gather_kernel(const T* __restrict__ dxp, const int* __restrict__ inv,
                                                        const float* __restrict__ dlogits, const T* __restrict__ w_router,
                                                        const T* __restrict__ dxr, T* __restrict__ dx, int d, int k, int M) {
  constexpr int N = Vec16<T>::N;
  __shared__ float dl[kMaxExperts];
  __shared__ int rows[kMaxExperts];
  const long t = blockIdx.x;
  if (threadIdx.x < M) dl[threadIdx.x] = dlogits[t * M + threadIdx.x];
  if (threadIdx.x < k) rows[threadIdx.x] = inv[t * k + threadIdx.x];
  __syncthreads();
  const int nvec = d / N;
  for (int c = threadIdx.x; c < nvec; c += 256) {
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    for (int j = 0; j < k; ++j) {
      Vec16<T> q;
      q.load_once(dxp + (long)rows[j] * d + c * N);
      float f[N];
      q.unpack(f);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] += f[i];
    }
    if (dxr != nullptr) {
      Vec16<T> q;
      q.load_once(dxr + t * d + c * N);
      float f[N];
      q.unpack(f);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] += f[i];
    } else {
      for (int e = 0; e < M; ++e) {
        Vec16<T> q;
        q.load(w_router + (long)e * d + c * N);
        float f[N];
        q.unpack(f);
        const float s = dl[e];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(s, f[i], acc[i]);
      }
    }
    Vec16<T> o;
    o.pack(acc);
    o.store_once(dx + t * d + c * N);
  }
}

// Backward of the weighted combine as a stand-alone step: for the k routed pairs of token t,
// dyp[inv[t*k+j], :] = gate[t,j] * dy[t, :] and dgate[t,j] = <dy[t, :], yp[inv[t*k+j], :]>.  One block per token: the
// token's dy row is read once and its k scaled copies written, the k rows of yp are read once for the dots.
// KU > 0: k == KU, the thread's k rows of yp are all requested before the first is used.
template <typename T, int KU>
__global__ __launch_bounds__(256) void grad_scatter_kernel(const T* __restrict__ dy, const T* __restrict__ yp,
                                                           const int* __restrict__ inv, const float* __restrict__ gate,
                                                           T* __restrict__ dyp, float* __restrict__ dgate, int d, int k) {
  constexpr int N = Vec16<T>::N;
  __shared__ int rows[kMaxExperts];
  __shared__ float gts[kMaxExperts];
  __shared__ float part[kMaxExperts][4];
  const long t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid < k) { rows[tid] = inv[t * k + tid]; gts[tid] = gate[t * k + tid]; }
  __syncthreads();
  const int nvec = d / N;
  if (KU > 0) {
    float dots[KU > 0 ? KU : 1];
#pragma unroll
    for (int j = 0; j < KU; ++j) dots[j] = 0.f;
    for (int c = tid; c < nvec; c += 256) {
      Vec16<T> q, qy[KU > 0 ? KU : 1];
      q.load_once(dy + t * d + c * N);
#pragma unroll
      for (int j = 0; j < KU; ++j) qy[j].load_once(yp + (long)rows[j] * d + c * N);
      float g[N];
      q.unpack(g);
#pragma unroll
      for (int j = 0; j < KU; ++j) {
        float f[N], o[N];
        qy[j].unpack(f);
#pragma unroll
        for (int i = 0; i < N; ++i) { dots[j] = fmaf(g[i], f[i], dots[j]); o[i] = gts[j] * g[i]; }
        Vec16<T> w;
        w.pack(o);
        w.store_once(dyp + (long)rows[j] * d + c * N);
      }
    }
#pragma unroll
    for (int j = 0; j < KU; ++j) {
      const float v = wave_sum(dots[j]);
      if (lane == 0) part[j][wv] = v;
    }
  } else {
    for (int j = 0; j < k; ++j) {
      float dot = 0.f;
      for (int c = tid; c < nvec; c += 256) {
        Vec16<T> q, qy;
        q.load(dy + t * d + c * N);                    // read again for the next pair: from the cache
        qy.load_once(yp + (long)rows[j] * d + c * N);
        float g[N], f[N], o[N];
        q.unpack(g);
        qy.unpack(f);
#pragma unroll
        for (int i = 0; i < N; ++i) { dot = fmaf(g[i], f[i], dot); o[i] = gts[j] * g[i]; }
        Vec16<T> w;
        w.pack(o);
        w.store_once(dyp + (long)rows[j] * d + c * N);
      }
      const float v = wave_sum(dot);
      if (lane == 0) part[j][wv] = v;
    }
  }
  __syncthreads();
  if (tid < k) dgate[t * k + tid] = (part[tid][0] + part[tid][1]) + (part[tid][2] + part[tid][3]);   // fixed order
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int n_partial, long n,
                                                              float* __restrict__ out, int accumulate) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  float4 acc = accumulate ? *reinterpret_cast<const float4*>(out + i) : make_float4(0.f, 0.f, 0.f, 0.f);
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = 0; p < n_partial; ++p) {
    const float4 v = *reinterpret_cast<const float4*>(partial + (long)p * n + i);
    sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
  }
  acc.x += sum.x; acc.y += sum.y; acc.z += sum.z; acc.w += sum.w;
  *reinterpret_cast<float4*>(out + i) = acc;
}

inline int flat_grid(long total_vec) {
  long b = (total_vec + 255) / 256;       // one vector per thread where the grid allows it
  if (b < 1) b = 1;
  if (b > 1 << 20) b = 1 << 20;
  return (int)b;
}

inline int ok() { return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP; }

}  // namespace

int launch_permute(int dtype, const void* x, const int* inv, int k, void* xp, int T, int d, hipStream_t s) {
  if (dtype == SPES_F32) {
    const int nvec = d / 4;
    hipLaunchKernelGGL(permute_kernel<float>, dim3(flat_grid((long)T * nvec)), dim3(256), 0, s, (const float*)x, inv, k, (float*)xp,
                       (long)T * nvec, nvec, d);
  } else {
    const int nvec = d / 8;
    hipLaunchKernelGGL(permute_kernel<bf16_t>, dim3(flat_grid((long)T * nvec)), dim3(256), 0, s, (const bf16_t*)x, inv, k,
                       (bf16_t*)xp, (long)T * nvec, nvec, d);
  }
  return ok();
}

template <typename T>
void combine_dispatch(const void* yp, const int* inv, const float* gate, void* y, int Tn, int d, int k, hipStream_t s) {
  const int nvec = d / Vec16<T>::N;
  const long total = (long)Tn * nvec;
  const dim3 grid(flat_grid(total));
#define SPES_COMBINE(KU) \
  hipLaunchKernelGGL((combine_kernel<T, KU>), grid, dim3(256), 0, s, (const T*)yp, inv, gate, (T*)y, total, nvec, d, k)
  if (k == 8) SPES_COMBINE(8);
  else if (k == 4) SPES_COMBINE(4);
  else if (k == 2) SPES_COMBINE(2);
  else if (k == 1) SPES_COMBINE(1);
  else SPES_COMBINE(0);
#undef SPES_COMBINE
}

int launch_combine(int dtype, const void* yp, const int* inv, const float* gate, void* y, int T, int d, int k, hipStream_t s) {
  if (dtype == SPES_F32) combine_dispatch<float>(yp, inv, gate, y, T, d, k, s);
  else combine_dispatch<bf16_t>(yp, inv, gate, y, T, d, k, s);
  return ok();
}

template <typename T>
void grad_scatter_dispatch(const void* dy, const void* yp, const int* inv, const float* gate, void* dyp, float* dgate, int Tn,
                           int d, int k, hipStream_t s) {
#define SPES_SCATTER(KU) \
  hipLaunchKernelGGL((grad_scatter_kernel<T, KU>), dim3(Tn), dim3(256), 0, s, (const T*)dy, (const T*)yp, inv, gate, (T*)dyp, dgate, d, k)
  if (k == 8) SPES_SCATTER(8);
  else if (k == 4) SPES_SCATTER(4);
  else if (k == 2) SPES_SCATTER(2);
  else if (k == 1) SPES_SCATTER(1);
  else SPES_SCATTER(0);
#undef SPES_SCATTER
}

int launch_grad_scatter(int dtype, const void* dy, const void* yp, const int* inv, const float* gate, void* dyp, float* dgate,
                        int T, int d, int k, hipStream_t s) {
  if (dtype == SPES_F32) grad_scatter_dispatch<float>(dy, yp, inv, gate, dyp, dgate, T, d, k, s);
  else grad_scatter_dispatch<bf16_t>(dy, yp, inv, gate, dyp, dgate, T, d, k, s);
  return ok();
}

int launch_reduce_partials(const float* partial, int n_partial, long n, float* out, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(cdiv(n, 1024)), dim3(256), 0, s, partial, n_partial, n, out, accumulate);
  return ok();
}

int launch_dx_gather(int dtype, const void* dxp, const int* inv, const float* dlogits, const void* w_router, const void* dxr,
                     void* dx, int T, int d, int k, int M, hipStream_t s) {
  if (dtype == SPES_F32)
    hipLaunchKernelGGL(dx_gather_kernel<float>, dim3(T), dim3(256), 0, s, (const float*)dxp, inv, dlogits,
                       (const float*)w_router, (const float*)dxr, (float*)dx, d, k, M);
  else
    hipLaunchKernelGGL(dx_gather_kernel<bf16_t>, dim3(T), dim3(256), 0, s, (const bf16_t*)dxp, inv, dlogits,
                       (const bf16_t*)w_router, (const bf16_t*)dxr, (bf16_t*)dx, d, k, M);
  return ok();
}

}  // namespace spes
