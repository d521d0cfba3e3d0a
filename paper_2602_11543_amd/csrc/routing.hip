// Routing: softmax/top-k gating, per-expert histogram, prefix scan and the
// stable permutation into expert-contiguous order (paper Sec. 3.2: softmax
// routing, drop-less dispatch).  Integer results are deterministic: no
// order-dependent atomics decide a position.
#include "kernels.h"

namespace spes {
namespace {

// One wavefront per token, one router score per lane.
// logits holds n_part partial score matrices (the router contraction is cut along d_model); their sum plus the
// bias is written back to the first one.
__global__ __launch_bounds__(256) void topk_gate_kernel(float* __restrict__ logits, int n_part, long part_stride,
                                                        const float* __restrict__ bias,
                                                        int T, int M, int k, int renorm, int* __restrict__ topk_idx,
                                                        float* __restrict__ topk_gate, int* __restrict__ idx_copy,
                                                        float* __restrict__ gate_copy, float* __restrict__ lse) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float s = -INFINITY;
  if (lane < M) {
    s = logits[(long)t * M + lane];
    for (int p = 1; p < n_part; ++p) s += logits[p * part_stride + (long)t * M + lane];
    if (bias != nullptr) s += bias[lane];
    if (bias != nullptr || n_part > 1) logits[(long)t * M + lane] = s;   // the backward recomputes probabilities from this score
  }
  const float mx = wave_max(s);
  const float ex = (lane < M) ? expf(s - mx) : 0.f;
  const float sum = wave_sum(ex);
  const float p = ex / sum;
  if (lane == 0) lse[t] = mx + logf(sum);

  bool taken = false;
  int my_idx = 0;
  float my_p = 0.f, psel = 0.f;
  for (int j = 0; j < k; ++j) {
    // selection on the scores: the largest one not taken yet, and among equal scores the lowest lane, which is the
    // lowest expert id (lanes beyond M hold -inf and M >= k, so a real expert is always found)
    const float v = taken ? -INFINITY : s;
    const float top = wave_max(v);
    const int i = __ffsll((long long)__ballot(v == top && !taken)) - 1;
    if (lane == i) taken = true;
    const float pw = lane_value(p, i);
    psel += pw;
    if (lane == j) { my_idx = i; my_p = pw; }
  }
  if (lane < k) {
    const float g = renorm ? my_p / psel : my_p;
    topk_idx[(long)t * k + lane] = my_idx;
    topk_gate[(long)t * k + lane] = g;
    idx_copy[(long)t * k + lane] = my_idx;
    gate_copy[(long)t * k + lane] = g;
  }
}

constexpr int kRankItems = 8;
constexpr int kRankChunk = 256 * kRankItems;   // routed pairs per block

__global__ __launch_bounds__(256) void count_kernel(const int* __restrict__ idx, int R, int* __restrict__ block_counts) {
  __shared__ int h[kMaxExperts];
  if (threadIdx.x < kMaxExperts) h[threadIdx.x] = 0;
  __syncthreads();
  const long base = (long)blockIdx.x * kRankChunk;
#pragma unroll
  for (int i = 0; i < kRankItems; ++i) {
    const long flat = base + i * 256 + threadIdx.x;
    if (flat < R) atomicAdd(&h[idx[flat]], 1);
  }
  __syncthreads();
  if (threadIdx.x < kMaxExperts) block_counts[blockIdx.x * kMaxExperts + threadIdx.x] = h[threadIdx.x];
}

__device__ __forceinline__ int wave_exclusive_scan(int v, int lane) {
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int n = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += n;
  }
  return inc - v;
}

// One wavefront: lane e owns expert e.  Turns per-block counts into per-block
// first positions, and writes counts, offsets and the row-tile tables.
__global__ __launch_bounds__(64) void scan_kernel(int* __restrict__ block_counts, int nblk, int M, int* __restrict__ expert_count,
                                                  int* __restrict__ offset, int bm0, int* __restrict__ tab0, int bm1,
                                                  int* __restrict__ tab1, int max_tiles, float* __restrict__ aux) {
  const int e = threadIdx.x;
  // a new forward pass withdraws the auxiliary-loss gradient terms left for the previous backward pass
  aux[e] = 0.f;
  if (e < kAuxExtra) aux[kMaxExperts + e] = 0.f;
  int total = 0;
#pragma unroll 8
  for (int b = 0; b < nblk; ++b) total += block_counts[b * kMaxExperts + e];
  const int off = wave_exclusive_scan(total, e);
  int running = off;
  // eight independent loads in flight per step: this single wavefront is latency-bound
  int b = 0;
  for (; b + 8 <= nblk; b += 8) {
    int c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = block_counts[(b + u) * kMaxExperts + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      block_counts[(b + u) * kMaxExperts + e] = running;
      running += c[u];
    }
  }
  for (; b < nblk; ++b) {
    const int c = block_counts[b * kMaxExperts + e];
    block_counts[b * kMaxExperts + e] = running;
    running += c;
  }
  if (e < M) { expert_count[e] = total; offset[e] = off; }
  if (e == M - 1) offset[M] = off + total;
  // table layout: [0] = number of tiles, [1 .. max_tiles] expert of each tile, [1+max_tiles ..] first row
  for (int which = 0; which < 2; ++which) {
    const int bm = which ? bm1 : bm0;
    int* tab = which ? tab1 : tab0;
    if (bm <= 0 || tab == nullptr) continue;
    const int nt = (total + bm - 1) / bm;
    const int t0 = wave_exclusive_scan(nt, e);
    for (int i = 0; i < nt; ++i) {
      tab[1 + t0 + i] = e;
      tab[1 + max_tiles + t0 + i] = off + i * bm;
    }
    if (e == 63) tab[0] = t0 + nt;
  }
}

__global__ __launch_bounds__(256) void scatter_kernel(const int* __restrict__ idx, const float* __restrict__ gate, int R, int k,
                                                      const int* __restrict__ block_base, int* __restrict__ perm,
                                                      int* __restrict__ inv, int* __restrict__ row_token,
                                                      float* __restrict__ row_gate) {
  __shared__ int running[kMaxExperts];
  __shared__ int wcnt[4][kMaxExperts];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid < kMaxExperts) {
    running[tid] = block_base[blockIdx.x * kMaxExperts + tid];
    wcnt[0][tid] = wcnt[1][tid] = wcnt[2][tid] = wcnt[3][tid] = 0;
  }
  __syncthreads();
  const long base = (long)blockIdx.x * kRankChunk;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int i = 0; i < kRankItems; ++i) {
    const long flat = base + i * 256 + tid;
    const bool valid = flat < R;
    const int e = valid ? idx[flat] : 0;
    // lanes of this wavefront routed to the same expert
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
      const bool bit = (e >> b) & 1;
      const unsigned long long m = __ballot(valid && bit);
      peers &= bit ? m : ~m;
    }
    const int rank = __popcll(peers & lt);
    if (valid && rank == 0) wcnt[w][e] = __popcll(peers);
    __syncthreads();
    if (valid) {
      int r = running[e] + rank;
      for (int ww = 0; ww < w; ++ww) r += wcnt[ww][e];
      perm[r] = (int)flat;
      inv[flat] = r;
      row_token[r] = (int)(flat / k);      // the same tables in expert-contiguous order, for the GEMM gathers
      row_gate[r] = gate[flat];
    }
    __syncthreads();
    if (tid < kMaxExperts) {
      running[tid] += wcnt[0][tid] + wcnt[1][tid] + wcnt[2][tid] + wcnt[3][tid];
      wcnt[0][tid] = wcnt[1][tid] = wcnt[2][tid] = wcnt[3][tid] = 0;
    }
    __syncthreads();
  }
}

// dlogits from dgate (one wavefront per token).  renorm=0: softmax Jacobian on
// the sparse dp; renorm=1: the renormalised gates are a softmax over the
// selected scores alone.
__global__ __launch_bounds__(256) void gating_bwd_kernel(const float* __restrict__ logits, const float* __restrict__ lse,
                                                         const int* __restrict__ topk_idx, const float* __restrict__ topk_gate,
                                                         const float* __restrict__ dgate_part, int n_part, long part_stride,
                                                         const int* __restrict__ inv, float* __restrict__ dgate, int T, int M,
                                                         int k, int renorm, const float* __restrict__ aux,
                                                         float* __restrict__ dlogits, bf16_t* __restrict__ dlogits_bf) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  // lane j < k holds selected pair j
  int sel = -1; float g = 0.f, dg = 0.f;
  if (lane < k) {
    sel = topk_idx[(long)t * k + lane];
    g = topk_gate[(long)t * k + lane];
    const long r = inv[(long)t * k + lane];
    for (int p = 0; p < n_part; ++p) dg += dgate_part[p * part_stride + r];   // column-tile partials, fixed order
    dgate[(long)t * k + lane] = dg;
  }
  float out = 0.f;
  const float lse_t = lse[t];
  const float p = (lane < M) ? expf(logits[(long)t * M + lane] - lse_t) : 0.f;
  // Every term below has the shape v_e * (u_e - sum_j u_j v_j) with sum_j v_j = 1.  When routing collapses onto one
  // expert (v -> 1 for the top score) that difference cancels completely in fp32 although the true value is about
  // u * (1 - v).  Only the top entry can come close to 1, so it alone is written as
  // v_m * (u_m * sum_{j != m} v_j - sum_{j != m} u_j v_j), which subtracts nothing large; selection is in descending
  // score order, so the top expert is the one of slot 0.
  const int top = __builtin_amdgcn_readlane(sel, 0);
  const float pz = (lane == top) ? 0.f : p;
  const float p_others = wave_sum(pz);
  const float p_top = lane_value(p, top);
  if (renorm) {
    const float gz = (lane == 0) ? 0.f : g;                  // lanes beyond k hold zero gates
    const float g_others = wave_sum(gz);
    const float dot_others = wave_sum(gz * dg);
    const float g0 = lane_value(g, 0), dg0 = lane_value(dg, 0);
    const float mine = (lane == 0) ? g0 * (dg0 * g_others - dot_others) : g * (dg - (dot_others + g0 * dg0));
    // scatter lane j's value to lane sel
    for (int j = 0; j < k; ++j) {
      const int ej = __builtin_amdgcn_readlane(sel, j);     // j is the same for the whole wavefront: scalar reads
      const float vj = lane_value(mine, j);
      if (lane == ej) out = vj;
    }
  } else {
    float dp = 0.f;
    for (int j = 0; j < k; ++j) {
      const int ej = __builtin_amdgcn_readlane(sel, j);
      const float vj = lane_value(dg, j);
      if (lane == ej) dp = vj;
    }
    const float dot_others = wave_sum(dp * pz);
    const float dp_top = lane_value(dp, top);
    out = (lane == top) ? p_top * (dp_top * p_others - dot_others) : p * (dp - (dot_others + dp_top * p_top));
  }
  // auxiliary router losses: aux[e] = dL/dp_e of the load-balancing term (the same for every token),
  // aux[kMaxExperts] = the z-loss factor 2 z / T; both are zero unless armed after the forward pass
  {
    const float c = (lane < M) ? aux[lane] : 0.f;
    const float c_others = wave_sum(c * pz);
    const float c_top = lane_value(c, top);
    const float lb = (lane == top) ? p_top * (c_top * p_others - c_others) : p * (c - (c_others + c_top * p_top));
    out += lb + aux[kMaxExperts] * lse_t * p;
  }
  if (lane < M) {
    dlogits[(long)t * M + lane] = out;
    if (dlogits_bf != nullptr) dlogits_bf[(long)t * M + lane] = f32_to_bf16(out);
  }
}

// Partial sums for the auxiliary router losses: per block, sum_t p_te for every expert and sum_t lse_t^2.
__global__ __launch_bounds__(256) void aux_partial_kernel(const float* __restrict__ logits, const float* __restrict__ lse, int T,
                                                          int M, float* __restrict__ part) {
  __shared__ float acc[4][kMaxExperts + 1];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float ps = 0.f, zs = 0.f;
  // four tokens per step keep four independent loads in flight; the summation order is fixed by the grid alone
  const int step = gridDim.x * 4;
  int t = blockIdx.x * 4 + w;
  for (; t + 3 * step < T; t += 4 * step) {
    float l[4], x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      l[u] = lse[t + u * step];
      x[u] = (lane < M) ? logits[(long)(t + u * step) * M + lane] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ps += expf(x[u] - l[u]);
      zs = fmaf(l[u], l[u], zs);
    }
  }
  for (; t < T; t += step) {
    const float l = lse[t];
    if (lane < M) ps += expf(logits[(long)t * M + lane] - l);
    zs = fmaf(l, l, zs);
  }
  acc[w][lane] = ps;
  if (lane == 0) acc[w][kMaxExperts] = zs;
  __syncthreads();
  if (w == 0) {
    part[blockIdx.x * (kMaxExperts + 1) + lane] = (acc[0][lane] + acc[1][lane]) + (acc[2][lane] + acc[3][lane]);
    if (lane == 0)
      part[blockIdx.x * (kMaxExperts + 1) + kMaxExperts] =
          (acc[0][kMaxExperts] + acc[1][kMaxExperts]) + (acc[2][kMaxExperts] + acc[3][kMaxExperts]);
  }
}

// L_lb = M sum_e f_e P_e and L_z = mean_t lse_t^2 from the block partials (fixed summation order), and the
// gradient factors the gating backward kernel applies.
__global__ __launch_bounds__(256) void aux_final_kernel(const float* __restrict__ part, int nblk, const int* __restrict__ offset,
                                                        int T, int M, int k, float lb_coef, float z_coef, float grad_scale,
                                                        float* __restrict__ losses, float* __restrict__ aux) {
  __shared__ float acc[4][kMaxExperts + 1];
  const int e = threadIdx.x & 63, w = threadIdx.x >> 6;
  float ps = 0.f, zs = 0.f;
  for (int b = w; b < nblk; b += 4) {          // wavefront w adds blocks w, w+4, ...; the four sums are then added in order
    ps += part[b * (kMaxExperts + 1) + e];
    zs += part[b * (kMaxExperts + 1) + kMaxExperts];
  }
  acc[w][e] = ps;
  if (e == 0) acc[w][kMaxExperts] = zs;
  __syncthreads();
  if (w != 0) return;
  ps = (acc[0][e] + acc[1][e]) + (acc[2][e] + acc[3][e]);
  zs = (acc[0][kMaxExperts] + acc[1][kMaxExperts]) + (acc[2][kMaxExperts] + acc[3][kMaxExperts]);
  const float f = (e < M) ? (float)(offset[e + 1] - offset[e]) / ((float)T * (float)k) : 0.f;
  const float P = (e < M) ? ps / (float)T : 0.f;
  const float lb = (float)M * wave_sum(f * P);
  if (e == 0) { losses[0] = lb; losses[1] = zs / (float)T; }
  aux[e] = grad_scale * lb_coef * (float)M * f / (float)T;
  if (e == 0) aux[kMaxExperts] = grad_scale * z_coef * 2.f / (float)T;
}

}  // namespace

int routing_blocks(int R) { return cdiv(R, kRankChunk); }

int launch_topk_gate(float* logits, int n_part, const float* bias, int T, int M, int k, int renorm, int* idx, float* gate,
                     int* idx_copy, float* gate_copy, float* lse, hipStream_t s) {
  hipLaunchKernelGGL(topk_gate_kernel, dim3(cdiv(T, 4)), dim3(256), 0, s, logits, n_part, (long)T * M, bias, T, M, k, renorm,
                     idx, gate, idx_copy, gate_copy, lse);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

int launch_routing_tables(const int* idx, const float* gate, int R, int M, int k, int* block_counts, int* expert_count,
                          int* offset, int* perm, int* inv, int* row_token, float* row_gate, int bm0, int* tab0, int bm1,
                          int* tab1, int max_tiles, float* aux, hipStream_t s) {
  const int nblk = routing_blocks(R);
  hipLaunchKernelGGL(count_kernel, dim3(nblk), dim3(256), 0, s, idx, R, block_counts);
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(64), 0, s, block_counts, nblk, M, expert_count, offset, bm0, tab0, bm1, tab1,
                     max_tiles, aux);
  hipLaunchKernelGGL(scatter_kernel, dim3(nblk), dim3(256), 0, s, idx, gate, R, k, block_counts, perm, inv, row_token, row_gate);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

int launch_gating_bwd(const float* logits, const float* lse, const int* idx, const float* gate, const float* dgate_part,
                      int n_part, long part_stride, const int* inv, float* dgate, int T, int M, int k, int renorm, const float* aux,
                      float* dlogits, bf16_t* dlogits_bf, hipStream_t s) {
  hipLaunchKernelGGL(gating_bwd_kernel, dim3(cdiv(T, 4)), dim3(256), 0, s, logits, lse, idx, gate, dgate_part, n_part, part_stride,
                     inv, dgate, T, M, k, renorm, aux, dlogits, dlogits_bf);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

int launch_router_aux(const float* logits, const float* lse, const int* offset, int T, int M, int k, float lb_coef, float z_coef,
                      float grad_scale, float* part, float* losses, float* aux, hipStream_t s) {
  const int nblk = cdiv(T, 4 * 16) < kAuxBlocks ? cdiv(T, 4 * 16) : kAuxBlocks;
  hipLaunchKernelGGL(aux_partial_kernel, dim3(nblk), dim3(256), 0, s, logits, lse, T, M, part);
  hipLaunchKernelGGL(aux_final_kernel, dim3(1), dim3(256), 0, s, part, nblk, offset, T, M, k, lb_coef, z_coef, grad_scale, losses, aux);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

}  // namespace spes
