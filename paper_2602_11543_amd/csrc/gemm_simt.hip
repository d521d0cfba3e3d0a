// Grouped GEMM on the vector ALUs: fp32 FMA, LDS-tiled, any operand strides.
//
// This is the full-precision path (fp32 storage mode needs 1e-5 agreement, which
// rules out bf16 matrix cores) and the path for small or oddly strided
// contractions.  64x64 output tile per 256-thread block, 4x4 outputs per thread,
// K advanced 16 at a time through LDS.
#include "gemm.h"

namespace spes {
namespace {

constexpr int BM = 64, BN = 64, BK = 16;

template <typename T>
__device__ __forceinline__ float ld(const void* base, long idx) {
  return Elem<T>::load(reinterpret_cast<const T*>(base) + idx);
}

template <typename TA, typename TB, int MODE, int EPI>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const GemmArgs g) {
  constexpr bool DUAL = (EPI == kEpiSwiglu);
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[DUAL ? 2 : 1][BK][BN + 4];
  __shared__ float Red[EPI == kEpiDSwiglu ? BM : 1][17];

  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int n0 = blockIdx.x * BN;

  long m0, m_end;        // rows of A / C covered by this block
  long k_begin, k_end;   // contraction range
  long b_group = 0, c_group = 0;
  if (MODE == kRaggedM) {
    const int tile = blockIdx.y;
    if (tile >= *g.n_tiles) return;
    const int e = g.tile_expert[tile];
    m0 = g.tile_row0[tile];
    m_end = min((long)g.offset[e + 1], m0 + BM);
    k_begin = 0; k_end = g.Kdim;
    b_group = (long)e * g.b_gs;
  } else {
    const int grp = blockIdx.z;
    m0 = (long)blockIdx.y * BM;
    m_end = min((long)g.Mdim, m0 + BM);
    if (g.offset != nullptr) {
      const int e = g.group_expert[grp];
      k_begin = g.offset[e]; k_end = g.offset[e + 1];
    } else {
      k_begin = (long)grp * g.kchunk; k_end = min((long)g.Kdim, k_begin + g.kchunk);
    }
    c_group = (long)grp * g.c_gs;
  }

  float acc[DUAL ? 2 : 1][4][4];
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[p][i][j] = 0.f;
  // Long contractions are summed in two levels: every kFlush K-tiles the running sums move into `total`, so the
  // rounding error grows with sqrt(kFlush*BK) + sqrt(K / (kFlush*BK)) instead of sqrt(K).
  constexpr int kFlush = 8;
  float total[DUAL ? 2 : 1][4][4];
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) total[p][i][j] = 0.f;
  int since_flush = 0;

  const bool a_kfast = (g.a_ks == 1), b_kfast = (g.b_ks == 1);
  const int npass = DUAL ? 1 : g.npairs;
  for (int pass = 0; pass < npass; ++pass) {
    const void* Ap = g.A[pass];
    for (long kk = k_begin; kk < k_end; kk += BK) {
      // stage A: 64 x 16 elements, 4 per thread, walking the contiguous direction
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int ml, kl;
        if (a_kfast) { ml = tid >> 2; kl = (tid & 3) * 4 + i; } else { kl = tid >> 4; ml = (tid & 15) * 4 + i; }
        const long m = m0 + ml, k = kk + kl;
        float v = 0.f;
        if (m < m_end && k < k_end) {
          if (MODE == kRaggedM) {
            const long row = g.a_rows ? (long)g.a_rows[m] : m;
            v = ld<TA>(Ap, row * g.a_ms + k * g.a_ks);
          } else {
            const long row = g.a_rows ? (long)g.a_rows[k] : k;
            v = ld<TA>(Ap, m * g.a_ms + row * g.a_ks);
          }
        }
        As[kl][ml] = v;
      }
#pragma unroll
      for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
        const void* Bp = g.B[DUAL ? p : pass];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int nl, kl;
          if (b_kfast) { nl = tid >> 2; kl = (tid & 3) * 4 + i; } else { kl = tid >> 4; nl = (tid & 15) * 4 + i; }
          const long n = n0 + nl, k = kk + kl;
          float v = 0.f;
          if (n < g.Ndim && k < k_end) {
            const long row = (MODE == kGroupedK && g.b_rows) ? (long)g.b_rows[k] : k;
            v = ld<TB>(Bp, b_group + n * g.b_ns + row * g.b_ks);
          }
          Bs[p][kl][nl] = v;
        }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BK; ++k) {
        float a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
          float b[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) b[j] = Bs[p][k][tx * 4 + j];
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[p][i][j] = fmaf(a[i], b[j], acc[p][i][j]);
        }
      }
      if (++since_flush == kFlush) {
        since_flush = 0;
#pragma unroll
        for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) { total[p][i][j] += acc[p][i][j]; acc[p][i][j] = 0.f; }
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[p][i][j] += total[p][i][j];

  float dots[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const long m = m0 + ty * 4 + i;
    if (m >= m_end) continue;
    const float rs = (EPI == kEpiDSwiglu) ? g.row_scale[m] : 1.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const long n = n0 + tx * 4 + j;
      if (n >= g.Ndim) continue;
      const long ci = c_group + m * g.c_ms + n;
      if (EPI == kEpiStore) {
        if (g.c_f32) {
          float* c = reinterpret_cast<float*>(g.C[0]) + ci;
          *c = g.accumulate ? (*c + acc[0][i][j]) : acc[0][i][j];
        } else {
          Elem<TB>::store(reinterpret_cast<TB*>(g.C[0]) + ci, acc[0][i][j]);
        }
      } else if (EPI == kEpiSwiglu) {
        const float a = acc[0][i][j], b = acc[DUAL ? 1 : 0][i][j];
        reinterpret_cast<float*>(g.C[0])[ci] = a;
        reinterpret_cast<float*>(g.C[1])[ci] = b;
        Elem<TB>::store(reinterpret_cast<TB*>(g.C[2]) + ci, a * sigmoidf_(a) * b);
      } else {
        const float u = acc[0][i][j];
        const float a = reinterpret_cast<const float*>(g.E[0])[ci], b = reinterpret_cast<const float*>(g.E[1])[ci];
        const float sg = sigmoidf_(a);
        const float h = a * sg * b;
        dots[i] = fmaf(u, h, dots[i]);
        const float dh = rs * u;
        Elem<TB>::store(reinterpret_cast<TB*>(g.C[2]) + ci, rs * h);
        Elem<TB>::store(reinterpret_cast<TB*>(g.C[0]) + ci, dh * b * sg * (1.f + a * (1.f - sg)));
        Elem<TB>::store(reinterpret_cast<TB*>(g.C[1]) + ci, dh * a * sg);
      }
    }
  }
  if (EPI == kEpiDSwiglu) {
    // gate-gradient partial of this column tile: fixed-order sum over the 16 column threads of each row
#pragma unroll
    for (int i = 0; i < 4; ++i) Red[ty * 4 + i][tx] = dots[i];
    __syncthreads();
    if (tid < BM && m0 + tid < m_end) {
      float sum = 0.f;
#pragma unroll
      for (int c = 0; c < 16; ++c) sum += Red[tid][c];
      g.rowdot[(long)blockIdx.x * g.rowdot_stride + m0 + tid] = sum;
    }
  }
}

template <typename TA, typename TB, int MODE, int EPI>
int launch(const GemmArgs& g, hipStream_t s) {
  dim3 grid;
  if (MODE == kRaggedM) {
    grid = dim3(cdiv(g.Ndim, BN), g.max_tiles, 1);
  } else {
    grid = dim3(cdiv(g.Ndim, BN), cdiv(g.Mdim, BM), g.n_groups);
  }
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return SPES_OK;
  hipLaunchKernelGGL((gemm_simt_kernel<TA, TB, MODE, EPI>), grid, dim3(256), 0, s, g);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

template <typename TA, typename TB>
int dispatch(int mode, int epi, const GemmArgs& g, hipStream_t s) {
  if (mode == kRaggedM) {
    if (epi == kEpiStore) return launch<TA, TB, kRaggedM, kEpiStore>(g, s);
    if (epi == kEpiSwiglu) return launch<TA, TB, kRaggedM, kEpiSwiglu>(g, s);
    return launch<TA, TB, kRaggedM, kEpiDSwiglu>(g, s);
  }
  if (epi == kEpiStore) return launch<TA, TB, kGroupedK, kEpiStore>(g, s);
  return SPES_EINVAL;
}

}  // namespace

// Row tile of the ragged-M table this kernel expects, and its column tile.
int simt_row_tile() { return BM; }
int simt_col_tile() { return BN; }

int launch_gemm_simt(int dtype_a, int dtype_b, int mode, int epi, const GemmArgs& g, hipStream_t s) {
  if (dtype_a == SPES_F32 && dtype_b == SPES_F32) return dispatch<float, float>(mode, epi, g, s);
  if (dtype_a == SPES_BF16 && dtype_b == SPES_BF16) return dispatch<bf16_t, bf16_t>(mode, epi, g, s);
  if (dtype_a == SPES_F32 && dtype_b == SPES_BF16) return dispatch<float, bf16_t>(mode, epi, g, s);
  return SPES_EINVAL;
}

}  // namespace spes
