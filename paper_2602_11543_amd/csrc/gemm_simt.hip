// Grouped GEMM on the vector ALUs: fp32 FMA, LDS-tiled, any operand strides.
//
// This is the full-precision path (fp32 storage mode needs 1e-5 agreement, which
// rules out bf16 matrix cores) and the path for small or oddly strided
// contractions.  (16*TR)x64 output tile per 256-thread block, TR x 4 outputs per thread (TR = 4, 2 or 1: the
// launcher takes shorter tiles when the taller ones would leave most CUs without a block),
// K advanced 32 at a time through LDS; the next K-tile is requested into registers
// before the current one is multiplied, so its memory latency hides behind the FMAs
// (the shapes this path serves put one block on a CU, where nothing else would).
#include "gemm.h"

namespace spes {
namespace {

constexpr int kRowTile = 64;          // row tile of the ragged-row table; a block takes 16*TR of its rows
constexpr int BN = 64, BK = 32;

template <typename T>
__device__ __forceinline__ float ld(const void* base, long idx) {
  return Elem<T>::load(reinterpret_cast<const T*>(base) + idx);
}

template <typename TA, typename TB, int MODE, int EPI, int TR>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const GemmArgs g) {
  constexpr bool DUAL = (EPI == kEpiSwiglu);
  constexpr int BM = 16 * TR;
  constexpr int kPerA = BM * BK / 256, kPerB = BN * BK / 256;   // elements of an operand tile per thread
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
    const int tile = blockIdx.y / (kRowTile / BM);
    if (tile >= *g.n_tiles) return;
    const int e = g.tile_expert[tile];
    m0 = g.tile_row0[tile] + (blockIdx.y % (kRowTile / BM)) * BM;
    m_end = min((long)g.offset[e + 1], m0 + BM);
    if (m0 >= m_end) return;
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

  float acc[DUAL ? 2 : 1][TR][4];
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[p][i][j] = 0.f;
  // Long contractions are summed in two levels: every kFlush K-tiles the running sums move into `total`, so the
  // rounding error grows with sqrt(kFlush*BK) + sqrt(K / (kFlush*BK)) instead of sqrt(K).
  constexpr int kFlush = 4;
  float total[DUAL ? 2 : 1][TR][4];
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) total[p][i][j] = 0.f;
  int since_flush = 0;

  const bool a_kfast = (g.a_ks == 1), b_kfast = (g.b_ks == 1);
  const int npass = DUAL ? 1 : g.npairs;
  const long ktiles = k_end > k_begin ? (k_end - k_begin + BK - 1) / BK : 0;
  const long ntiles = ktiles * npass;              // K-tiles of all (A,B) pairs, pair after pair

  // position of this thread's element i inside an operand tile, walking the contiguous direction of the operand
  // (k fast: kPer consecutive k of one row; k slow: kPer consecutive rows of one k)
  constexpr int TPA = 256 / BM, TPB = 256 / BN;    // threads per row of the tile, k fast
  const int a_row = a_kfast ? tid / TPA : (tid & 7) * kPerA, a_k = a_kfast ? (tid % TPA) * kPerA : tid >> 3;
  const int b_row = b_kfast ? tid / TPB : (tid & 7) * kPerB, b_k = b_kfast ? (tid % TPB) * kPerB : tid >> 3;

  float ra[kPerA], rb[DUAL ? 2 : 1][kPerB];
  // requests K-tile t (of all pairs) into ra / rb; elements outside the tile's rows, columns or contraction range are 0
  auto fetch = [&](long t) {
    const int pass = (int)(t / ktiles);
    const long kk = k_begin + (t - pass * ktiles) * BK;
    const void* Ap = g.A[pass];
#pragma unroll
    for (int i = 0; i < kPerA; ++i) {
      const int ml = a_kfast ? a_row : a_row + i, kl = a_kfast ? a_k + i : a_k;
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
      ra[i] = v;
    }
#pragma unroll
    for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
      const void* Bp = g.B[DUAL ? p : pass];
#pragma unroll
      for (int i = 0; i < kPerB; ++i) {
        const int nl = b_kfast ? b_row : b_row + i, kl = b_kfast ? b_k + i : b_k;
        const long n = n0 + nl, k = kk + kl;
        float v = 0.f;
        if (n < g.Ndim && k < k_end) {
          const long row = (MODE == kGroupedK && g.b_rows) ? (long)g.b_rows[k] : k;
          v = ld<TB>(Bp, b_group + n * g.b_ns + row * g.b_ks);
        }
        rb[p][i] = v;
      }
    }
  };

  if (ntiles > 0) fetch(0);
  for (long t = 0; t < ntiles; ++t) {
#pragma unroll
    for (int i = 0; i < kPerA; ++i) As[a_kfast ? a_k + i : a_k][a_kfast ? a_row : a_row + i] = ra[i];
#pragma unroll
    for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
      for (int i = 0; i < kPerB; ++i) Bs[p][b_kfast ? b_k + i : b_k][b_kfast ? b_row : b_row + i] = rb[p][i];
    __syncthreads();
    if (t + 1 < ntiles) fetch(t + 1);              // in flight while this tile is multiplied
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[TR];
#pragma unroll
      for (int i = 0; i < TR; ++i) a[i] = As[k][ty * TR + i];
#pragma unroll
      for (int p = 0; p < (DUAL ? 2 : 1); ++p) {
        float b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[p][k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < TR; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[p][i][j] = fmaf(a[i], b[j], acc[p][i][j]);
      }
    }
    if (++since_flush == kFlush) {
      since_flush = 0;
#pragma unroll
      for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
        for (int i = 0; i < TR; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) { total[p][i][j] += acc[p][i][j]; acc[p][i][j] = 0.f; }
    }
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < (DUAL ? 2 : 1); ++p)
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[p][i][j] += total[p][i][j];

  float dots[TR];
#pragma unroll
  for (int i = 0; i < TR; ++i) dots[i] = 0.f;
#pragma unroll
  for (int i = 0; i < TR; ++i) {
    const long m = m0 + ty * TR + i;
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
    for (int i = 0; i < TR; ++i) Red[ty * TR + i][tx] = dots[i];
    __syncthreads();
    if (tid < BM && m0 + tid < m_end) {
      float sum = 0.f;
#pragma unroll
      for (int c = 0; c < 16; ++c) sum += Red[tid][c];
      g.rowdot[(long)blockIdx.x * g.rowdot_stride + m0 + tid] = sum;
    }
  }
}

template <typename TA, typename TB, int MODE, int EPI, int TR>
int launch_tile(const GemmArgs& g, hipStream_t s) {
  constexpr int BM = 16 * TR;
  dim3 grid;
  if (MODE == kRaggedM) {
    grid = dim3(cdiv(g.Ndim, BN), g.max_tiles * (kRowTile / BM), 1);
  } else {
    grid = dim3(cdiv(g.Ndim, BN), cdiv(g.Mdim, BM), g.n_groups);
  }
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return SPES_OK;
  hipLaunchKernelGGL((gemm_simt_kernel<TA, TB, MODE, EPI, TR>), grid, dim3(256), 0, s, g);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

// 64-row tiles when they give every CU two blocks or more, otherwise 32- or 16-row tiles (a block of a small problem
// is bound by its own serial K loop, so more, shorter blocks finish sooner)
template <typename TA, typename TB, int MODE, int EPI>
int launch(const GemmArgs& g, hipStream_t s) {
  const long rows64 = (MODE == kRaggedM) ? g.max_tiles : (long)cdiv(g.Mdim, kRowTile) * g.n_groups;
  const long blocks64 = rows64 * cdiv(g.Ndim, BN);
  if (blocks64 >= 512) return launch_tile<TA, TB, MODE, EPI, 4>(g, s);
  if (blocks64 >= 256) return launch_tile<TA, TB, MODE, EPI, 2>(g, s);
  return launch_tile<TA, TB, MODE, EPI, 1>(g, s);
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
int simt_row_tile() { return kRowTile; }
int simt_col_tile() { return BN; }

int launch_gemm_simt(int dtype_a, int dtype_b, int mode, int epi, const GemmArgs& g, hipStream_t s) {
  if (dtype_a == SPES_F32 && dtype_b == SPES_F32) return dispatch<float, float>(mode, epi, g, s);
  if (dtype_a == SPES_BF16 && dtype_b == SPES_BF16) return dispatch<bf16_t, bf16_t>(mode, epi, g, s);
  if (dtype_a == SPES_F32 && dtype_b == SPES_BF16) return dispatch<float, bf16_t>(mode, epi, g, s);
  return SPES_EINVAL;
}

}  // namespace spes
