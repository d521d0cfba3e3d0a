// Grouped bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// A 256-thread block (four wavefronts, 2 x 2) computes a BM x BN output tile, each
// wavefront a (BM/2) x (BN/2) sub-tile as TM x TN MFMA tiles of 32 x 32 held in AGPRs.
// Operand tiles are staged global -> registers -> LDS with two LDS stages:
//   * the global loads of K-tile t+2 are issued right after the registers of tile t+1
//     were written to LDS, so they have a whole iteration to land;
//   * MFMA fragments are double-buffered in registers: the reads of k-step s+1 are
//     issued before the MFMAs of k-step s, and the first fragments of the next K-tile
//     are read (after the block barrier) under the last MFMAs of the current one.
// Both operands live in LDS as [row][k] with a row pitch of BK*2+16 bytes, which
// spreads the fragment reads (16 rows x one 16-byte chunk) over all banks.
// An operand whose contraction index is the slow memory axis (the weights in the
// input-gradient GEMMs, both operands of the weight-gradient GEMMs) is transposed in
// registers (8x8 blocks, v_perm) on its way into LDS.
// Loads are unconditional: rows and k beyond the operand are clamped to valid
// addresses, the k tail is zeroed by select, surplus rows are never stored.
//
// The MFMA operands are swapped (weights tile as the "A" input) so that each lane ends
// up holding runs of four consecutive output columns of one row: epilogues then work
// on 8- and 16-byte vectors along the contiguous dimension.
//
// Tiles are enumerated on a 1-D grid and dealt out so that every XCD (workgroups are
// assigned to the eight XCDs round-robin) gets one contiguous range of tiles: tiles
// that share an expert's weight panel or a row panel meet in the same L2.
#include "gemm.h"

namespace spes {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kXcds = 8;

template <int BM_, int BN_, int BK_, int MINB_>
struct Cfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, MINB = MINB_;
  static constexpr int TM = BM / 64, TN = BN / 64;          // MFMA tiles per wavefront along m, n
  static constexpr int KSTEPS = BK / 16;
  static constexpr int CH = BK / 8;                         // 16-byte chunks of data per LDS row
  static constexpr int PITCH = CH + 1;                      // row pitch in 16-byte units
  static constexpr int RP = 256 / CH;                       // rows staged per pass (K-contiguous operand)
  static constexpr int NA = BM / RP, NB = BN / RP;          // staging registers (uint4) per thread, K-contiguous
  static constexpr int A_VEC = BM * PITCH, B_VEC = BN * PITCH;
  static constexpr int STAGE_VEC = A_VEC + B_VEC;
  // K-strided staging: 8x8 blocks, (rows/8)*CH of them per tile, spread over the 256 threads
  static constexpr int ABLK = BM / 8 * CH, BBLK = BN / 8 * CH;
  static constexpr int NAB = ABLK >= 256 ? ABLK / 256 : 1, NBB = BBLK >= 256 ? BBLK / 256 : 1;
  static constexpr int RA = NA > 8 * NAB ? NA : 8 * NAB;    // staging register counts covering both kinds
  static constexpr int RB = NB > 8 * NBB ? NB : 8 * NBB;
};

__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ uint4 sel4(bool keep, const uint4& v) { return keep ? v : zero4(); }
__device__ __forceinline__ uint32_t pack2(float a, float b) { return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16); }

// out row i of an 8x8 block gets k_0..k_7 of row i; in[j] holds rows 0..7 at k_j
__device__ __forceinline__ uint4 transpose_row(const uint4* in, int i) {
  uint32_t w[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const uint32_t lo = (i >> 1) == 0 ? in[2 * m].x : (i >> 1) == 1 ? in[2 * m].y : (i >> 1) == 2 ? in[2 * m].z : in[2 * m].w;
    const uint32_t hi =
        (i >> 1) == 0 ? in[2 * m + 1].x : (i >> 1) == 1 ? in[2 * m + 1].y : (i >> 1) == 2 ? in[2 * m + 1].z : in[2 * m + 1].w;
    w[m] = (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

template <int MODE, int EPI, bool A_KC, bool B_KC, typename C>
__global__ __launch_bounds__(256, C::MINB) void gemm_mfma_kernel(const GemmArgs g) {
  constexpr int BM = C::BM, BN = C::BN, BK = C::BK, TM = C::TM, TN = C::TN, CH = C::CH, RP = C::RP;
  __shared__ uint4 smem[2 * C::STAGE_VEC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhalf = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int BNO = (EPI == kEpiSwiglu) ? BN / 2 : BN;   // output columns per tile

  // ---- which tile ----
  const int gx = cdiv(g.Ndim, BNO);
  long total;
  if (MODE == kRaggedM) total = (long)(*g.n_tiles) * gx; else total = (long)g.n_groups * cdiv(g.Mdim, BM) * gx;
  const long per_xcd = (total + kXcds - 1) / kXcds;
  const long slot = blockIdx.x / kXcds;
  const long logical = (long)(blockIdx.x % kXcds) * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int nt = (int)(logical % gx);
  const long mt_all = logical / gx;

  long m0, m_end, k_begin, k_end, b_group = 0, c_group = 0;
  if (MODE == kRaggedM) {
    const int e = g.tile_expert[mt_all];
    m0 = g.tile_row0[mt_all];
    m_end = min((long)g.offset[e + 1], m0 + BM);
    k_begin = 0; k_end = g.Kdim;
    b_group = (long)e * g.b_gs;
  } else {
    const int my = cdiv(g.Mdim, BM);
    const int grp = (int)(mt_all / my);
    m0 = (mt_all % my) * BM;
    m_end = min((long)g.Mdim, m0 + BM);
    if (g.offset != nullptr) {
      const int e = g.group_expert[grp];
      k_begin = g.offset[e]; k_end = g.offset[e + 1];
    } else {
      k_begin = (long)grp * g.kchunk; k_end = min((long)g.Kdim, k_begin + g.kchunk);
    }
    c_group = (long)grp * g.c_gs;
  }
  const long n0 = (long)nt * BNO;

  // ---- K-contiguous operands: source row of each staged tile row (clamped into the operand) ----
  long arow[A_KC ? C::NA : 1];
  long brow[B_KC ? C::NB : 1];
  bool bsecond[B_KC ? C::NB : 1];   // fused SwiGLU: the row comes from the second matrix
  if (A_KC) {
#pragma unroll
    for (int i = 0; i < C::NA; ++i) {
      long m = m0 + tid / CH + RP * i;
      m = m < m_end ? m : m_end - 1;
      arow[i] = ((MODE == kRaggedM && g.a_rows) ? (long)g.a_rows[m] : m) * g.a_ms;
    }
  }
  if (B_KC) {
#pragma unroll
    for (int i = 0; i < C::NB; ++i) {
      const int nl = tid / CH + RP * i;
      long col;
      bsecond[i] = false;
      if (EPI == kEpiSwiglu) {
        // tile row nl -> wave column, then (BN/4) gate columns followed by the matching (BN/4) up columns
        constexpr int W = BN / 2, H = BN / 4;
        col = n0 + (nl / W) * H + (nl % H);
        bsecond[i] = ((nl % W) / H) != 0;
      } else {
        col = n0 + nl;
      }
      col = col < g.Ndim ? col : g.Ndim - 1;
      brow[i] = b_group + col * g.b_ns;
    }
  }

  f32x16 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const int npass = (EPI == kEpiSwiglu) ? 1 : g.npairs;
  const long klen = k_end - k_begin;
  const int nk = (int)((klen + BK - 1) / BK);
  const int nsteps = nk * npass;

  uint4 ra[C::RA], rb[C::RB];
  unsigned a_keep = 0, b_keep = 0;   // which staged k (bit j; K-contiguous: all or none) lie inside the contraction range

  // global -> registers for K-tile `step`
  auto gload = [&](int step) {
    const int pass = step / nk;
    const long k0 = k_begin + (long)(step - pass * nk) * BK;
    if (A_KC) {
      const bf16_t* base = reinterpret_cast<const bf16_t*>(g.A[pass]);
      const long k = k0 + (tid % CH) * 8;
      const bool kin = k < k_end;
      const long kc = kin ? k : k_begin;
#pragma unroll
      for (int i = 0; i < C::NA; ++i) ra[i] = *reinterpret_cast<const uint4*>(base + arow[i] + kc);
      a_keep = kin ? 0xffu : 0u;
    } else {
      const bf16_t* base = reinterpret_cast<const bf16_t*>(g.A[pass]);
#pragma unroll
      for (int q = 0; q < C::NAB; ++q) {
        const int blk = tid + 256 * q;
        if (C::ABLK >= 256 || blk < C::ABLK) {
          const long k = k0 + (blk % CH) * 8;
          long row = m0 + (blk / CH) * 8;
          row = row < m_end ? row : m0;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const long kj = k + j < k_end ? k + j : k_end - 1;
            const long kr = g.a_rows ? (long)g.a_rows[kj] : kj;
            ra[q * 8 + j] = *reinterpret_cast<const uint4*>(base + kr * g.a_ks + row);
          }
          const long left = k_end - k;
          a_keep = left >= 8 ? 0xffu : left <= 0 ? 0u : ((1u << left) - 1u);   // same k for every q: ABLK >= 256 only if CH | 256
        }
      }
    }
    if (B_KC) {
      const bf16_t* base0 = reinterpret_cast<const bf16_t*>(g.B[(EPI == kEpiSwiglu) ? 0 : pass]);
      const bf16_t* base1 = reinterpret_cast<const bf16_t*>(g.B[1]);
      const long k = k0 + (tid % CH) * 8;
      const bool kin = k < k_end;
      const long kc = kin ? k : k_begin;
#pragma unroll
      for (int i = 0; i < C::NB; ++i) {
        const bf16_t* base = (EPI == kEpiSwiglu && bsecond[i]) ? base1 : base0;
        rb[i] = *reinterpret_cast<const uint4*>(base + brow[i] + kc);
      }
      b_keep = kin ? 0xffu : 0u;
    } else {
      const bf16_t* base = reinterpret_cast<const bf16_t*>(g.B[pass]) + b_group;
#pragma unroll
      for (int q = 0; q < C::NBB; ++q) {
        const int blk = tid + 256 * q;
        if (C::BBLK >= 256 || blk < C::BBLK) {
          const long k = k0 + (blk % CH) * 8;
          long row = n0 + (blk / CH) * 8;
          row = row < g.Ndim ? row : n0;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const long kj = k + j < k_end ? k + j : k_end - 1;
            rb[q * 8 + j] = *reinterpret_cast<const uint4*>(base + kj * g.b_ks + row);
          }
          const long left = k_end - k;
          b_keep = left >= 8 ? 0xffu : left <= 0 ? 0u : ((1u << left) - 1u);
        }
      }
    }
  };

  // registers -> LDS stage
  auto stash = [&](int stage) {
    uint4* ta = smem + stage * C::STAGE_VEC;
    uint4* tb = ta + C::A_VEC;
    if (A_KC) {
#pragma unroll
      for (int i = 0; i < C::NA; ++i) ta[(tid / CH + RP * i) * C::PITCH + tid % CH] = sel4(a_keep != 0, ra[i]);
    } else {
#pragma unroll
      for (int q = 0; q < C::NAB; ++q) {
        const int blk = tid + 256 * q;
        if (C::ABLK >= 256 || blk < C::ABLK) {
          if (a_keep != 0xffu) {
#pragma unroll
            for (int j = 0; j < 8; ++j) ra[q * 8 + j] = sel4((a_keep >> j) & 1u, ra[q * 8 + j]);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) ta[((blk / CH) * 8 + i) * C::PITCH + blk % CH] = transpose_row(&ra[q * 8], i);
        }
      }
    }
    if (B_KC) {
#pragma unroll
      for (int i = 0; i < C::NB; ++i) tb[(tid / CH + RP * i) * C::PITCH + tid % CH] = sel4(b_keep != 0, rb[i]);
    } else {
#pragma unroll
      for (int q = 0; q < C::NBB; ++q) {
        const int blk = tid + 256 * q;
        if (C::BBLK >= 256 || blk < C::BBLK) {
          if (b_keep != 0xffu) {
#pragma unroll
            for (int j = 0; j < 8; ++j) rb[q * 8 + j] = sel4((b_keep >> j) & 1u, rb[q * 8 + j]);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) tb[((blk / CH) * 8 + i) * C::PITCH + blk % CH] = transpose_row(&rb[q * 8], i);
        }
      }
    }
  };

  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frags = [&](int stage, int ks, int set) {
    const uint4* ta = smem + stage * C::STAGE_VEC;
    const uint4* tb = ta + C::A_VEC;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      fa[set][i] = __builtin_bit_cast(bf16x8, ta[(wm * (BM / 2) + i * 32 + l32) * C::PITCH + ks * 2 + lhalf]);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      fb[set][j] = __builtin_bit_cast(bf16x8, tb[(wn * (BN / 2) + j * 32 + l32) * C::PITCH + ks * 2 + lhalf]);
  };
  auto mfmas = [&](int set) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int i = 0; i < TM; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[j][i], 0, 0, 0);
  };

  if (nsteps > 0) {
    gload(0);
    stash(0);
    if (nsteps > 1) gload(1);
    __syncthreads();
    read_frags(0, 0, 0);
    constexpr int WRITE_KS = C::KSTEPS >= 4 ? 1 : 0;
    for (int t = 0; t < nsteps; ++t) {
      const int cur = t & 1;
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS; ++ks) {
        const int set = ks & 1;
        if (ks + 1 < C::KSTEPS) {
          read_frags(cur, ks + 1, set ^ 1);
        } else if (t + 1 < nsteps) {
          read_frags(cur ^ 1, 0, set ^ 1);     // next K-tile, published by the barrier below
        }
        if (ks == WRITE_KS) {
          if (t + 1 < nsteps && !(g.dbg & 2)) stash(cur ^ 1);
          if (t + 2 < nsteps && !(g.dbg & 1)) gload(t + 2);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (!(g.dbg & 4)) mfmas(set);
        __builtin_amdgcn_sched_barrier(0);
        if (ks == C::KSTEPS - 2) __syncthreads();
      }
    }
  }

  // ---- epilogue: lane holds row m = .. + l32 and, per register group gq, columns gq*8 + lhalf*4 + 0..3 ----
  if (g.dbg & 8) return;
  if (EPI == kEpiStore) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const long m = m0 + wm * (BM / 2) + i * 32 + l32;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const long n = n0 + wn * (BN / 2) + j * 32 + gq * 8 + lhalf * 4;
          if (n >= g.Ndim) continue;
          const long ci = c_group + m * g.c_ms + n;
          const float v0 = acc[j][i][gq * 4], v1 = acc[j][i][gq * 4 + 1], v2 = acc[j][i][gq * 4 + 2], v3 = acc[j][i][gq * 4 + 3];
          if (g.c_f32) {
            float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C[0]) + ci);
            float4 o = make_float4(v0, v1, v2, v3);
            if (g.accumulate) { const float4 old = *c; o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w; }
            *c = o;
          } else {
            *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[0]) + ci) = make_uint2(pack2(v0, v1), pack2(v2, v3));
          }
        }
    }
  } else if (EPI == kEpiSwiglu) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const long m = m0 + wm * (BM / 2) + i * 32 + l32;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN / 2; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const long n = n0 + wn * (BN / 4) + j * 32 + gq * 8 + lhalf * 4;
          if (n >= g.Ndim) continue;
          const long ci = m * g.c_ms + n;
          float a[4], b[4], h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[e] = acc[j][i][gq * 4 + e];
            b[e] = acc[j + TN / 2][i][gq * 4 + e];
            h[e] = a[e] * sigmoidf_(a[e]) * b[e];
          }
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C[0]) + ci) = make_float4(a[0], a[1], a[2], a[3]);
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C[1]) + ci) = make_float4(b[0], b[1], b[2], b[3]);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[2]) + ci) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
        }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const long m = m0 + wm * (BM / 2) + i * 32 + l32;
      const bool min_ = m < m_end;
      const float rs = min_ ? g.row_scale[m] : 0.f;
      float dot = 0.f;
      if (min_) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const long n = n0 + wn * (BN / 2) + j * 32 + gq * 8 + lhalf * 4;
            if (n >= g.Ndim) continue;
            const long ci = m * g.c_ms + n;
            const float4 av = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g.E[0]) + ci);
            const float4 bv = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g.E[1]) + ci);
            const float a[4] = {av.x, av.y, av.z, av.w}, b[4] = {bv.x, bv.y, bv.z, bv.w};
            float da[4], db[4], hg[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float u = acc[j][i][gq * 4 + e];
              const float sg = sigmoidf_(a[e]);
              const float as = a[e] * sg;          // SiLU(a)
              const float h = as * b[e];
              dot = fmaf(u, h, dot);
              const float dh = rs * u;
              da[e] = dh * b[e] * (sg + as * (1.f - sg));
              db[e] = dh * as;
              hg[e] = rs * h;
            }
            *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[0]) + ci) = make_uint2(pack2(da[0], da[1]), pack2(da[2], da[3]));
            *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[1]) + ci) = make_uint2(pack2(db[0], db[1]), pack2(db[2], db[3]));
            *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[2]) + ci) = make_uint2(pack2(hg[0], hg[1]), pack2(hg[2], hg[3]));
          }
      }
      // the two half-waves hold the two column halves of the same row
      dot += __shfl_xor(dot, 32, kWave);
      if (min_ && lhalf == 0) g.rowdot[(long)(nt * 2 + wn) * g.rowdot_stride + m] = dot;
    }
  }
}

// tile configurations: 256 x 128 x 32 with two blocks per CU (2 x 60 KB of LDS, 128 accumulators per lane),
// or 256 x 256 x 64 with one block per CU (144 KB of LDS, 256 accumulators per lane)
typedef Cfg<256, 128, 32, 2> Small;
typedef Cfg<256, 256, 64, 1> Large;
int g_tile = 0;   // 0: Small, 1: Large
int g_dbg = 0;

template <int MODE, int EPI, bool A_KC, bool B_KC, typename C>
int launch_cfg(const GemmArgs& g, hipStream_t s) {
  const int bno = (EPI == kEpiSwiglu) ? C::BN / 2 : C::BN;
  const int gx = cdiv(g.Ndim, bno);
  long total = (MODE == kRaggedM) ? (long)g.max_tiles * gx : (long)g.n_groups * cdiv(g.Mdim, C::BM) * gx;
  if (total <= 0) return SPES_OK;
  total = (total + kXcds - 1) / kXcds * kXcds;
  GemmArgs gg = g;
  gg.dbg = g_dbg;
  hipLaunchKernelGGL((gemm_mfma_kernel<MODE, EPI, A_KC, B_KC, C>), dim3((unsigned)total), dim3(256), 0, s, gg);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

template <int MODE, int EPI, bool A_KC, bool B_KC>
int launch(const GemmArgs& g, hipStream_t s) {
  if (g_tile == 1) return launch_cfg<MODE, EPI, A_KC, B_KC, Large>(g, s);
  return launch_cfg<MODE, EPI, A_KC, B_KC, Small>(g, s);
}

}  // namespace

void mfma_set_tile(int t) { g_tile = t & 0xff; g_dbg = t >> 8; }
int mfma_row_tile() { return 256; }
// number of gate-gradient partials per row that the kEpiDSwiglu epilogue writes for ndim columns
int mfma_rowdot_parts(int ndim) { return 2 * cdiv(ndim, g_tile == 1 ? Large::BN : Small::BN); }
// bf16 operands only.  a_kcontig / b_kcontig: the contraction index is the fast memory axis of that operand.
int launch_gemm_mfma(int mode, int epi, bool a_kcontig, bool b_kcontig, const GemmArgs& g, hipStream_t s) {
  if (mode == kRaggedM) {
    if (!a_kcontig) return SPES_EINVAL;
    if (epi == kEpiSwiglu && b_kcontig) return launch<kRaggedM, kEpiSwiglu, true, true>(g, s);
    if (epi == kEpiStore && b_kcontig) return launch<kRaggedM, kEpiStore, true, true>(g, s);
    if (epi == kEpiStore && !b_kcontig) return launch<kRaggedM, kEpiStore, true, false>(g, s);
    if (epi == kEpiDSwiglu && !b_kcontig) return launch<kRaggedM, kEpiDSwiglu, true, false>(g, s);
    return SPES_EINVAL;
  }
  if (epi != kEpiStore) return SPES_EINVAL;
  if (a_kcontig && b_kcontig) return launch<kGroupedK, kEpiStore, true, true>(g, s);
  if (!a_kcontig && !b_kcontig) return launch<kGroupedK, kEpiStore, false, false>(g, s);
  return SPES_EINVAL;
}

}  // namespace spes
