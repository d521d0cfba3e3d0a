// Grouped bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// Block tile 256 x 256 x 64, four wavefronts in a 2 x 2 arrangement, each owning a
// 128 x 128 sub-tile as 4 x 4 MFMA tiles (256 accumulator registers per lane).
// Operand tiles are staged global -> registers -> LDS with two LDS stages (128 KB),
// so the loads of the next K-tile are in flight while the current one is multiplied.
// Both operands live in LDS as [row][k] with a row pitch of 144 bytes (128 of data, 16
// of padding): fragment reads (16 rows x one 16-byte chunk) and the transposed staging
// writes (rows 8 apart) then spread over all 64 banks.
// An operand whose contraction index is the slow memory axis (the weights in the
// input-gradient GEMMs, both operands of the weight-gradient GEMMs) is transposed in
// registers (8x8 blocks, v_perm) on its way into LDS.
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

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kChunks = BK / 8;                 // 16-byte chunks of data per LDS row
constexpr int kPitch = kChunks + 1;             // row pitch in 16-byte units
constexpr int kTileVec = BM * kPitch;           // uint4 per operand tile
constexpr int kXcds = 8;

__device__ __forceinline__ int lds_idx(int row, int chunk) { return row * kPitch + chunk; }

// ---- staging of one operand tile --------------------------------------------------
// K-contiguous operand: thread t owns chunk (t & 7) of rows (t >> 3) + 32 i, i = 0..7.
struct RowOffs {
  long o[8];   // element offset of the row start; < 0: row outside the operand (reads as zero)
};

__device__ __forceinline__ void load_kcontig(const bf16_t* base, const RowOffs& ro, long k0, long k_end, uint4 (&r)[8]) {
  const long k = k0 + (threadIdx.x & 7) * 8;
  const bool kin = k < k_end;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    r[i] = make_uint4(0, 0, 0, 0);
    if (kin && ro.o[i] >= 0) r[i] = *reinterpret_cast<const uint4*>(base + ro.o[i] + k);
  }
}

// fused SwiGLU: rows i with ((i >> 1) & 1) set come from the second matrix (see the row map in the kernel)
__device__ __forceinline__ void load_kcontig2(const bf16_t* base0, const bf16_t* base1, const RowOffs& ro, long k0, long k_end,
                                              uint4 (&r)[8]) {
  const long k = k0 + (threadIdx.x & 7) * 8;
  const bool kin = k < k_end;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    r[i] = make_uint4(0, 0, 0, 0);
    if (kin && ro.o[i] >= 0) r[i] = *reinterpret_cast<const uint4*>((((i >> 1) & 1) ? base1 : base0) + ro.o[i] + k);
  }
}

__device__ __forceinline__ void store_kcontig(uint4* tile, const uint4 (&r)[8]) {
  const int c = threadIdx.x & 7, r0 = threadIdx.x >> 3;
#pragma unroll
  for (int i = 0; i < 8; ++i) tile[lds_idx(r0 + 32 * i, c)] = r[i];
}

// K-strided operand (element (row, k) at base + k*kstride + row): thread t owns the 8 x 8 block of
// k-block (t & 7) and row-block (t >> 3): eight 16-byte loads along the rows, one per k.
__device__ __forceinline__ void load_kstrided(const bf16_t* base, long kstride, const int* krows, long k0, long k_end, long row0,
                                              long row_end, uint4 (&r)[8]) {
  const long k = k0 + (threadIdx.x & 7) * 8;
  const long row = row0 + (threadIdx.x >> 3) * 8;
  const bool rin = row < row_end;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    r[j] = make_uint4(0, 0, 0, 0);
    if (rin && k + j < k_end) {
      const long kr = krows ? (long)krows[k + j] : k + j;
      r[j] = *reinterpret_cast<const uint4*>(base + kr * kstride + row);
    }
  }
}

// in[j] holds rows n0..n0+7 at k_j; out row i gets k_0..k_7 of row n0+i
__device__ __forceinline__ void store_kstrided(uint4* tile, const uint4 (&in)[8]) {
  const int kb = threadIdx.x & 7, nb = threadIdx.x >> 3;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint32_t w[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      // (k=2m, k=2m+1) of row i: low or high half of word i/2 of in[2m], in[2m+1]
      const uint32_t lo_src = (i >> 1) == 0 ? in[2 * m].x : (i >> 1) == 1 ? in[2 * m].y : (i >> 1) == 2 ? in[2 * m].z : in[2 * m].w;
      const uint32_t hi_src =
          (i >> 1) == 0 ? in[2 * m + 1].x : (i >> 1) == 1 ? in[2 * m + 1].y : (i >> 1) == 2 ? in[2 * m + 1].z : in[2 * m + 1].w;
      w[m] = (i & 1) ? __builtin_amdgcn_perm(hi_src, lo_src, 0x07060302u)    // high halves
                     : __builtin_amdgcn_perm(hi_src, lo_src, 0x05040100u);   // low halves
    }
    tile[lds_idx(nb * 8 + i, kb)] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ uint32_t pack2(float a, float b) { return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16); }

// -----------------------------------------------------------------------------------
template <int MODE, int EPI, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256, 1) void gemm_mfma_kernel(const GemmArgs g) {
  __shared__ uint4 smem[2 * 2 * kTileVec];   // [stage][A|B][256 rows x 9 chunks] = 144 KB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhalf = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- which tile ----
  const int gx = (EPI == kEpiSwiglu) ? cdiv(g.Ndim, BN / 2) : cdiv(g.Ndim, BN);
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
  // first output column of this tile; with the fused SwiGLU the 256 tile columns are 128 gate + 128 up columns
  const long n0 = (EPI == kEpiSwiglu) ? (long)nt * (BN / 2) : (long)nt * BN;

  // ---- per-thread row offsets of K-contiguous operands (fixed over the K loop) ----
  RowOffs arow, brow;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    arow.o[i] = -1;
    brow.o[i] = -1;
    if (A_KC) {
      const long m = m0 + (tid >> 3) + 32 * i;
      if (m < m_end) arow.o[i] = ((MODE == kRaggedM && g.a_rows) ? (long)g.a_rows[m] : m) * g.a_ms;
    }
    if (B_KC) {
      const int nl = (tid >> 3) + 32 * i;
      if (EPI == kEpiSwiglu) {
        // tile row nl: wave column nl/128, then 64 gate columns followed by the matching 64 up columns
        // (rows with bit 6 of nl set, i.e. (i >> 1) & 1, read the up projection)
        const long fcol = n0 + (nl >> 7) * 64 + (nl & 63);
        if (fcol < g.Ndim) brow.o[i] = b_group + fcol * g.b_ns;
      } else if (n0 + nl < g.Ndim) {
        brow.o[i] = b_group + (n0 + nl) * g.b_ns;
      }
    }
  }

  f32x16 acc[4][4];   // [n sub-tile][m sub-tile]
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const int npass = (EPI == kEpiSwiglu) ? 1 : g.npairs;
  const long klen = k_end - k_begin;
  const int nk = (int)((klen + BK - 1) / BK);
  const int nsteps = nk * npass;

  uint4 ra[8], rb[8];
  auto fetch = [&](int step) {
    const int pass = step / nk;
    const long k0 = k_begin + (long)(step - pass * nk) * BK;
    if (A_KC) {
      load_kcontig(reinterpret_cast<const bf16_t*>(g.A[pass]), arow, k0, k_end, ra);
    } else {
      load_kstrided(reinterpret_cast<const bf16_t*>(g.A[pass]), g.a_ks, g.a_rows, k0, k_end, m0, m_end, ra);
    }
    if (B_KC) {
      if (EPI == kEpiSwiglu)
        load_kcontig2(reinterpret_cast<const bf16_t*>(g.B[0]), reinterpret_cast<const bf16_t*>(g.B[1]), brow, k0, k_end, rb);
      else
        load_kcontig(reinterpret_cast<const bf16_t*>(g.B[pass]), brow, k0, k_end, rb);
    } else {
      load_kstrided(reinterpret_cast<const bf16_t*>(g.B[pass]) + b_group, g.b_ks, nullptr, k0, k_end, n0, g.Ndim, rb);
    }
  };
  auto stash = [&](int stage) {
    uint4* ta = smem + stage * 2 * kTileVec;
    uint4* tb = ta + kTileVec;
    if (A_KC) store_kcontig(ta, ra); else store_kstrided(ta, ra);
    if (B_KC) store_kcontig(tb, rb); else store_kstrided(tb, rb);
  };

  if (nsteps > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();
  for (int step = 0; step < nsteps; ++step) {
    const int cur = step & 1;
    if (step + 1 < nsteps) fetch(step + 1);
    const uint4* ta = smem + cur * 2 * kTileVec;
    const uint4* tb = ta + kTileVec;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[4], bfr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = __builtin_bit_cast(bf16x8, ta[lds_idx(wm * 128 + i * 32 + l32, ks * 2 + lhalf)]);
#pragma unroll
      for (int j = 0; j < 4; ++j) bfr[j] = __builtin_bit_cast(bf16x8, tb[lds_idx(wn * 128 + j * 32 + l32, ks * 2 + lhalf)]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[j][i], 0, 0, 0);
    }
    if (step + 1 < nsteps) stash(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds row m = .. + l32 and, per register group gq, columns gq*8 + lhalf*4 + 0..3 ----
  if (EPI == kEpiStore) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long m = m0 + wm * 128 + i * 32 + l32;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const long n = n0 + wn * 128 + j * 32 + gq * 8 + lhalf * 4;
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
    for (int i = 0; i < 4; ++i) {
      const long m = m0 + wm * 128 + i * 32 + l32;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const long n = n0 + wn * 64 + j * 32 + gq * 8 + lhalf * 4;
          if (n >= g.Ndim) continue;
          const long ci = m * g.c_ms + n;
          float a[4], b[4], h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[e] = acc[j][i][gq * 4 + e];
            b[e] = acc[j + 2][i][gq * 4 + e];
            h[e] = a[e] * sigmoidf_(a[e]) * b[e];
          }
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C[0]) + ci) = make_float4(a[0], a[1], a[2], a[3]);
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C[1]) + ci) = make_float4(b[0], b[1], b[2], b[3]);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.C[2]) + ci) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
        }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long m = m0 + wm * 128 + i * 32 + l32;
      const bool min_ = m < m_end;
      const float rs = min_ ? g.row_scale[m] : 0.f;
      float dot = 0.f;
      if (min_) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const long n = n0 + wn * 128 + j * 32 + gq * 8 + lhalf * 4;
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
              const float h = a[e] * sg * b[e];
              dot = fmaf(u, h, dot);
              const float dh = rs * u;
              da[e] = dh * b[e] * sg * (1.f + a[e] * (1.f - sg));
              db[e] = dh * a[e] * sg;
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

template <int MODE, int EPI, bool A_KC, bool B_KC>
int launch(const GemmArgs& g, hipStream_t s) {
  const int gx = (EPI == kEpiSwiglu) ? cdiv(g.Ndim, BN / 2) : cdiv(g.Ndim, BN);
  long total = (MODE == kRaggedM) ? (long)g.max_tiles * gx : (long)g.n_groups * cdiv(g.Mdim, BM) * gx;
  if (total <= 0) return SPES_OK;
  total = (total + kXcds - 1) / kXcds * kXcds;
  hipLaunchKernelGGL((gemm_mfma_kernel<MODE, EPI, A_KC, B_KC>), dim3((unsigned)total), dim3(256), 0, s, g);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

}  // namespace

int mfma_row_tile() { return BM; }
// number of gate-gradient partials per row that the kEpiDSwiglu epilogue writes for Ndim columns
int mfma_rowdot_parts(int ndim) { return 2 * cdiv(ndim, BN); }

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
