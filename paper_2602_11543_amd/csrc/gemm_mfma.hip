// Grouped bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate).
//
// A 256-thread block (four wavefronts, 2 x 2) computes a BM x BN output tile, each
// wavefront a (BM/2) x (BN/2) sub-tile as TM x TN MFMA tiles of 16 x 16 held in AGPRs.
// The 16x16x32 form of the instruction is used because it is the cheaper one in power, and
// power is what bounds these kernels: on the same operand values a register-resident loop of it
// sustains about 2.1 PFLOP/s at 2.1 GHz where the 32x32x16 form sustains 1.85 PFLOP/s at
// 1.83 GHz (it moves half as many accumulator registers per multiply-add).
// Operand tiles are staged global -> registers -> LDS with two LDS stages:
//   * a register is written to LDS (K-tile t+1) and at once reloaded from global
//     memory (K-tile t+2), so every load has a whole iteration to land;
//   * those writes and loads are issued one at a time between MFMAs, and the main
//     loop is a single basic block, so the matrix pipe never waits behind a burst
//     of memory instructions and the compiler's wait counts are exact;
//   * MFMA fragments are double-buffered in registers: the reads of k-step s+1 are
//     issued before the MFMAs of k-step s, and the first fragments of the next K-tile
//     are read (after the block barrier) under the last MFMAs of the current one.
// An operand whose contraction index is the fast memory axis lives in LDS as [row][k]
// without padding; the 16-byte chunks of a row are permuted by the row number (kc_unit)
// so that both the fragment reads (16 rows x one chunk) and the staging writes (2 rows x
// 8 chunks) of a group of sixteen lanes cover all banks.
// An operand whose contraction index is the slow memory axis (the weights in the
// input-gradient GEMMs, both operands of the weight-gradient GEMMs) keeps its memory
// order in LDS, [k][row] with a pitch of rows*2+64 bytes: it is loaded in 512-byte
// runs along a k-row, and the MFMA fragments (eight consecutive k of one row per lane)
// come out of LDS through the transposing read ds_read_b64_tr_b16, four k at a time.
// Operands are read through buffer resources (uniform base and byte count, a per-lane
// 32-bit offset fixed for the whole tile, a uniform offset that moves with the K-tile):
// the loop computes no addresses, and loads are unconditional - a read beyond the tensor
// returns zero, a read beyond the tile returns data that is never used (the k tail is
// zeroed by select on its way into LDS, surplus rows are never stored).
//
// The MFMA operands are swapped (weights tile as the "A" input) so that each lane ends
// up holding runs of four consecutive output columns of one row: epilogues then work
// on 8- and 16-byte vectors along the contiguous dimension.
//
// Tiles are enumerated on a 1-D grid and dealt out so that every XCD (workgroups are
// assigned to the eight XCDs round-robin) gets one contiguous range of tiles: tiles
// that share an expert's weight panel or a row panel meet in the same L2.
#include <type_traits>

#include "gemm.h"

namespace spes {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kXcds = 8;

template <int BM_, int BN_, int BK_, int MINB_>
struct Cfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, MINB = MINB_;
  static constexpr int TM = BM / 32, TN = BN / 32;          // 16 x 16 MFMA tiles per wavefront along m, n
  static constexpr int TS = BM / 64;                        // 32-row slabs of a wavefront's sub-tile (epilogues)
  static constexpr int KSTEPS = BK / 32;                    // one MFMA contracts 32 k
  static constexpr int CH = BK / 8;                         // 16-byte chunks of data per LDS row
  static constexpr int PITCH = CH;                          // row pitch in 16-byte units: no padding, the chunks of a row are
                                                            // permuted instead (kc_unit below)
  static constexpr int RP = 256 / CH;                       // rows staged per pass (K-contiguous operand)
  static constexpr int NA = BM / RP, NB = BN / RP;          // staging registers (uint4) per thread, K-contiguous
  static constexpr int KPA_ = BM / 8 + 4, KPB_ = BN / 8 + 4;
  // an operand's LDS region holds either layout: [row][k] with a padded row, or [k][row] (below) with a padded k-row
  static constexpr int A_VEC = BM * PITCH > BK * KPA_ ? BM * PITCH : BK * KPA_;
  static constexpr int B_VEC = BN * PITCH > BK * KPB_ ? BN * PITCH : BK * KPB_;
  static constexpr int STAGE_VEC = A_VEC + B_VEC;
  // K-strided operand: [k][row] in LDS; a k-row of the tile is BM/8 (BN/8) chunks and 64 bytes of padding, so that
  // the four k-rows one transposing read touches start 16 banks apart
  static constexpr int KPA = BM / 8 + 4, KPB = BN / 8 + 4;  // k-row pitch in 16-byte units
  static constexpr int KRA = 256 / (BM / 8), KRB = 256 / (BN / 8);   // k-rows staged per pass
  static constexpr int NAS = BK / KRA, NBS = BK / KRB;      // staging registers per thread, K-strided
  static constexpr int RA = NA > NAS ? NA : NAS;            // staging register counts covering both kinds
  static constexpr int RB = NB > NBS ? NB : NBS;
  static_assert(BK * KPA <= A_VEC && BK * KPB <= B_VEC, "the [k][row] layout must fit the operand's LDS region");
};

// Position (in 16-byte units) of chunk c of row `row` in the [row][k] LDS layout of a K-contiguous operand with CH
// chunks per row: the chunk index is XORed with bits 1.. of the row.  Sixteen units span all 64 banks; the unit of
// (row, c) modulo 16 is (row & 1) * 8 + (c ^ (row >> 1) & 7), so the sixteen rows one group of lanes reads at a
// common chunk (a fragment read), and the two rows times eight chunks one group of lanes writes, each cover all banks.
template <int CH>
__device__ __forceinline__ int kc_unit(int row, int c) { return row * CH + (c ^ ((row >> 1) & (CH - 1))); }

__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }
// branch-free: the main loop must stay one basic block so that the compiler counts outstanding loads exactly
__device__ __forceinline__ uint4 sel4(bool keep, const uint4& v) {
  const uint32_t m = keep ? 0xffffffffu : 0u;
  return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
}
// element-wise copy (an aggregate copy of a staging register keeps the whole register array in scratch memory)
__device__ __forceinline__ uint4 copy4(const uint4& v) { return make_uint4(v.x, v.y, v.z, v.w); }
__device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16x2(a, b); }

// raw buffer resource over `bytes` bytes from `base`; loads at byte offsets at or beyond `bytes` return zero
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
// 16 bytes at base + lane_off + uniform_off
__device__ __forceinline__ uint4 buffer_load16(rsrc_t rs, unsigned lane_off, unsigned uniform_off) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)lane_off, (int)uniform_off, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
// Transposing LDS read.  Within each group of 16 lanes, lane s supplies the address of four consecutive 16-bit
// elements (think of them as row s of a 16 x 4 matrix); lane i receives column i%4 of rows i/4, i/4+4, i/4+8, i/4+12.
// With lane s pointing at [k0 + s/4][r0 + 4*(s%4)] of a [k][row] tile, lane i gets k0..k0+3 of row r0+i.
__device__ __forceinline__ uint2 lds_read_tr(const bf16_t* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
  return __builtin_bit_cast(uint2, v);
}

constexpr int kGroupRows = 4;      // row tiles per group of the tile order (ragged-row GEMMs) ...
constexpr int kGroupMinCols = 8;   // ... used when the output has at least this many column tiles

// A_KG / B_KG: the K-strided operand A / B takes its k-rows through the index table a_rows / b_rows (the dy rows,
// or the input rows, of an expert's routed pairs)
template <int MODE, int EPI, bool A_KC, bool B_KC, bool A_KG, bool B_KG, typename C>
__global__ __launch_bounds__(256, C::MINB) void gemm_mfma_kernel(const GemmArgs g) {
  constexpr int BM = C::BM, BN = C::BN, BK = C::BK, TM = C::TM, TN = C::TN, CH = C::CH, RP = C::RP;
  __shared__ uint4 smem[2 * C::STAGE_VEC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lq = lane >> 4;          // an MFMA operand: lane holds row l16, k = lq*8 .. lq*8+7 of a 32-wide k-step
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int BNO = (EPI == kEpiSwiglu) ? BN / 2 : BN;   // output columns per tile

  // ---- which tile ----
  const int n_base = MODE == kRaggedM ? g.n_base : 0;
  const int gx = cdiv(g.Ndim - n_base, BNO);
  long total;
  if (MODE == kRaggedM) total = (long)(*g.n_tiles) * gx; else total = (long)g.n_groups * cdiv(g.Mdim, BM) * gx;
  long logical;
  if (MODE == kGroupedK && g.offset != nullptr) {
    // ragged contraction lengths: tiles are taken in block order (round-robin over the XCDs) and the groups are
    // visited longest first, so the long tiles start early and the short ones fill in behind them
    logical = blockIdx.x;
    if (logical >= total) return;
  } else {
    const long per_xcd = (total + kXcds - 1) / kXcds;
    const long slot = blockIdx.x / kXcds;
    logical = (long)(blockIdx.x % kXcds) * per_xcd + slot;
    if (slot >= per_xcd || logical >= total) return;
  }
  int nt;
  long mt_all;
  if (MODE == kRaggedM && gx >= kGroupMinCols) {
    // Row tiles are taken kGroupRows at a time and the column tiles run inside such a group, so that the 32 tiles an
    // XCD works on at once are about kGroupRows row panels times 32/kGroupRows column panels: with the plain
    // row-major order a wide output (many column tiles) has every CU of the XCD stream its own weight panel, and the
    // next row tile of the expert streams them all again.
    const long rows_all = total / gx;
    const long per_group = (long)kGroupRows * gx;
    const long grp_i = logical / per_group, within = logical - grp_i * per_group;
    const long left = rows_all - grp_i * kGroupRows;
    const int gm = (int)(left < kGroupRows ? left : kGroupRows);
    nt = (int)(within / gm);
    mt_all = grp_i * kGroupRows + within % gm;
  } else {
    nt = (int)(logical % gx);
    mt_all = logical / gx;
  }

  long m0, m_end, k_begin, k_end, b_group = 0, c_group = 0;
  bool ds_store2 = true;
  if (MODE == kRaggedM) {
    const int e = g.tile_expert[mt_all];
    ds_store2 = ((g.c2_skip >> e) & 1ull) == 0;
    m0 = g.tile_row0[mt_all];
    m_end = min((long)g.offset[e + 1], m0 + BM);
    k_begin = 0; k_end = g.Kdim;
    b_group = (long)e * g.b_gs;
  } else {
    const int my = cdiv(g.Mdim, BM);
    int grp = (int)(mt_all / my);
    m0 = (mt_all % my) * BM;
    m_end = min((long)g.Mdim, m0 + BM);
    if (g.offset != nullptr) {
      // grp counts positions in descending order of length; find the group that holds this position
      // (lane j < n_groups owns group j; ties go to the lower group, so the order is a permutation)
      const int mine = lane < g.n_groups ? g.offset[g.group_expert[lane] + 1] - g.offset[g.group_expert[lane]] : -1;
      int rank = 0;
      for (int j = 0; j < g.n_groups; ++j) {
        const int other = __shfl(mine, j, kWave);
        rank += (other > mine || (other == mine && j < lane)) ? 1 : 0;
      }
      const unsigned long long hit = __ballot(lane < g.n_groups && rank == grp);
      grp = __ffsll((long long)hit) - 1;
      const int e = g.group_expert[grp];
      k_begin = g.offset[e]; k_end = g.offset[e + 1];
    } else {
      k_begin = (long)grp * g.kchunk; k_end = min((long)g.Kdim, k_begin + g.kchunk);
    }
    c_group = (long)grp * g.c_gs;
  }
  const long n0 = n_base + (long)nt * BNO;

  // ---- operands are read through buffer resources: a base (uniform) with a byte count, a 32-bit byte offset per
  // lane that is fixed for the whole tile, and a uniform offset that moves with the K-tile.  Nothing in the loop
  // computes an address, and no clamp is needed for memory safety: a read inside the tensor but outside the tile
  // returns data that is never used (masked k tail, rows that are not stored), a read beyond the tensor returns zero.
  const unsigned a_bytes = (unsigned)(g.a_elems * 2), b_bytes = (unsigned)((g.b_elems - b_group) * 2);
  const rsrc_t a_rsrc[2] = {make_rsrc(g.A[0], a_bytes), make_rsrc(g.A[1] ? g.A[1] : g.A[0], a_bytes)};
  const rsrc_t b_rsrc[2] = {make_rsrc(reinterpret_cast<const bf16_t*>(g.B[0]) + b_group, b_bytes),
                            make_rsrc(reinterpret_cast<const bf16_t*>(g.B[1] ? g.B[1] : g.B[0]) + b_group, b_bytes)};
  // K-contiguous operands: byte offset of this thread's chunk in K-tile 0, per staging register
  unsigned aoff[A_KC ? C::NA : 1];
  unsigned boff[B_KC ? C::NB : 1];
  if (A_KC) {
#pragma unroll
    for (int i = 0; i < C::NA; ++i) {
      long m = m0 + tid / CH + RP * i;
      if (MODE == kRaggedM && g.a_rows) m = g.a_rows[m < m_end ? m : m_end - 1];       // the index table is only that long
      aoff[i] = (unsigned)((m * g.a_ms + (tid % CH) * 8) * 2);
    }
  }
  // fused SwiGLU: staging register i holds rows of the gate matrix (B[0]) or of the up matrix (B[1]); tile row nl ->
  // wave column, then (BN/4) gate columns followed by the matching (BN/4) up columns
  constexpr int SW_W = BN / 2, SW_H = BN / 4;
  static_assert(EPI != kEpiSwiglu || (SW_H % RP == 0), "a staging register must not straddle the gate / up boundary");
  if (B_KC) {
#pragma unroll
    for (int i = 0; i < C::NB; ++i) {
      const int nl = tid / CH + RP * i;
      const long col = (EPI == kEpiSwiglu) ? n0 + (nl / SW_W) * SW_H + (nl % SW_H) : n0 + nl;
      boff[i] = (unsigned)((col * g.b_ns + (tid % CH) * 8) * 2);
    }
  }

  // acc[j][i][r] = C(m = i*16 + l16, n = j*16 + lq*4 + r) of the wavefront's sub-tile
  f32x4 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[j][i][r] = 0.f;

  const int npass = (EPI == kEpiSwiglu) ? 1 : g.npairs;
  const long klen = k_end - k_begin;
  const int nk = (int)((klen + BK - 1) / BK);
  const int nsteps = nk * npass;

  // ---- staging registers and the pieces of the global -> register -> LDS pipeline ----
  // The loads and LDS writes of one K-tile are cut into pieces that the main loop issues one at a time between
  // MFMAs: a wavefront that issues sixteen 1 KB loads (or writes) back to back sits behind the memory queues for
  // well over a thousand cycles with its matrix pipe idle, while one piece every few MFMAs is absorbed for free.
  // Piece i = write staging register i to LDS (tile t+1), then reload it (tile t+2).
  uint4 ra[C::RA], rb[C::RB];
  unsigned a_keep = 0, b_keep = 0;       // k inside the contraction range, for the tile held in ra / rb (K-strided: bit i for register i)
  unsigned a_keep_n = 0, b_keep_n = 0;   // the same for the tile being loaded
  constexpr int NPA = A_KC ? C::NA : C::NAS;
  constexpr int NPB = B_KC ? C::NB : C::NBS;
  constexpr int NP = NPA + NPB;

  // scalar coordinates of the K-tile being loaded
  int l_step = 0, l_kq = 0, l_pass = 0;           // tile number, k of the tile relative to the group, pass
  const int klen32 = (int)(k_end - k_begin);
  // K-strided operands: byte offset of this thread's chunk in k-row 0 of K-tile 0
  const unsigned a_ks_off = (unsigned)(((long)(tid / (BM / 8)) * g.a_ks + m0 + (tid % (BM / 8)) * 8) * 2);
  const unsigned b_ks_off = (unsigned)(((long)(tid / (BN / 8)) * g.b_ks + n0 + (tid % (BN / 8)) * 8) * 2);
  // gathered k-rows of the tile about to be loaded; fetched one tile ahead so that no load waits on an index
  constexpr int ACH = BM / 8, BCH = BN / 8;     // 16-byte chunks per k-row of a K-strided tile
  int kidx[A_KG ? C::NAS : 1];
  int kidx_b[B_KG ? C::NBS : 1];
  auto load_kidx = [&](int step) {
    if (A_KG) {
      const int st = step < nsteps ? step : nsteps - 1;
      const long k = k_begin + (long)(st % nk) * BK + tid / ACH;
#pragma unroll
      for (int j = 0; j < C::NAS; ++j) kidx[j] = g.a_rows[k + j * C::KRA < k_end ? k + j * C::KRA : k_end - 1];
    }
  };
  auto load_kidx_b = [&](int step) {
    if (B_KG) {
      const int st = step < nsteps ? step : nsteps - 1;
      const long k = k_begin + (long)(st % nk) * BK + tid / BCH;
#pragma unroll
      for (int j = 0; j < C::NBS; ++j) kidx_b[j] = g.b_rows[k + j * C::KRB < k_end ? k + j * C::KRB : k_end - 1];
    }
  };
  // registers 0..n-1 of a K-strided operand hold k-rows inside the contraction range
  // (first_kq = k of the thread's first register relative to the group; rows_per_pass is a power of two)
  auto keep_bits = [&](int first_kq, int rows_per_pass, int nreg) -> unsigned {
    const int left = klen32 - first_kq;
    int n = (left + rows_per_pass - 1) >> __builtin_ctz(rows_per_pass);      // arithmetic shift: negative stays negative
    n = max(0, min(n, nreg));
    return (1u << n) - 1u;
  };
  auto set_load_tile = [&](int step) {
    l_pass = step / nk;
    l_step = step;
    l_kq = (step - l_pass * nk) * BK;
    if (A_KC) {
      a_keep_n = (l_kq + (tid % CH) * 8 < klen32) ? 0xffu : 0u;
    } else {
      a_keep_n = keep_bits(l_kq + tid / ACH, C::KRA, C::NAS);
    }
    if (B_KC) {
      b_keep_n = (l_kq + (tid % CH) * 8 < klen32) ? 0xffu : 0u;
    } else {
      b_keep_n = keep_bits(l_kq + tid / BCH, C::KRB, C::NBS);
    }
  };

  auto load_a = [&](int idx) {   // idx: staging register
    const rsrc_t rs = l_pass ? a_rsrc[1] : a_rsrc[0];
    if (A_KC) {
      ra[idx] = buffer_load16(rs, aoff[idx], (unsigned)((k_begin + l_kq) * 2));
    } else if (A_KG) {
      ra[idx] = buffer_load16(rs, (unsigned)kidx[idx] * (unsigned)(g.a_ks * 2) + (unsigned)((m0 + (tid % ACH) * 8) * 2), 0u);
      if (idx == C::NAS - 1) load_kidx(l_step + 1);
    } else {
      ra[idx] = buffer_load16(rs, a_ks_off, (unsigned)((k_begin + l_kq + idx * C::KRA) * g.a_ks * 2));
    }
  };
  auto load_b = [&](int idx) {
    if (B_KC) {
      // (the register -> matrix assignment of the fused SwiGLU is the same for every thread)
      const bool second = (EPI == kEpiSwiglu) ? (((RP * idx) % SW_W) / SW_H) != 0 : l_pass != 0;
      rb[idx] = buffer_load16(second ? b_rsrc[1] : b_rsrc[0], boff[idx], (unsigned)((k_begin + l_kq) * 2));
    } else if (B_KG) {
      rb[idx] = buffer_load16(l_pass ? b_rsrc[1] : b_rsrc[0],
                              (unsigned)kidx_b[idx] * (unsigned)(g.b_ks * 2) + (unsigned)((n0 + (tid % BCH) * 8) * 2), 0u);
      if (idx == C::NBS - 1) load_kidx_b(l_step + 1);
    } else {
      rb[idx] = buffer_load16(l_pass ? b_rsrc[1] : b_rsrc[0], b_ks_off, (unsigned)((k_begin + l_kq + idx * C::KRB) * g.b_ks * 2));
    }
  };
  // `masked`: the tile may reach beyond the contraction range and its k tail is zeroed on the way into LDS.  Only the
  // last K-tile of a pass can need that; every other tile goes to LDS as it came (the four selects per register are
  // most of the vector-ALU work of an iteration, and the matrix pipe waits while they issue).
  auto write_a = [&](int stage, int idx, bool masked) {
    uint4* ta = smem + stage * C::STAGE_VEC;
    if (A_KC) {
      ta[kc_unit<CH>(tid / CH + RP * idx, tid % CH)] = masked ? sel4(a_keep != 0, ra[idx]) : copy4(ra[idx]);
    } else {
      ta[(tid / ACH + idx * C::KRA) * C::KPA + tid % ACH] = masked ? sel4((a_keep >> idx) & 1u, ra[idx]) : copy4(ra[idx]);
    }
  };
  auto write_b = [&](int stage, int idx, bool masked) {
    uint4* tb = smem + stage * C::STAGE_VEC + C::A_VEC;
    if (B_KC) {
      tb[kc_unit<CH>(tid / CH + RP * idx, tid % CH)] = masked ? sel4(b_keep != 0, rb[idx]) : copy4(rb[idx]);
    } else {
      tb[(tid / BCH + idx * C::KRB) * C::KPB + tid % BCH] = masked ? sel4((b_keep >> idx) & 1u, rb[idx]) : copy4(rb[idx]);
    }
  };
  // piece p of the pipeline step "tile t+1 to LDS stage `stage`, tile t+2 into registers"
  auto piece = [&](int p, int stage, bool do_write, bool do_load, bool masked) {
    if (p < NPA) {
      if (do_write) write_a(stage, p, masked);
      if (do_load) load_a(p);
    } else {
      if (do_write) write_b(stage, p - NPA, masked);
      if (do_load) load_b(p - NPA);
    }
  };

  bf16x8 fa[2][TM], fb[2][TN];
  const int tr_k = lq * 8 + (lane & 15) / 4;                     // k-row (within a k-step) this lane points the transposing read at
  const int tr_r = (lane & 3) * 4;                               // row (within a 16-row MFMA tile) likewise
  auto read_frag_a = [&](int stage, int ks, int set, int i) {
    const uint4* ta = smem + stage * C::STAGE_VEC;
    if (A_KC) {
      fa[set][i] = __builtin_bit_cast(bf16x8, ta[kc_unit<CH>(wm * (BM / 2) + i * 16 + l16, ks * 4 + lq)]);
    } else {
      const bf16_t* p = reinterpret_cast<const bf16_t*>(ta + (ks * 32 + tr_k) * C::KPA) + wm * (BM / 2) + i * 16 + tr_r;
      const uint2 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * C::KPA * 8);
      fa[set][i] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
  };
  auto read_frag_b = [&](int stage, int ks, int set, int j) {
    const uint4* tb = smem + stage * C::STAGE_VEC + C::A_VEC;
    if (B_KC) {
      fb[set][j] = __builtin_bit_cast(bf16x8, tb[kc_unit<CH>(wn * (BN / 2) + j * 16 + l16, ks * 4 + lq)]);
    } else {
      const bf16_t* p = reinterpret_cast<const bf16_t*>(tb + (ks * 32 + tr_k) * C::KPB) + wn * (BN / 2) + j * 16 + tr_r;
      const uint2 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * C::KPB * 8);
      fb[set][j] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
  };
  // fragment w of a k-step in the order the MFMAs first need them: B0, A0 .. A(TM-1), B1 .. B(TN-1)
  auto read_frag = [&](int stage, int ks, int set, int w) {
    if (w == 0) read_frag_b(stage, ks, set, 0);
    else if (w <= TM) read_frag_a(stage, ks, set, w - 1);
    else read_frag_b(stage, ks, set, w - TM);
  };
  auto read_frags = [&](int stage, int ks, int set) {
#pragma unroll
    for (int w = 0; w < TM + TN; ++w) read_frag(stage, ks, set, w);
  };

  if (nsteps > 0) {
    // prologue: tile 0 -> registers -> LDS stage 0, tile 1 -> registers
    load_kidx(0);
    load_kidx_b(0);
    set_load_tile(0);
#pragma unroll
    for (int p = 0; p < NP; ++p) piece(p, 0, false, true, true);
    a_keep = a_keep_n; b_keep = b_keep_n;
    set_load_tile(nsteps > 1 ? 1 : 0);
#pragma unroll
    for (int p = 0; p < NP; ++p) piece(p, 0, true, true, true);
    a_keep = a_keep_n; b_keep = b_keep_n;
    __syncthreads();
    read_frags(0, 0, 0);

    constexpr int MF = TM * TN;                       // MFMAs per k-step
    constexpr int NF = TM + TN;                       // fragments per k-step
    static_assert(C::KSTEPS == 2 && NP == NF, "the schedule below deals one staging register per fragment over a K-tile of two k-steps");
    constexpr int FR = MF / NF;                       // MFMA gaps per fragment in the first k-step
    constexpr int R1 = FR > 1 ? 1 : 0, R2 = FR > 2 ? 2 : FR - 1;
    constexpr int QB = MF - 2 * NF >= 0 ? MF / 4 : 0; // the barrier sits before this MFMA of the second k-step ...
    constexpr int RT = (MF - QB) / NF;                // ... and the next K-tile's fragments follow it, one every RT gaps
    static_assert(FR >= 1 && RT >= 1, "more fragments than MFMA gaps");
    // One iteration: MFMAs of K-tile t from LDS stage t&1, K-tile t+1 from registers to the other stage, K-tile t+2
    // from memory to registers.  No branches in here: past the last K-tile the pipeline keeps running on clamped
    // tiles whose results are never used (a spare LDS write, a repeated load).
    // Everything besides the MFMAs is dealt out over the gaps between them, at most one memory instruction per gap
    // where the tile is large enough.  First k-step, gaps w*FR .. w*FR+2: fragment w of the second k-step, the LDS
    // write of staging register w (K-tile t+1), its reload (K-tile t+2).  Second k-step: the block barrier that
    // publishes K-tile t+1, then the fragments of its first k-step.
    auto iteration = [&](int t, auto masked_c) __attribute__((always_inline)) {
      constexpr bool MASKED = decltype(masked_c)::value;
      const int cur = t & 1;
      set_load_tile(t + 2 < nsteps ? t + 2 : nsteps - 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < MF; ++q) {
        const int j = q / TM, i = q % TM;
        acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[0][j], fa[0][i], acc[j][i], 0, 0, 0);
        const int w = q / FR, r = q % FR;
        if (w < NF) {
          if (r == 0) read_frag(cur, 1, 1, w);
          if (r == R1) piece(w, cur ^ 1, true, false, MASKED);
          if (r == R2) piece(w, cur ^ 1, false, true, MASKED);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int q = 0; q < MF; ++q) {
        const int j = q / TM, i = q % TM;
        if (q == QB) {
          a_keep = a_keep_n; b_keep = b_keep_n;
          __syncthreads();
          __builtin_amdgcn_sched_barrier(0);
        }
        acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[1][j], fa[1][i], acc[j][i], 0, 0, 0);
        if (q >= QB && (q - QB) % RT == 0 && (q - QB) / RT < NF) read_frag(cur ^ 1, 0, 0, (q - QB) / RT);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // The body exists twice: an inner loop without the k-tail selects for the tiles in the middle of a pass, and one
    // straight-line copy with them for the iteration that writes the last tile of a pass (and for the final iteration,
    // whose write is the spare one).  w = t + 1 is the tile written in iteration t.
    int w = 1, pass_end = nk - 1;
    while (true) {
      const int stop = pass_end < nsteps ? pass_end : nsteps;
      for (; w < stop; ++w) iteration(w - 1, std::false_type{});
      iteration(w - 1, std::true_type{});
      ++w;
      pass_end += nk;
      if (w > nsteps) break;
    }
  }

  // ---- epilogue ----
  // The MFMA leaves each lane with 4-column runs of one row per register group, which would scatter 32-byte
  // pieces over 32 rows per store.  Each wavefront therefore turns its sub-tile through a private LDS region,
  // 32 rows at a time, and comes back with lanes laid along the columns: every global access below is a run of
  // 256 to 512 contiguous bytes per row.
  constexpr int ECOLS = TN * 16, EPITCH = ECOLS + 4; // floats per LDS row
  constexpr int TS = C::TS;                          // 32-row slabs: slab i holds the MFMA row tiles 2i and 2i+1
  float* ep = reinterpret_cast<float*>(smem) + wave * (32 * EPITCH);
  // output addresses are a per-tile base (uniform) plus a 32-bit element offset: row within the tile times the row
  // stride plus the column; rows are compared with the tile's valid row count in 32 bits as well
  const int e_rows = (int)(m_end - m0);
  const long e_tile = c_group + m0 * g.c_ms;
  const int e_r0 = wm * (BM / 2);
  // dSwiGLU epilogue: lanes lie along the columns (DS_CPR lanes per row, eight columns each, so that the bf16
  // results leave in 16-byte stores); the saved fp32 projections come in batches of half a 32-row slab
  constexpr int DS_CPR = ECOLS / 8, DS_RPI = 64 / DS_CPR, DS_NB = 2, DS_HALF = 32 / DS_RPI / DS_NB;
  const int ds_c8 = lane % DS_CPR;
  const long ds_n = n0 + wn * (BN / 2) + ds_c8 * 8;
  // addresses are a per-tile base (uniform) plus a 32-bit offset: one register per address instead of two
  const long ds_tile = m0 * g.c_ms;
  const int ds_rows = (int)(m_end - m0);                        // valid rows of the tile
  const int ds_r0 = wm * (BM / 2) + lane / DS_CPR;
  const bool ds_nin = ds_n < g.Ndim;
  const unsigned ds_ncl = ds_nin ? (unsigned)ds_n : 0u;
  const bf16_t* ds_a = reinterpret_cast<const bf16_t*>(g.E[0]) + ds_tile;
  const bf16_t* ds_b = reinterpret_cast<const bf16_t*>(g.E[1]) + ds_tile;
  const bf16_t* ds_d = reinterpret_cast<const bf16_t*>(g.E[2]) + ds_tile;
  bf16_t* ds_c0 = reinterpret_cast<bf16_t*>(g.C[0]) + ds_tile;
  bf16_t* ds_c1 = reinterpret_cast<bf16_t*>(g.C[1]) + ds_tile;
  bf16_t* ds_c2 = reinterpret_cast<bf16_t*>(g.C[2]) + ds_tile;
  uint4 av[EPI == kEpiDSwiglu ? DS_HALF : 1], bv[EPI == kEpiDSwiglu ? DS_HALF : 1], dv[EPI == kEpiDSwiglu ? DS_HALF : 1];
  auto load_ab = [&](int i, int hf) {
    if (EPI == kEpiDSwiglu) {
#pragma unroll
      for (int q = 0; q < DS_HALF; ++q) {
        const int rt = ds_r0 + i * 32 + (hf * DS_HALF + q) * DS_RPI;     // row within the tile
        const unsigned ci = (unsigned)(rt < ds_rows ? rt : ds_rows - 1) * (unsigned)g.c_ms + ds_ncl;
        av[q] = *reinterpret_cast<const uint4*>(ds_a + ci);
        bv[q] = *reinterpret_cast<const uint4*>(ds_b + ci);
        dv[q] = *reinterpret_cast<const uint4*>(ds_d + ci);
      }
    }
  };
  load_ab(0, 0);
  __syncthreads();                                   // the staging tiles are dead from here on
#pragma unroll
  for (int i = 0; i < TS; ++i) {
    if (EPI == kEpiStore && !g.c_f32) {
      // bf16 output: round first, so that half as many bytes make the trip through LDS; rows of ECOLS bf16 with a
      // pitch of ECOLS*2+8 bytes (the 32 rows one write instruction touches fall into different banks)
      constexpr int BPITCH = ECOLS * 2 + 8;
      char* eb = reinterpret_cast<char*>(ep);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
          *reinterpret_cast<uint2*>(eb + (ii * 16 + l16) * BPITCH + (j * 16 + lq * 4) * 2) =
              make_uint2(pack2(acc[j][2 * i + ii][0], acc[j][2 * i + ii][1]), pack2(acc[j][2 * i + ii][2], acc[j][2 * i + ii][3]));
      constexpr int CPR = ECOLS / 8, RPI = 64 / CPR;   // lanes per row (eight columns each), rows per access
      const int c8 = lane % CPR;
      const long n = n0 + wn * (BN / 2) + c8 * 8;
      const bool n_in = n < g.Ndim;
      bf16_t* ct = reinterpret_cast<bf16_t*>(g.C[0]) + e_tile;
#pragma unroll
      for (int st = 0; st < 32 / RPI; ++st) {
        const int row = st * RPI + lane / CPR;
        const uint2 lo = *reinterpret_cast<const uint2*>(eb + row * BPITCH + c8 * 16);
        const uint2 hi = *reinterpret_cast<const uint2*>(eb + row * BPITCH + c8 * 16 + 8);
        const int rt = e_r0 + i * 32 + row;
        if (rt < e_rows && n_in)
          *reinterpret_cast<uint4*>(ct + ((unsigned)rt * (unsigned)g.c_ms + (unsigned)n)) = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
      continue;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        // The lane holds the 4-column group j*4 + lq of row ii*16 + l16.  The dSwiGLU epilogue reads two adjacent
        // groups per lane: even groups are kept in the first half of the LDS row and odd groups in the second, so that
        // each of its reads is contiguous across the lanes (the SwiGLU epilogue does the same inside the gate half
        // and inside the up half of its row: tiles j < TN/2 are the gate columns, the others the up columns)
        const int col = (EPI == kEpiDSwiglu) ? (lq & 1) * (ECOLS / 2) + (j * 2 + (lq >> 1)) * 4
                      : (EPI == kEpiSwiglu)  ? (j / (TN / 2)) * (ECOLS / 2) + (lq & 1) * (ECOLS / 4) + ((j % (TN / 2)) * 2 + (lq >> 1)) * 4
                                             : j * 16 + lq * 4;
        *reinterpret_cast<float4*>(ep + (ii * 16 + l16) * EPITCH + col) =
            make_float4(acc[j][2 * i + ii][0], acc[j][2 * i + ii][1], acc[j][2 * i + ii][2], acc[j][2 * i + ii][3]);
      }
    if (EPI == kEpiStore) {
      constexpr int CPR = ECOLS / 4, RPI = 64 / CPR;   // lanes per row, rows per access
      const int c4 = lane % CPR;
      const long n = n0 + wn * (BN / 2) + c4 * 4;
      const bool n_in = n < g.Ndim;
      float* ct = reinterpret_cast<float*>(g.C[0]) + e_tile;
#pragma unroll
      for (int st = 0; st < 32 / RPI; ++st) {
        const int row = st * RPI + lane / CPR;
        const float4 v = *reinterpret_cast<const float4*>(ep + row * EPITCH + c4 * 4);
        const int rt = e_r0 + i * 32 + row;
        if (rt < e_rows && n_in) {
          float4* c = reinterpret_cast<float4*>(ct + ((unsigned)rt * (unsigned)g.c_ms + (unsigned)n));
          float4 o = v;
          if (g.accumulate) { const float4 old = *c; o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w; }
          *c = o;
        }
      }
    } else if (EPI == kEpiSwiglu) {
      // LDS columns [0, ECOLS/2) hold the gate projection, [ECOLS/2, ECOLS) the up projection of the same output columns,
      // each with its even 4-column groups first and its odd ones behind.  A lane takes eight output columns of a row
      // (16-byte bf16 stores); the two rows that one 16-lane phase of a read touches are eight rows apart, which is 32
      // banks with this pitch.
      static_assert(EPI != kEpiSwiglu || (TN == 8 && ECOLS == 128), "lane layout of the SwiGLU epilogue");
      const int c8 = lane & 7, rsel = lane >> 3;
      const long n = n0 + wn * (BN / 4) + c8 * 8;
      const bool n_in = n < g.Ndim;
      bf16_t* cat = reinterpret_cast<bf16_t*>(g.C[0]) + e_tile;
      bf16_t* cbt = reinterpret_cast<bf16_t*>(g.C[1]) + e_tile;
      bf16_t* cht = reinterpret_cast<bf16_t*>(g.C[2]) + e_tile;
      bf16_t* cdt = reinterpret_cast<bf16_t*>(g.C[3]) + e_tile;
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const int row = (st >> 1) * 16 + (st & 1) * 4 + (rsel >> 1) + 8 * (rsel & 1);
        const float* rp = ep + row * EPITCH + c8 * 4;
        const float4 a0 = *reinterpret_cast<const float4*>(rp), a1 = *reinterpret_cast<const float4*>(rp + ECOLS / 4);
        const float4 b0 = *reinterpret_cast<const float4*>(rp + ECOLS / 2), b1 = *reinterpret_cast<const float4*>(rp + 3 * ECOLS / 4);
        const int rt = e_r0 + i * 32 + row;
        if (rt < e_rows && n_in) {
          const unsigned ci = (unsigned)rt * (unsigned)g.c_ms + (unsigned)n;
          const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w}, b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
          // The backward needs a and b only to bf16 accuracy, but h = SiLU(a) b nearly to fp32 accuracy (its gate
          // gradient is a difference of nearly equal sums when experts are near copies).  Saved are therefore a and b
          // rounded to bf16 and the bf16 value of what the rounded pair misses, h - SiLU(bf16 a) (bf16 b): h comes back
          // to about 2^-17 from six bytes per element instead of eight.  The miss is taken to first order in the two
          // rounding steps (the second-order term is below 2^-18 of h), which needs no second sigmoid.
          uint32_t ap[4], bp[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) { ap[e] = pack2(a[2 * e], a[2 * e + 1]); bp[e] = pack2(b[2 * e], b[2 * e + 1]); }
          float h[8], dl[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sg = sigmoidf_(a[e]);
            const float sl = a[e] * sg;                               // SiLU(a)
            h[e] = sl * b[e];
            const float ar = __uint_as_float((e & 1) ? (ap[e >> 1] & 0xffff0000u) : (ap[e >> 1] << 16));
            const float br = __uint_as_float((e & 1) ? (bp[e >> 1] & 0xffff0000u) : (bp[e >> 1] << 16));
            const float dsl = sg + sl * (1.f - sg);                   // SiLU'(a)
            dl[e] = dsl * (a[e] - ar) * br + sl * (b[e] - br);
          }
          // the saved values are next read by the backward pass: streaming stores (h, which the next GEMM reads, stays plain)
          store_stream(reinterpret_cast<uint4*>(cat + ci), make_uint4(ap[0], ap[1], ap[2], ap[3]));
          store_stream(reinterpret_cast<uint4*>(cbt + ci), make_uint4(bp[0], bp[1], bp[2], bp[3]));
          store_stream(reinterpret_cast<uint4*>(cdt + ci),
                       make_uint4(pack2(dl[0], dl[1]), pack2(dl[2], dl[3]), pack2(dl[4], dl[5]), pack2(dl[6], dl[7])));
          *reinterpret_cast<uint4*>(cht + ci) = make_uint4(pack2(h[0], h[1]), pack2(h[2], h[3]), pack2(h[4], h[5]), pack2(h[6], h[7]));
        }
      }
    } else {
#pragma unroll
      for (int hf = 0; hf < DS_NB; ++hf) {
        uint4 oa[DS_HALF], ob[DS_HALF], oh[DS_HALF];
        float dots[DS_HALF];
#pragma unroll
        for (int q = 0; q < DS_HALF; ++q) {
          const int row = (hf * DS_HALF + q) * DS_RPI + lane / DS_CPR;
          const float4 u0 = *reinterpret_cast<const float4*>(ep + row * EPITCH + ds_c8 * 4);
          const float4 u1 = *reinterpret_cast<const float4*>(ep + row * EPITCH + ECOLS / 2 + ds_c8 * 4);
          const int rt = ds_r0 + i * 32 + (hf * DS_HALF + q) * DS_RPI;
          const float rs = g.row_scale[m0 + (rt < ds_rows ? rt : ds_rows - 1)];
          const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
          const uint32_t aw[4] = {av[q].x, av[q].y, av[q].z, av[q].w}, bw[4] = {bv[q].x, bv[q].y, bv[q].z, bv[q].w},
                         dw[4] = {dv[q].x, dv[q].y, dv[q].z, dv[q].w};
          float a[8], b[8], hc[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[2 * e] = __uint_as_float(aw[e] << 16); a[2 * e + 1] = __uint_as_float(aw[e] & 0xffff0000u);
            b[2 * e] = __uint_as_float(bw[e] << 16); b[2 * e + 1] = __uint_as_float(bw[e] & 0xffff0000u);
            hc[2 * e] = __uint_as_float(dw[e] << 16); hc[2 * e + 1] = __uint_as_float(dw[e] & 0xffff0000u);
          }
          float da[8], db[8], hg[8], dot = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sg = sigmoidf_(a[e]);
            const float as = a[e] * sg;          // SiLU of the saved (bf16) gate projection
            const float h = as * b[e] + hc[e];   // the forward's h: what the rounded pair gives plus the saved correction
            dot = fmaf(u[e], h, dot);
            const float dh = rs * u[e];
            da[e] = dh * b[e] * (sg + as * (1.f - sg));
            db[e] = dh * as;
            hg[e] = rs * h;
          }
          oa[q] = make_uint4(pack2(da[0], da[1]), pack2(da[2], da[3]), pack2(da[4], da[5]), pack2(da[6], da[7]));
          ob[q] = make_uint4(pack2(db[0], db[1]), pack2(db[2], db[3]), pack2(db[4], db[5]), pack2(db[6], db[7]));
          oh[q] = make_uint4(pack2(hg[0], hg[1]), pack2(hg[2], hg[3]), pack2(hg[4], hg[5]), pack2(hg[6], hg[7]));
          if (!(rt < ds_rows && ds_nin)) dot = 0.f;
          // gate-gradient partial of this row over the wavefront's columns: the CPR lanes of a row sit side by side
#pragma unroll
          for (int o = DS_CPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, kWave);
          dots[q] = dot;
        }
        // The saved projections of the next half-slab are requested before this one's results are stored: one
        // in-order counter covers loads and stores, so a load issued after a store would wait for that store to
        // be acknowledged, and every half-slab would pay a full load and a full store round trip in sequence.
        __builtin_amdgcn_sched_barrier(0);
        if (hf + 1 < DS_NB) load_ab(i, hf + 1);
        else if (i + 1 < TS) load_ab(i + 1, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < DS_HALF; ++q) {
          const int rt = ds_r0 + i * 32 + (hf * DS_HALF + q) * DS_RPI;
          if (rt < ds_rows && ds_nin) {
            const unsigned ci = (unsigned)rt * (unsigned)g.c_ms + ds_ncl;
            *reinterpret_cast<uint4*>(ds_c0 + ci) = oa[q];
            *reinterpret_cast<uint4*>(ds_c1 + ci) = ob[q];
            if (ds_store2) *reinterpret_cast<uint4*>(ds_c2 + ci) = oh[q];
          }
          if (ds_c8 == 0 && rt < ds_rows) g.rowdot[(long)(g.rowdot_slot0 + nt * 2 + wn) * g.rowdot_stride + m0 + rt] = dots[q];
        }
      }
    }
  }
}

// one tile configuration: 256 x 256 x 64, one block per CU (144 KB of LDS, 256 accumulators per lane in AGPRs)
typedef Cfg<256, 256, 64, 1> Tile;

// narrow outputs (the router's M <= 64 expert columns: half the matrix work on padding), the half-full last column
// tile of a ragged-row GEMM, and launches of few tiles
typedef Cfg<256, 128, 64, 1> TileNarrow;
// few output rows (the router's weight gradient has M <= 64 of them)
typedef Cfg<128, 256, 64, 1> TileShort;
// a contraction of a single K-tile (the router's input gradient contracts over the M <= 64 experts) is all prologue
// and epilogue: small tiles, two blocks per CU, so that one block's memory phases overlap the other's
typedef Cfg<128, 128, 64, 2> TileSmall;

template <int MODE, int EPI, bool A_KC, bool B_KC, bool A_KG = false, bool B_KG = false, typename C = Tile>
int launch(const GemmArgs& g, hipStream_t s) {
  static_assert(!A_KG || !A_KC, "k-row gather: K-strided A only");
  static_assert(!B_KG || (!B_KC && MODE == kGroupedK), "k-row gather of B: K-strided B of a grouped contraction only");
  static_assert(!(A_KG && B_KG), "one gathered operand per launch");
  if (B_KG && g.npairs != 1) return SPES_EINVAL;
  // operands are addressed with 32-bit byte offsets from their base
  if (g.a_elems <= 0 || g.b_elems <= 0) return SPES_EINVAL;
  if (g.a_elems >= (1L << 31) || g.b_elems >= (1L << 31)) return SPES_ESHAPE;
  const int bno = (EPI == kEpiSwiglu) ? C::BN / 2 : C::BN;
  const int gx = cdiv(g.Ndim - (MODE == kRaggedM ? g.n_base : 0), bno);
  long total = (MODE == kRaggedM) ? (long)g.max_tiles * gx : (long)g.n_groups * cdiv(g.Mdim, C::BM) * gx;
  if (total <= 0) return SPES_OK;
  total = (total + kXcds - 1) / kXcds * kXcds;
  hipLaunchKernelGGL((gemm_mfma_kernel<MODE, EPI, A_KC, B_KC, A_KG, B_KG, C>), dim3((unsigned)total), dim3(256), 0, s, g);
  return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP;
}

}  // namespace

// Few tiles: a launch costs its number of rounds of 256 concurrent tiles, the last of them partly empty.  Half-width
// tiles cost 0.6 of a full one each and fill the rounds better; they are taken where that arithmetic says so (a layer
// of a few thousand tokens), never for a launch of many rounds.  est_tiles: expected number of row tiles (0: unknown).
static bool few_tiles_narrow(int ndim, int est_tiles) {
  if (est_tiles <= 0 || ndim % Tile::BN != 0) return false;
  const long full = (long)est_tiles * (ndim / Tile::BN);
  const long rounds_full = (full + 255) / 256, rounds_half = (2 * full + 255) / 256;
  return rounds_full <= 4 && 0.6 * rounds_half < 0.95 * rounds_full;
}

int mfma_row_tile() { return Tile::BM; }
// number of gate-gradient partials per row that the kEpiDSwiglu epilogue writes for ndim columns (two per column tile)
int mfma_rowdot_parts(int ndim, int est_tiles) {
  return few_tiles_narrow(ndim, est_tiles) ? 2 * (ndim / TileNarrow::BN) : 2 * cdiv(ndim, Tile::BN);
}

// bf16 operands only.  a_kcontig / b_kcontig: the contraction index is the fast memory axis of that operand.
int launch_gemm_mfma(int mode, int epi, bool a_kcontig, bool b_kcontig, const GemmArgs& g, hipStream_t s) {
  if (mode == kRaggedM) {
    if (!a_kcontig || g.b_rows) return SPES_EINVAL;
    // A last column tile that is at most half full goes to a launch of its own on the half-width tile (which costs
    // 0.6 of a full one) instead of running a full-width tile on half-empty operands.
    const int tail = g.Ndim % Tile::BN;
    if (epi != kEpiSwiglu && g.n_base == 0 && g.Ndim > Tile::BN && tail > 0 && tail <= TileNarrow::BN) {
      GemmArgs head = g, rest = g;
      head.Ndim = g.Ndim - tail;
      head.est_tiles = 0;            // both parts keep the slot numbering of full-width tiles
      rest.n_base = g.Ndim - tail;
      rest.rowdot_slot0 = 2 * (head.Ndim / Tile::BN);
      const int rc = launch_gemm_mfma(mode, epi, a_kcontig, b_kcontig, head, s);
      if (rc != SPES_OK) return rc;
      if (epi == kEpiStore && b_kcontig) return launch<kRaggedM, kEpiStore, true, true, false, false, TileNarrow>(rest, s);
      if (epi == kEpiStore && !b_kcontig) return launch<kRaggedM, kEpiStore, true, false, false, false, TileNarrow>(rest, s);
      if (epi == kEpiDSwiglu && !b_kcontig) return launch<kRaggedM, kEpiDSwiglu, true, false, false, false, TileNarrow>(rest, s);
      return SPES_EINVAL;
    }
    if (epi != kEpiSwiglu && g.n_base == 0 && few_tiles_narrow(g.Ndim, g.est_tiles)) {
      if (epi == kEpiStore && b_kcontig) return launch<kRaggedM, kEpiStore, true, true, false, false, TileNarrow>(g, s);
      if (epi == kEpiStore && !b_kcontig) return launch<kRaggedM, kEpiStore, true, false, false, false, TileNarrow>(g, s);
      if (epi == kEpiDSwiglu && !b_kcontig) return launch<kRaggedM, kEpiDSwiglu, true, false, false, false, TileNarrow>(g, s);
      return SPES_EINVAL;
    }
    if (epi == kEpiSwiglu && b_kcontig) return launch<kRaggedM, kEpiSwiglu, true, true>(g, s);
    if (epi == kEpiStore && b_kcontig) return launch<kRaggedM, kEpiStore, true, true>(g, s);
    if (epi == kEpiStore && !b_kcontig) return launch<kRaggedM, kEpiStore, true, false>(g, s);
    if (epi == kEpiDSwiglu && !b_kcontig) return launch<kRaggedM, kEpiDSwiglu, true, false>(g, s);
    return SPES_EINVAL;
  }
  if (epi != kEpiStore) return SPES_EINVAL;
  if (a_kcontig && b_kcontig)
    return g.Ndim <= TileNarrow::BN ? launch<kGroupedK, kEpiStore, true, true, false, false, TileNarrow>(g, s)
                                    : launch<kGroupedK, kEpiStore, true, true>(g, s);
  if (a_kcontig && !b_kcontig)
    return (g.kchunk <= TileSmall::BK && g.n_groups == 1) ? launch<kGroupedK, kEpiStore, true, false, false, false, TileSmall>(g, s)
                                                          : launch<kGroupedK, kEpiStore, true, false>(g, s);
  if (g.b_rows && (a_kcontig || b_kcontig || g.a_rows)) return SPES_EINVAL;
  if (!a_kcontig && !b_kcontig) {
    if (g.a_rows) return launch<kGroupedK, kEpiStore, false, false, true>(g, s);
    if (g.b_rows) return launch<kGroupedK, kEpiStore, false, false, false, true>(g, s);
    if (g.Mdim <= TileShort::BM) return launch<kGroupedK, kEpiStore, false, false, false, false, TileShort>(g, s);
    return launch<kGroupedK, kEpiStore, false, false>(g, s);
  }
  return SPES_EINVAL;
}

}  // namespace spes
