// Problem description shared by the grouped GEMM kernels.
//
// Every contraction of the layer is written as  C(m,n) = sum_k A(m,k) * B(n,k)
// with element strides for each operand, in one of two groupings:
//
//  kRaggedM  (forward and input-gradient GEMMs): the rows m are the routed rows
//            in expert-contiguous order; a device-side tile table maps each row
//            tile to its expert, whose weight matrix is operand B.
//  kGroupedK (weight gradients, router GEMMs, the fp32 Gram matrix): each group
//            contracts over its own range of k -- the routed rows of one
//            trainable expert, or a uniform chunk of a long contraction.
#pragma once
#include "common.h"

namespace spes {

enum GemmMode { kRaggedM = 0, kGroupedK = 1 };
enum GemmEpi {
  kEpiStore = 0,    // C[0] = acc (or += when accumulate)
  kEpiSwiglu = 1,   // two accumulators a (pair 0), b (pair 1): C[0]=a, C[1]=b, C[2]=SiLU(a)*b.  Vector path: a, b in f32.
                    // Matrix-core path: a, b rounded to bf16 and C[3] = bf16(h - SiLU(bf16 a)*(bf16 b)), so that the backward
                    // has h to ~2^-17 from six bytes per element instead of eight
  kEpiDSwiglu = 2   // acc = u (row of dy times W_d); with saved a=E[0], b=E[1] (and E[2], the correction above), h = SiLU(a)*b:
                    //   rowdot[tile_n][m] = sum_n u*h (the gate gradient), dh = row_scale[m]*u,
                    //   C[0] = da = dh*b*s(1+a(1-s)), C[1] = db = dh*a*s, s = sigmoid(a), C[2] = row_scale[m]*h
};

struct GemmArgs {
  const void* A[2];
  const void* B[2];
  long a_elems, b_elems;  // matrix-core path: elements addressable from A[i] and from B[i] (reads beyond return zero)
  long a_ms, a_ks;        // element strides of A along m, k
  const int* a_rows;      // optional gather: kRaggedM reads row a_rows[m] in place of m; kGroupedK reads row a_rows[k] in place of k
  const int* b_rows;      // optional gather, kGroupedK with K-strided B only: B reads row b_rows[k] in place of k
  const float* row_scale; // kEpiDSwiglu: per-row factor (the gate of the routed pair)
  float* rowdot;          // kEpiDSwiglu: [gridDim.x, rowdot_stride] partial gate gradients
  long rowdot_stride;
  long b_ns, b_ks, b_gs;  // element strides of B along n, k, and per expert (kRaggedM)
  int npairs;             // kEpiStore/kEpiDSwiglu: (A,B) pairs accumulated into one result
  int Kdim;               // contraction length of each pair (kRaggedM) / total K (kGroupedK, uniform chunks)
  void* C[4];
  const void* E[3];
  long c_ms;              // row stride of C and E (n stride is 1)
  long c_gs;              // per-group stride of C (kGroupedK)
  int c_f32;              // C is float whatever the storage type
  int accumulate;
  int Mdim, Ndim;         // extent of m (kGroupedK) and of n
  int n_base;             // kRaggedM: first column this launch computes (columns n_base .. Ndim-1); 0 unless a launch is split
  int rowdot_slot0;       // kEpiDSwiglu: first partial slot this launch writes
  // kRaggedM
  const int* tile_expert;
  const int* tile_row0;
  const int* n_tiles;
  const int* offset;      // [M+1] first routed row of each expert
  int max_tiles;
  int est_tiles;          // expected number of row tiles (the count itself is only known on the device); 0: unknown
  unsigned long long c2_skip;  // kEpiDSwiglu: bit e set = nothing reads C[2] for expert e's rows; the matrix-core path leaves them unwritten
  // kGroupedK
  int n_groups;
  int kchunk;             // offset == nullptr: group g contracts k in [g*kchunk, min(Kdim,(g+1)*kchunk))
  unsigned char group_expert[64];  // offset != nullptr: group g contracts rows [offset[e], offset[e+1]), e = group_expert[g]
};

__device__ __forceinline__ float sigmoidf_(float a) { return __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

// launchers (storage type T of A/B/C unless stated); defined in gemm_simt.hip / gemm_mfma.hip
int launch_gemm_simt(int dtype_a, int dtype_b, int mode, int epi, const GemmArgs& g, hipStream_t s);
int launch_gemm_mfma(int mode, int epi, bool a_kcontig, bool b_kcontig, const GemmArgs& g, hipStream_t s);
int simt_row_tile();
int simt_col_tile();
int mfma_row_tile();
int mfma_rowdot_parts(int ndim, int est_tiles);

}  // namespace spes
