// Streaming kernels of the synchronisation step: the weighted average of
// node-local expert copies (paper Sec. 3.3 Eq. 4), and the expert-merging
// warm-up (Eq. 5-6): similarity -> top-K peers -> task-arithmetic mix.
// Pure HBM streams: 16-byte vectors, fp32 arithmetic, one rounding on store.
#include <vector>

#include "kernels.h"

namespace spes {
namespace {

constexpr int kMergeEntries = 224;   // (source pointer, weight) pairs per launch
constexpr int kMergeExperts = 32;    // experts per launch

struct MergeTable {
  const void* src[kMergeEntries];
  float w[kMergeEntries];            // weight / sum of weights over the expert's trainers
  long dst_off[kMergeExperts];       // element offset of the expert in dst
  int first[kMergeExperts + 1];      // entries [first[e], first[e+1]) belong to expert e of this launch
};

// dst = c_0 + sum_{i>0} w_i (c_i - c_0): equal to the weighted mean because the
// weights sum to one; exact when all copies agree and a plain copy for one trainer.
template <typename T>
__global__ __launch_bounds__(256) void sync_merge_kernel(const MergeTable tb, T* __restrict__ dst, long nvec) {
  constexpr int N = Vec16<T>::N;
  const int e = blockIdx.y;
  const int b = tb.first[e], n = tb.first[e + 1] - b;
  T* out = dst + tb.dst_off[e];
  const long stride = (long)gridDim.x * 256;
  for (long v = (long)blockIdx.x * 256 + threadIdx.x; v < nvec; v += stride) {
    Vec16<T> q;
    q.load_once(reinterpret_cast<const T*>(tb.src[b]) + v * N);
    if (n > 1) {
      float f0[N], acc[N];
      q.unpack(f0);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = f0[i];
      // four copies are requested before the first is used; the order of the additions stays s = 1, 2, ...
      int s = 1;
      for (; s + 4 <= n; s += 4) {
        Vec16<T> qs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) qs[u].load_once(reinterpret_cast<const T*>(tb.src[b + s + u]) + v * N);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float f[N];
          qs[u].unpack(f);
          const float w = tb.w[b + s + u];
#pragma unroll
          for (int i = 0; i < N; ++i) acc[i] = fmaf(w, f[i] - f0[i], acc[i]);
        }
      }
      for (; s < n; ++s) {
        Vec16<T> qs;
        qs.load_once(reinterpret_cast<const T*>(tb.src[b + s]) + v * N);
        float f[N];
        qs.unpack(f);
        const float w = tb.w[b + s];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(w, f[i] - f0[i], acc[i]);
      }
      q.pack(acc);
    }
    q.store_once(out + v * N);
  }
}

struct CountTable {
  int base, n;
  unsigned char c[1024];
};
__global__ void write_counts_kernel(const CountTable tb, int* __restrict__ trainer_count) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < tb.n) trainer_count[tb.base + i] = tb.c[i];
}

// Gram matrix of up to 64 bf16 rows, G = W W^T, as partial sums over chunks of the (long) row length: a pure stream of
// the matrix, read once (Eq. 5: all pairwise inner products of the flattened input projections).
// The rows lie a whole matrix row apart (megabytes, usually a power of two): an access that touches many rows at the
// same column lands on one memory channel.  Every load instruction therefore reads 1 KB of a single row (64 lanes x
// 16 bytes), and the 64 x 512 sub-tile goes through LDS (global -> registers -> LDS, the next sub-tile's loads in
// flight while this one is multiplied).  Both operands of every product are the same data: lane l reads the sixteen
// bytes of row l%32 (+32 for the second fragment) that a 32x32x16 MFMA expects at k = (l/32)*8 .. +8 of a k-step, and
// the two fragments feed all four 32x32 blocks of the 64x64 result; register r of lane l of block (i,j) holds
// G[32i + (r/4)*8 + (l/32)*4 + r%4][32j + l%32].  Wavefront w multiplies k-steps 8w .. 8w+7 of every sub-tile; the four
// wavefronts are added in order through LDS, the block partials in block order by gram_reduce_kernel.
typedef __attribute__((ext_vector_type(8))) __bf16 gram_bf16x8;
typedef __attribute__((ext_vector_type(16))) float gram_f32x16;
constexpr int kGramK = 512;                    // columns per sub-tile: 1 KB of every row
constexpr int kGramPitch = kGramK / 8 + 1;     // LDS row pitch in 16-byte units (odd: fragment reads spread over the banks)
constexpr int kGramRed = 65;                   // floats per row of the reduction buffer

__global__ __launch_bounds__(256, 2) void gram_bf16_kernel(const bf16_t* __restrict__ w, int M, long elems, long kchunk,
                                                           float* __restrict__ partial) {
  __shared__ uint4 tile[64 * kGramPitch];
  static_assert(sizeof(uint4) * 64 * kGramPitch >= sizeof(float) * 4 * 64 * kGramRed, "the reduction reuses the tile");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = lane & 31, half = lane >> 5;
  const long c0 = (long)blockIdx.x * kchunk;
  const long c1 = c0 + kchunk < elems ? c0 + kchunk : elems;
  gram_f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // staging register i of this thread: 16 bytes at column 8*lane of row 4*i + wave
  uint4 st[16];
  auto load_tile = [&](long k) {
    const long kk = k + lane * 8;                         // elems is a multiple of 8: a vector is inside or outside as a whole
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 4 * i + wave;
      st[i] = (r < M && kk < c1) ? load_stream(reinterpret_cast<const uint4*>(w + (long)r * elems + kk)) : make_uint4(0, 0, 0, 0);
    }
  };
  load_tile(c0);
  for (long k = c0; k < c1; k += kGramK) {
    __syncthreads();                                      // the previous sub-tile has been read by every wavefront
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[(4 * i + wave) * kGramPitch + lane] = st[i];
    __syncthreads();
    if (k + kGramK < c1) load_tile(k + kGramK);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int ks = wave * 8 + u;
      const gram_bf16x8 a = __builtin_bit_cast(gram_bf16x8, tile[row * kGramPitch + ks * 2 + half]);
      const gram_bf16x8 b = __builtin_bit_cast(gram_bf16x8, tile[(row + 32) * kGramPitch + ks * 2 + half]);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, b, acc[1][1], 0, 0, 0);
    }
  }
  __syncthreads();
  float* red = reinterpret_cast<float*>(tile);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        red[wave * 64 * kGramRed + (32 * i + (r / 4) * 8 + half * 4 + r % 4) * kGramRed + 32 * j + row] = acc[i][j][r];
  __syncthreads();
  float* out = partial + (long)blockIdx.x * M * M;
  for (int e = tid; e < M * M; e += 256) {
    const int i = e / M, j = e - i * M;
    const int at = i * kGramRed + j;
    out[e] = ((red[at] + red[64 * kGramRed + at]) + red[2 * 64 * kGramRed + at]) + red[3 * 64 * kGramRed + at];
  }
}

// Sum the Gram partials in a fixed order: entry i of the result lands in partial 0.  Wavefront q of a block adds the
// q-th quarter of the partials (ascending), the four quarter sums are then added in order.
__global__ __launch_bounds__(256) void gram_reduce_kernel(float* __restrict__ partial, int n_partial, int n) {
  __shared__ float quarter[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const int per = (n_partial + 3) / 4;
  const int p0 = q * per, p1 = p0 + per < n_partial ? p0 + per : n_partial;
  float acc = 0.f;
  if (i < n) {
    // sixteen loads in flight at a time; the additions keep the order p = p0, p0+1, ...
    int p = p0;
    for (; p + 16 <= p1; p += 16) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = partial[(long)(p + u) * n + i];
#pragma unroll
      for (int u = 0; u < 16; ++u) acc += v[u];
    }
    for (; p < p1; ++p) acc += partial[(long)p * n + i];
  }
  quarter[q][lane] = acc;
  __syncthreads();                 // every partial of these 64 entries has been read before entry i of partial 0 is overwritten
  if (q == 0 && i < n) partial[i] = ((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane];
}

// Normalise the Gram matrix to cosines and pick each row's top-K peers.  Eq. 5 is undefined for an expert whose
// input projection has zero norm; such a pair gets similarity 0.  Whatever the Gram matrix holds (a NaN from
// non-finite weights included), every peer written is a valid expert other than the row's own: the mix kernel
// indexes the store with it.
__global__ __launch_bounds__(256) void sim_topk_kernel(const float* __restrict__ gram, int M, int K,
                                                       float* __restrict__ sim, int* __restrict__ nbr) {
  __shared__ float G[kMaxExperts][kMaxExperts + 1];
  const int tid = threadIdx.x;
  for (int i = tid; i < M * M; i += 256) G[i / M][i % M] = gram[i];
  __syncthreads();
  const int lane = tid & 63, w = tid >> 6;
  for (int j = blockIdx.x * 4 + w; j < M; j += gridDim.x * 4) {     // one row per wavefront
    const bool valid = lane < M && lane != j;                       // lanes that may be chosen as a peer of j
    float a = -INFINITY;
    if (lane < M) {
      const float den = G[j][j] * G[lane][lane];
      a = den > 0.f ? G[j][lane] / sqrtf(den) : 0.f;
      if (sim != nullptr) sim[j * M + lane] = a;
      if (!(a == a)) a = -INFINITY;                                 // a NaN ranks below every number
    }
    bool taken = false;
    int mine = 0;
    for (int i = 0; i < K; ++i) {
      // the largest similarity not taken yet; among equal ones the lowest lane, which is the lowest expert id.
      // K < M, so at least one valid lane is still free, and a free valid lane always matches the maximum
      // taken over the free valid lanes
      const float v = (valid && !taken) ? a : -INFINITY;
      const float top = wave_max(v);
      const int ix = __ffsll((long long)__ballot(valid && !taken && v == top)) - 1;
      if (lane == ix) taken = true;
      if (lane == i) mine = ix;
    }
    if (lane < K) nbr[j * K + lane] = mine;
  }
}

// dst[j] = src[j] + scale * sum_{q in nbr[j]} (src[q] - src[j])
// One block per (expert, run of 256 vectors).  An expert's peers are other rows of the same matrix at the same columns,
// so the blocks are ordered to make those reads hit the L2: workgroups go to the eight XCDs round-robin, and XCD x
// takes the column runs x, x+8, ... with all M experts of a run on consecutive blocks.  The M rows of a run (M x 4 KB)
// are then in flight on one XCD at the same time and each is fetched from memory once instead of once per reader
// (measured: 256 MiB fetched per 256 MiB matrix, against 1187 MiB with the experts as the slow grid axis).  What is
// left is L2 bandwidth: 99 us + 10 us per peer for a 256 MiB matrix.  Staging the M rows of a run in LDS instead
// (one block per run, peers read from LDS) was measured slower: 130 us + 10 us per peer.
template <typename T>
__global__ __launch_bounds__(256) void warmup_mix_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                         const int* __restrict__ nbr, int M, int K, float scale, long nvec, long elems) {
  constexpr int N = Vec16<T>::N;
  const long b = blockIdx.x;
  const long within = b / 8;
  const int j = (int)(within % M);
  const long run = (within / M) * 8 + (b % 8);
  const long v = run * 256 + threadIdx.x;
  if (v >= nvec) return;
  Vec16<T> q;
  q.load(src + (long)j * elems + v * N);
  float f0[N], acc[N];
  q.unpack(f0);
#pragma unroll
  for (int i = 0; i < N; ++i) acc[i] = 0.f;
  // peers four at a time, all four reads requested before the first is used; the sum keeps the order of nbr
  for (int s0 = 0; s0 < K; s0 += 4) {
    Vec16<T> qs[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int peer = nbr[j * K + min(s0 + u, K - 1)];
      qs[u].load(src + (long)peer * elems + v * N);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float f[N];
      qs[u].unpack(f);
      const bool live = s0 + u < K;
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] += live ? f[i] - f0[i] : 0.f;
    }
  }
#pragma unroll
  for (int i = 0; i < N; ++i) acc[i] = fmaf(scale, acc[i], f0[i]);
  q.pack(acc);
  q.store_once(dst + (long)j * elems + v * N);
}

inline int ok() { return hipGetLastError() == hipSuccess ? SPES_OK : SPES_EHIP; }

// one 16-byte vector per thread where the grid allows it: more, shorter blocks measured 10 % faster than four vectors each
inline int stream_grid_x(long nvec) {
  long b = (nvec + 255) / 256;
  if (b < 1) b = 1;
  if (b > 8192) b = 8192;
  return (int)b;
}

template <typename T>
int flush(const MergeTable& tb, int n, void* dst, long elems, hipStream_t s) {
  if (n == 0) return SPES_OK;
  const long nvec = elems / Vec16<T>::N;
  hipLaunchKernelGGL(sync_merge_kernel<T>, dim3(stream_grid_x(nvec), n), dim3(256), 0, s, tb, (T*)dst, nvec);
  return ok();
}

}  // namespace

int launch_sync_merge(int dtype, int n_experts, long elems, int n_nodes, const void* const* node_store, const int* slot,
                      const float* node_weight, void* dst, int* trainer_count, hipStream_t s) {
  const size_t es = dtype == SPES_F32 ? 4 : 2;
  MergeTable tb;
  int n_in = 0, n_ent = 0;
  tb.first[0] = 0;
  std::vector<unsigned char> counts(n_experts, 0);
  for (int j = 0; j < n_experts; ++j) {
    int n = 0;
    double wsum = 0.0;
    for (int i = 0; i < n_nodes; ++i)
      if (slot[(long)i * n_experts + j] >= 0) { ++n; wsum += node_weight ? (double)node_weight[i] : 1.0; }
    counts[j] = (unsigned char)n;
    if (n == 0) continue;
    if (n_in == kMergeExperts || n_ent + n > kMergeEntries) {
      int rc = dtype == SPES_F32 ? flush<float>(tb, n_in, dst, elems, s) : flush<bf16_t>(tb, n_in, dst, elems, s);
      if (rc != SPES_OK) return rc;
      n_in = 0; n_ent = 0;
    }
    for (int i = 0; i < n_nodes; ++i) {
      const int sl = slot[(long)i * n_experts + j];
      if (sl < 0) continue;
      tb.src[n_ent] = static_cast<const char*>(node_store[i]) + (size_t)sl * elems * es;
      tb.w[n_ent] = (float)((node_weight ? (double)node_weight[i] : 1.0) / wsum);
      ++n_ent;
    }
    tb.dst_off[n_in] = (long)j * elems;
    tb.first[++n_in] = n_ent;
  }
  int rc = dtype == SPES_F32 ? flush<float>(tb, n_in, dst, elems, s) : flush<bf16_t>(tb, n_in, dst, elems, s);
  if (rc != SPES_OK) return rc;
  if (trainer_count != nullptr) {
    for (int base = 0; base < n_experts; base += 1024) {
      CountTable ct;
      ct.base = base;
      ct.n = n_experts - base < 1024 ? n_experts - base : 1024;
      for (int i = 0; i < ct.n; ++i) ct.c[i] = counts[base + i];
      hipLaunchKernelGGL(write_counts_kernel, dim3(cdiv(ct.n, 256)), dim3(256), 0, s, ct, trainer_count);
    }
    if (ok() != SPES_OK) return SPES_EHIP;
  }
  return SPES_OK;
}

// partial[b][M*M], b < n_groups: Gram partial of columns [b*kchunk, (b+1)*kchunk) of the bf16 matrix w [M, elems]
int launch_gram_bf16(const void* w, int M, long elems, int n_groups, long kchunk, float* partial, hipStream_t s) {
  if (M > 64 || kchunk % 8 != 0 || elems % 8 != 0) return SPES_ESHAPE;
  hipLaunchKernelGGL(gram_bf16_kernel, dim3(n_groups), dim3(256), 0, s, (const bf16_t*)w, M, elems, kchunk, partial);
  return ok();
}

int launch_sim_topk(float* partial, int n_partial, int M, int K, float* sim, int* nbr, hipStream_t s) {
  hipLaunchKernelGGL(gram_reduce_kernel, dim3(cdiv((long)M * M, 64)), dim3(256), 0, s, partial, n_partial, M * M);
  hipLaunchKernelGGL(sim_topk_kernel, dim3(cdiv(M, 4)), dim3(256), 0, s, partial, M, K, sim, nbr);
  return ok();
}

int launch_warmup_mix(int dtype, int M, long elems, int K, float alpha, const void* src, void* dst, const int* nbr, hipStream_t s) {
  const float scale = alpha / (float)K;
  const long nvec = elems / (dtype == SPES_F32 ? 4 : 8);
  const long runs8 = (long)cdiv(cdiv(nvec, 256), 8) * 8;         // column runs, rounded up to a whole turn of the XCDs
  const long blocks = runs8 * M;
  if (blocks <= 0) return SPES_OK;
  if (blocks > 0x7fffffffL) return SPES_ESHAPE;
  if (dtype == SPES_F32)
    hipLaunchKernelGGL(warmup_mix_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, (const float*)src, (float*)dst, nbr, M, K, scale,
                       nvec, elems);
  else
    hipLaunchKernelGGL(warmup_mix_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t*)src, (bf16_t*)dst, nbr, M, K,
                       scale, nvec, elems);
  return ok();
}

}  // namespace spes
