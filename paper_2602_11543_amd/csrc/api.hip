// C ABI of the library: argument checks, context layout and the launch
// sequences of the forward, backward, synchronisation and warm-up merge.
#include <cmath>
#include <cstring>
#include <mutex>

#include "kernels.h"

using namespace spes;

namespace {

constexpr int kLogitSplit = 4;    // chunks of d_model in the router GEMM on the matrix cores
constexpr int kRouterSplit = 64;   // chunks of the token axis in the router weight gradient

struct Layout {
  spes_moe_ctx_layout pub;
  size_t block_counts, tab_simt, tab_mfma, row_token, row_gate, hcorr, dgate_part, da, db, hg, dxp, wr_part, dlogits_bf, dxr, aux, aux_part;
  int max_tiles, max_tiles_mfma, est_tiles_mfma, max_col_tiles;
};

bool shape_ok(const spes_moe_shape* s) {
  if (s == nullptr) return false;
  if (s->T <= 0 || s->d_model <= 0 || s->n_experts <= 0 || s->d_ff <= 0 || s->top_k <= 0) return false;
  if (s->top_k > s->n_experts) return false;
  if (s->dtype != SPES_F32 && s->dtype != SPES_BF16) return false;
  return true;
}

int shape_supported(const spes_moe_shape* s) {
  if (!shape_ok(s)) return SPES_EINVAL;
  if (s->n_experts > kMaxExperts) return SPES_ESHAPE;
  if (s->d_model % 8 || s->d_ff % 8) return SPES_ESHAPE;
  const long R = (long)s->T * s->top_k;
  // the row tiles of the vector-ALU GEMMs (64 rows each, at most one partly filled tile per expert) are a grid
  // dimension of at most 65535
  if (R / 64 + kMaxExperts + 1 > 65535) return SPES_ESHAPE;
  if (s->dtype == SPES_BF16) {
    // the matrix-core GEMMs address their operands with 32-bit byte offsets: x / dy, the saved and scratch [R,f]
    // activations and the expert weight tensors must each stay below 2^31 elements
    const long lim = 1L << 31;
    if ((long)s->T * s->d_model >= lim || R * s->d_ff >= lim || (long)s->n_experts * s->d_ff * s->d_model >= lim) return SPES_ESHAPE;
  }
  return SPES_OK;
}

Layout make_layout(const spes_moe_shape* s) {
  Layout L;
  const size_t T = s->T, d = s->d_model, M = s->n_experts, f = s->d_ff, k = s->top_k;
  const size_t R = T * k, es = s->dtype == SPES_F32 ? 4 : 2;
  L.max_tiles = (int)(R / 64 + M + 1);
  L.max_tiles_mfma = (int)(R / 256 + M + 1);
  L.est_tiles_mfma = (int)(R / 256 + (M + 1) / 2);   // expected count: half of the experts end in a partly filled tile
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
  L.pub.logits = take(kLogitSplit * T * M * 4);   // partial score matrices; the first one ends up holding the scores
  L.pub.lse = take(T * 4);
  L.pub.topk_idx = take(R * 4);
  L.pub.topk_gate = take(R * 4);
  L.pub.offset = take((M + 1) * 4);
  L.pub.perm = take(R * 4);
  L.pub.inv = take(R * 4);
  L.block_counts = take((size_t)routing_blocks((int)R) * kMaxExperts * 4);
  L.tab_simt = take((1 + 2 * (size_t)L.max_tiles) * 4);
  L.tab_mfma = take((1 + 2 * (size_t)L.max_tiles) * 4);
  L.row_token = take(R * 4);
  L.row_gate = take(R * 4);
  // fp32 storage keeps the projections in fp32; bf16 storage keeps them in bf16 plus a bf16 correction of h
  L.pub.a = take(R * f * (es == 4 ? 4 : 2));
  L.pub.b = take(R * f * (es == 4 ? 4 : 2));
  L.hcorr = take(es == 4 ? 0 : R * f * 2);
  L.pub.h = take(R * f * es);
  L.pub.yp = take(R * d * es);
  L.pub.dlogits = take(T * M * 4);
  L.pub.dgate = take(T * k * 4);
  L.max_col_tiles = cdiv((long)f, 64) + 1;   // covers both GEMM paths: f/64 (vector ALU) and 2*ceil(f/128) (matrix core)
  L.dgate_part = take((size_t)L.max_col_tiles * R * 4);
  L.da = take(R * f * es);
  L.db = take(R * f * es);
  L.hg = take(R * f * es);
  L.dxp = take(R * d * es);
  L.wr_part = take((size_t)kRouterSplit * M * d * 4);
  L.dlogits_bf = take(T * M * 2);
  L.dxr = take(T * d * es);
  L.aux = take((kMaxExperts + kAuxExtra) * 4);
  L.aux_part = take((size_t)kAuxBlocks * (kMaxExperts + 1) * 4);
  L.pub.total = off;
  return L;
}

template <typename T>
T* at(void* base, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(base) + off); }

// bf16 storage runs the expert GEMMs on the matrix cores, fp32 storage on the vector ALUs
int expert_gemm(int dt, int mode, int epi, bool a_kcontig, bool b_kcontig, const GemmArgs& g, hipStream_t s) {
  if (dt == SPES_BF16) return launch_gemm_mfma(mode, epi, a_kcontig, b_kcontig, g, s);
  return launch_gemm_simt(dt, dt, mode, epi, g, s);
}

void ragged_tables(GemmArgs& g, void* ctx, const Layout& L, int dt) {
  int* tab = at<int>(ctx, dt == SPES_BF16 ? L.tab_mfma : L.tab_simt);
  g.n_tiles = tab;
  g.tile_expert = tab + 1;
  g.tile_row0 = tab + 1 + L.max_tiles;
  g.offset = at<int>(ctx, L.pub.offset);
  g.max_tiles = dt == SPES_BF16 ? L.max_tiles_mfma : L.max_tiles;   // launch bound on the number of row tiles
  g.est_tiles = dt == SPES_BF16 ? L.est_tiles_mfma : 0;
}

GemmArgs blank() {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.npairs = 1;
  g.n_groups = 1;
  return g;
}

// Optional stage timing: HIP events recorded on the caller's stream between the stages of fwd and bwd.
// This is the library's only process-level state; it holds no device memory.
constexpr int kMaxStages = 24;
struct Profile {
  bool on = false, created = false;
  hipEvent_t ev[2][kMaxStages + 1];
  const char* name[2][kMaxStages];
  int n[2] = {0, 0};
} g_prof;

void prof_begin(int which, hipStream_t s) {
  if (!g_prof.on) return;
  g_prof.n[which] = 0;
  (void)hipEventRecord(g_prof.ev[which][0], s);
}
void prof_mark(int which, const char* name, hipStream_t s) {
  if (!g_prof.on || g_prof.n[which] >= kMaxStages) return;
  const int i = g_prof.n[which]++;
  g_prof.name[which][i] = name;
  (void)hipEventRecord(g_prof.ev[which][i + 1], s);
}

#define SPES_TRY(expr) do { int rc_ = (expr); if (rc_ != SPES_OK) return rc_; } while (0)

}  // namespace

extern "C" {

SPES_API size_t spes_moe_ctx_bytes(const spes_moe_shape* shape) {
  if (shape_supported(shape) != SPES_OK) return 0;
  return make_layout(shape).pub.total;
}

SPES_API int spes_moe_ctx_describe(const spes_moe_shape* shape, spes_moe_ctx_layout* out) {
  if (out == nullptr) return SPES_EINVAL;
  SPES_TRY(shape_supported(shape));
  *out = make_layout(shape).pub;
  return SPES_OK;
}

SPES_API int spes_moe_fwd(const spes_moe_shape* shape, const void* x, const void* w_router, const float* router_bias,
                          const void* w_gate, const void* w_up, const void* w_down, void* y, int32_t* topk_idx,
                          float* topk_gate, int32_t* expert_count, void* ctx, void* stream) {
  SPES_TRY(shape_supported(shape));
  if (!x || !w_router || !w_gate || !w_up || !w_down || !y || !topk_idx || !topk_gate || !expert_count || !ctx)
    return SPES_EINVAL;
  if (!aligned16(x) || !aligned16(w_router) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(y) ||
      !aligned16(topk_idx) || !aligned16(topk_gate) || !aligned16(expert_count) || !aligned16(ctx) ||
      (router_bias && !aligned16(router_bias)))
    return SPES_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Layout L = make_layout(shape);
  const int T = shape->T, d = shape->d_model, M = shape->n_experts, f = shape->d_ff, k = shape->top_k, dt = shape->dtype;
  const long R = (long)T * k;

  prof_begin(0, s);
  int logit_parts = 1;
  // router scores: logits[T,M] = x W_r^T
  {
    GemmArgs g = blank();
    g.A[0] = x; g.a_ms = d; g.a_ks = 1; g.a_elems = (long)T * d;
    g.B[0] = w_router; g.b_ns = d; g.b_ks = 1; g.b_elems = (long)M * d;
    g.Kdim = d; g.kchunk = d; g.Mdim = T; g.Ndim = M;
    g.C[0] = at<float>(ctx, L.pub.logits); g.c_ms = M; g.c_f32 = 1;
    // the matrix-core epilogue stores four columns at a time; with only M <= 64 output columns the row tiles alone
    // would occupy a quarter of the CUs, so d_model is cut into partial products that the gating kernel adds up
    if (dt == SPES_BF16 && M % 4 == 0) {
      g.kchunk = (cdiv(d, kLogitSplit) + 63) / 64 * 64; g.n_groups = cdiv(d, g.kchunk); g.c_gs = (long)T * M;
      logit_parts = g.n_groups;
      SPES_TRY(launch_gemm_mfma(kGroupedK, kEpiStore, true, true, g, s));
    } else {
      SPES_TRY(launch_gemm_simt(dt, dt, kGroupedK, kEpiStore, g, s));
    }
  }
  prof_mark(0, "router_gemm", s);
  SPES_TRY(launch_topk_gate(at<float>(ctx, L.pub.logits), logit_parts, router_bias, T, M, k, shape->renorm_topk, topk_idx, topk_gate,
                            at<int>(ctx, L.pub.topk_idx), at<float>(ctx, L.pub.topk_gate), at<float>(ctx, L.pub.lse), s));
  prof_mark(0, "softmax_topk", s);
  SPES_TRY(launch_routing_tables(topk_idx, topk_gate, (int)R, M, k, at<int>(ctx, L.block_counts), expert_count,
                                 at<int>(ctx, L.pub.offset), at<int>(ctx, L.pub.perm), at<int>(ctx, L.pub.inv),
                                 at<int>(ctx, L.row_token), at<float>(ctx, L.row_gate),
                                 // only the row-tile table of the GEMM path this storage type runs on is built
                                 dt == SPES_BF16 ? 0 : simt_row_tile(), at<int>(ctx, L.tab_simt),
                                 dt == SPES_BF16 ? mfma_row_tile() : 0, at<int>(ctx, L.tab_mfma), L.max_tiles,
                                 at<float>(ctx, L.aux), s));
  prof_mark(0, "hist_scan_rank", s);
  // a = xp W_g^T, b = xp W_u^T, h = SiLU(a) * b with xp[r,:] = x[token of row r,:]: the GEMM reads its operand rows
  // through the row -> token table, the permuted copy of x is never written (spes_moe_permute materialises it)
  {
    GemmArgs g = blank();
    g.A[0] = x; g.a_ms = d; g.a_ks = 1; g.a_elems = (long)T * d; g.a_rows = at<int>(ctx, L.row_token);
    g.B[0] = w_gate; g.B[1] = w_up; g.b_ns = d; g.b_ks = 1; g.b_gs = (long)f * d; g.b_elems = (long)M * f * d;
    g.Kdim = d; g.Ndim = f;
    g.C[0] = at<void>(ctx, L.pub.a); g.C[1] = at<void>(ctx, L.pub.b); g.C[2] = at<void>(ctx, L.pub.h); g.c_ms = f;
    g.C[3] = at<void>(ctx, L.hcorr);
    ragged_tables(g, ctx, L, dt);
    SPES_TRY(expert_gemm(dt, kRaggedM, kEpiSwiglu, true, true, g, s));
  }
  prof_mark(0, "gemm_gate_up_swiglu", s);
  // yp = h W_d^T
  {
    GemmArgs g = blank();
    g.A[0] = at<void>(ctx, L.pub.h); g.a_ms = f; g.a_ks = 1; g.a_elems = R * f;
    g.B[0] = w_down; g.b_ns = f; g.b_ks = 1; g.b_gs = (long)d * f; g.b_elems = (long)M * d * f;
    g.Kdim = f; g.Ndim = d;
    g.C[0] = at<void>(ctx, L.pub.yp); g.c_ms = d;
    ragged_tables(g, ctx, L, dt);
    SPES_TRY(expert_gemm(dt, kRaggedM, kEpiStore, true, true, g, s));
  }
  prof_mark(0, "gemm_down", s);
  SPES_TRY(launch_combine(dt, at<void>(ctx, L.pub.yp), at<int>(ctx, L.pub.inv), topk_gate, y, T, d, k, s));
  prof_mark(0, "combine", s);
  return SPES_OK;
}

SPES_API int spes_moe_permute(const spes_moe_shape* shape, const void* x, const void* ctx, void* xp, void* stream) {
  SPES_TRY(shape_supported(shape));
  if (!x || !ctx || !xp) return SPES_EINVAL;
  if (!aligned16(x) || !aligned16(ctx) || !aligned16(xp)) return SPES_EALIGN;
  const Layout L = make_layout(shape);
  return launch_permute(shape->dtype, x, at<int>(const_cast<void*>(ctx), L.pub.inv), shape->top_k, xp, shape->T, shape->d_model,
                        static_cast<hipStream_t>(stream));
}

SPES_API int spes_moe_grad_scatter(const spes_moe_shape* shape, const void* dy, const void* ctx, void* dyp, float* dgate,
                                   void* stream) {
  SPES_TRY(shape_supported(shape));
  if (!dy || !ctx || !dyp || !dgate) return SPES_EINVAL;
  if (!aligned16(dy) || !aligned16(ctx) || !aligned16(dyp) || !aligned16(dgate)) return SPES_EALIGN;
  const Layout L = make_layout(shape);
  void* c = const_cast<void*>(ctx);
  return launch_grad_scatter(shape->dtype, dy, at<void>(c, L.pub.yp), at<int>(c, L.pub.inv), at<float>(c, L.pub.topk_gate), dyp,
                             dgate, shape->T, shape->d_model, shape->top_k, static_cast<hipStream_t>(stream));
}

SPES_API int spes_moe_router_aux(const spes_moe_shape* shape, void* ctx, float lb_coef, float z_coef, float grad_scale,
                                 float* losses, void* stream) {
  SPES_TRY(shape_supported(shape));
  if (!ctx || !losses) return SPES_EINVAL;
  if (!aligned16(ctx)) return SPES_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Layout L = make_layout(shape);
  return launch_router_aux(at<float>(ctx, L.pub.logits), at<float>(ctx, L.pub.lse), at<int>(ctx, L.pub.offset), shape->T,
                           shape->n_experts, shape->top_k, lb_coef, z_coef, grad_scale, at<float>(ctx, L.aux_part), losses,
                           at<float>(ctx, L.aux), s);
}

SPES_API int spes_moe_bwd(const spes_moe_shape* shape, const void* dy, const void* x, const void* w_router,
                          const void* w_gate, const void* w_up, const void* w_down, void* ctx,
                          const uint8_t* trainable_mask, void* dx, float* d_w_router, float* d_w_gate, float* d_w_up,
                          float* d_w_down, int32_t accumulate, void* stream) {
  SPES_TRY(shape_supported(shape));
  if (!dy || !x || !w_router || !w_gate || !w_up || !w_down || !ctx || !trainable_mask || !dx || !d_w_router) return SPES_EINVAL;
  const int T = shape->T, d = shape->d_model, M = shape->n_experts, f = shape->d_ff, k = shape->top_k, dt = shape->dtype;
  int n_train = 0;
  unsigned char train_list[kMaxExperts];
  for (int e = 0; e < M; ++e)
    if (trainable_mask[e]) train_list[n_train++] = (unsigned char)e;
  if (n_train > 0 && (!d_w_gate || !d_w_up || !d_w_down)) return SPES_EINVAL;
  if (!aligned16(dy) || !aligned16(x) || !aligned16(w_router) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) ||
      !aligned16(ctx) || !aligned16(dx) || !aligned16(d_w_router) || !aligned16(d_w_gate) || !aligned16(d_w_up) ||
      !aligned16(d_w_down))
    return SPES_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Layout L = make_layout(shape);
  const int* inv = at<int>(ctx, L.pub.inv);
  const float* gate = at<float>(ctx, L.pub.topk_gate);   // the forward's own copies: its outputs belong to the caller
  const int* idx = at<int>(ctx, L.pub.topk_idx);

  // u = dy[token] W_d per routed row; its epilogue yields the gate gradient <u, h> (per column tile) and,
  // through the SwiGLU, da and db of the gate-scaled upstream gradient
  const long R = (long)T * k;
  const int n_part = dt == SPES_BF16 ? mfma_rowdot_parts(f, L.est_tiles_mfma) : cdiv(f, simt_col_tile());
  // bf16 storage: the two router contractions run on the matrix cores from a bf16 copy of dlogits
  const bool router_mfma = dt == SPES_BF16 && M % 8 == 0;
  prof_begin(1, s);
  {
    GemmArgs g = blank();
    g.A[0] = dy; g.a_ms = d; g.a_ks = 1; g.a_rows = at<int>(ctx, L.row_token); g.a_elems = (long)T * d;
    g.B[0] = w_down; g.b_ns = 1; g.b_ks = f; g.b_gs = (long)d * f; g.b_elems = (long)M * d * f;
    g.Kdim = d; g.Ndim = f;
    g.E[0] = at<void>(ctx, L.pub.a); g.E[1] = at<void>(ctx, L.pub.b); g.E[2] = at<void>(ctx, L.hcorr);
    g.C[0] = at<void>(ctx, L.da); g.C[1] = at<void>(ctx, L.db); g.C[2] = at<void>(ctx, L.hg); g.c_ms = f;
    g.row_scale = at<float>(ctx, L.row_gate);
    g.rowdot = at<float>(ctx, L.dgate_part); g.rowdot_stride = R;
    // gate * h feeds only the down-projection weight gradient, which exists for the trainable experts alone
    for (int e = 0; e < M; ++e)
      if (!trainable_mask[e]) g.c2_skip |= 1ull << e;
    ragged_tables(g, ctx, L, dt);
    SPES_TRY(expert_gemm(dt, kRaggedM, kEpiDSwiglu, true, false, g, s));
  }
  prof_mark(1, "gemm_dgrad_down_dswiglu", s);
  SPES_TRY(launch_gating_bwd(at<float>(ctx, L.pub.logits), at<float>(ctx, L.pub.lse), idx, gate, at<float>(ctx, L.dgate_part),
                             n_part, R, inv, at<float>(ctx, L.pub.dgate), T, M, k, shape->renorm_topk,
                             at<float>(ctx, L.aux), at<float>(ctx, L.pub.dlogits), router_mfma ? at<bf16_t>(ctx, L.dlogits_bf) : nullptr, s));
  prof_mark(1, "gating_bwd", s);
  // dxp = da W_g + db W_u
  {
    GemmArgs g = blank();
    g.npairs = 2;
    g.A[0] = at<void>(ctx, L.da); g.A[1] = at<void>(ctx, L.db); g.a_ms = f; g.a_ks = 1; g.a_elems = R * f;
    g.B[0] = w_gate; g.B[1] = w_up; g.b_ns = 1; g.b_ks = d; g.b_gs = (long)f * d; g.b_elems = (long)M * f * d;
    g.Kdim = f; g.Ndim = d;
    g.C[0] = at<void>(ctx, L.dxp); g.c_ms = d;
    ragged_tables(g, ctx, L, dt);
    SPES_TRY(expert_gemm(dt, kRaggedM, kEpiStore, true, false, g, s));
  }
  prof_mark(1, "gemm_dgrad_gate_up", s);
  // weight gradients of the trainable experts only, into their compact slots
  if (n_train > 0) {
    GemmArgs g = blank();
    g.n_groups = n_train;
    memcpy(g.group_expert, train_list, n_train);
    g.offset = at<int>(ctx, L.pub.offset);
    g.c_f32 = 1; g.accumulate = accumulate;
    // dW_d[d,f] = dy[token]^T (gate * h) over the expert's rows
    g.A[0] = dy; g.a_ms = 1; g.a_ks = d; g.a_rows = at<int>(ctx, L.row_token); g.a_elems = (long)T * d;
    g.B[0] = at<void>(ctx, L.hg); g.b_ns = 1; g.b_ks = f; g.b_elems = R * f;
    g.Mdim = d; g.Ndim = f; g.C[0] = d_w_down; g.c_ms = f; g.c_gs = (long)d * f;
    SPES_TRY(expert_gemm(dt, kGroupedK, kEpiStore, false, false, g, s));
    prof_mark(1, "wgrad_down", s);
    // dW_g[f,d] = da^T xp ; dW_u[f,d] = db^T xp
    g.B[0] = x; g.b_rows = at<int>(ctx, L.row_token); g.b_ns = 1; g.b_ks = d; g.b_elems = (long)T * d;
    g.a_ms = 1; g.a_ks = f; g.a_rows = nullptr; g.a_elems = R * f; g.Mdim = f; g.Ndim = d; g.c_ms = d; g.c_gs = (long)f * d;
    g.A[0] = at<void>(ctx, L.da); g.C[0] = d_w_gate;
    SPES_TRY(expert_gemm(dt, kGroupedK, kEpiStore, false, false, g, s));
    prof_mark(1, "wgrad_gate", s);
    g.A[0] = at<void>(ctx, L.db); g.C[0] = d_w_up;
    SPES_TRY(expert_gemm(dt, kGroupedK, kEpiStore, false, false, g, s));
    prof_mark(1, "wgrad_up", s);
  }
  // dW_r[M,d] = dlogits^T x; the token axis is cut into chunks whose partial products are then added in a fixed order
  {
    GemmArgs g = blank();
    g.a_ms = 1; g.a_ks = M; g.a_elems = (long)T * M;
    g.B[0] = x; g.b_ns = 1; g.b_ks = d; g.b_elems = (long)T * d;
    g.Kdim = T; g.Mdim = M; g.Ndim = d;
    g.C[0] = at<float>(ctx, L.wr_part); g.c_ms = d; g.c_gs = (long)M * d; g.c_f32 = 1;
    if (router_mfma) {
      g.A[0] = at<void>(ctx, L.dlogits_bf);
      g.kchunk = (cdiv(T, kRouterSplit / 2) + 63) / 64 * 64; g.n_groups = cdiv(T, g.kchunk);
      SPES_TRY(launch_gemm_mfma(kGroupedK, kEpiStore, false, false, g, s));
    } else {
      g.A[0] = at<float>(ctx, L.pub.dlogits);
      g.kchunk = cdiv(T, kRouterSplit); g.n_groups = cdiv(T, g.kchunk);
      SPES_TRY(launch_gemm_simt(SPES_F32, dt, kGroupedK, kEpiStore, g, s));
    }
    SPES_TRY(launch_reduce_partials(at<float>(ctx, L.wr_part), g.n_groups, (long)M * d, d_w_router, accumulate, s));
  }
  prof_mark(1, "router_wgrad", s);
  // router part of the input gradient, dxr[T,d] = dlogits W_r, as its own small GEMM in bf16 mode
  if (router_mfma) {
    GemmArgs g = blank();
    g.A[0] = at<void>(ctx, L.dlogits_bf); g.a_ms = M; g.a_ks = 1; g.a_elems = (long)T * M;
    g.B[0] = w_router; g.b_ns = 1; g.b_ks = d; g.b_elems = (long)M * d;
    g.Kdim = M; g.kchunk = (M + 63) / 64 * 64; g.Mdim = T; g.Ndim = d;
    g.C[0] = at<void>(ctx, L.dxr); g.c_ms = d;
    SPES_TRY(launch_gemm_mfma(kGroupedK, kEpiStore, true, false, g, s));
    prof_mark(1, "router_dgrad", s);
  }
  // dx = unpermuted sum of dxp + router part
  SPES_TRY(launch_dx_gather(dt, at<void>(ctx, L.dxp), inv, at<float>(ctx, L.pub.dlogits), w_router,
                            router_mfma ? at<void>(ctx, L.dxr) : nullptr, dx, T, d, k, M, s));
  prof_mark(1, "unpermute_sum_router_dgrad", s);
  return SPES_OK;
}

SPES_API int spes_masked_adamw(int32_t n_experts, int64_t elems, int32_t dtype, void* param, const uint8_t* trainable_mask,
                               float* master, float* m, float* v, const float* grad, float lr, float beta1, float beta2,
                               float eps, float weight_decay, int32_t step, float grad_scale, void* stream) {
  if (n_experts < 1 || elems < 1 || step < 1 || (dtype != SPES_F32 && dtype != SPES_BF16) || !param || !trainable_mask)
    return SPES_EINVAL;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return SPES_EINVAL;
  if (elems % 8) return SPES_ESHAPE;
  bool any = false;
  for (int e = 0; e < n_experts; ++e) any = any || trainable_mask[e];
  if (!any) return SPES_OK;
  if (!m || !v || !grad || (!master && dtype != SPES_F32)) return SPES_EINVAL;
  if (!aligned16(param) || !aligned16(m) || !aligned16(v) || !aligned16(grad) || (master && !aligned16(master))) return SPES_EALIGN;
  return launch_masked_adamw(dtype, n_experts, elems, param, trainable_mask, master, m, v, grad, lr, beta1, beta2, eps,
                             weight_decay, step, grad_scale, static_cast<hipStream_t>(stream));
}

SPES_API int spes_upcycle_init(int32_t n_experts, int64_t elems, int32_t dtype, const void* dense, float fraction, float sigma,
                               uint64_t seed, uint64_t stream_id, void* out, void* stream) {
  if (n_experts < 1 || elems < 1 || (dtype != SPES_F32 && dtype != SPES_BF16) || !dense || !out) return SPES_EINVAL;
  if (!(fraction >= 0.f && fraction <= 1.f) || !(sigma >= 0.f)) return SPES_EINVAL;
  if (elems % 8) return SPES_ESHAPE;
  if (!aligned16(dense) || !aligned16(out)) return SPES_EALIGN;
  const unsigned thr = (unsigned)floor((double)fraction * 256.0);
  return launch_upcycle_init(dtype, n_experts, elems, dense, thr, sigma, seed, stream_id, out, static_cast<hipStream_t>(stream));
}

SPES_API int spes_expert_pack(int32_t n_experts, int64_t elems, int32_t dtype, void* store, const uint8_t* trainable_mask,
                              void* packed, int32_t to_store, void* stream) {
  if (n_experts < 1 || elems < 1 || (dtype != SPES_F32 && dtype != SPES_BF16) || !store || !trainable_mask) return SPES_EINVAL;
  if (elems % 8) return SPES_ESHAPE;
  bool any = false;
  for (int e = 0; e < n_experts; ++e) any = any || trainable_mask[e];
  if (!any) return SPES_OK;
  if (!packed) return SPES_EINVAL;
  if (!aligned16(store) || !aligned16(packed)) return SPES_EALIGN;
  return launch_expert_pack(dtype, n_experts, elems, store, trainable_mask, packed, to_store != 0, static_cast<hipStream_t>(stream));
}

SPES_API int spes_expert_merge(int32_t n_experts, int64_t elems, int32_t dtype, int32_t n_nodes,
                               const void* const* node_store, const int32_t* slot, const float* node_weight, void* dst,
                               int32_t* trainer_count, void* stream) {
  if (n_experts <= 0 || elems <= 0 || n_nodes <= 0 || !node_store || !slot || !dst) return SPES_EINVAL;
  if (dtype != SPES_F32 && dtype != SPES_BF16) return SPES_EINVAL;
  if (elems % 8) return SPES_ESHAPE;
  if (!aligned16(dst) || (trainer_count && !aligned16(trainer_count))) return SPES_EALIGN;
  for (int i = 0; i < n_nodes; ++i) {
    bool used = false;
    for (int j = 0; j < n_experts; ++j) used |= slot[(long)i * n_experts + j] >= 0;
    if (used && !node_store[i]) return SPES_EINVAL;
    if (used && !aligned16(node_store[i])) return SPES_EALIGN;
    if (node_weight && !(node_weight[i] > 0.f)) return SPES_EINVAL;
  }
  for (int j = 0; j < n_experts; ++j) {
    int n = 0;
    for (int i = 0; i < n_nodes; ++i) n += slot[(long)i * n_experts + j] >= 0;
    if (n > 224) return SPES_ESHAPE;
  }
  return launch_sync_merge(dtype, n_experts, elems, n_nodes, node_store, slot, node_weight, dst, trainer_count,
                           static_cast<hipStream_t>(stream));
}

// chunks of the long contraction of the Gram matrix, one partial sum each
constexpr int kMaxGramGroups = 512;
static int gram_groups(int64_t elems_in) {
  long g = (elems_in + 4095) / 4096;
  if (g > kMaxGramGroups) g = kMaxGramGroups;
  if (g < 1) g = 1;
  return (int)g;
}

SPES_API size_t spes_warmup_scratch_bytes(int32_t n_experts, int64_t elems_in) {
  if (n_experts <= 0 || n_experts > kMaxExperts || elems_in <= 0) return 0;
  return (size_t)gram_groups(elems_in) * n_experts * n_experts * 4;
}

SPES_API int spes_expert_warmup_merge(int32_t n_experts, int32_t dtype, int32_t top_K, float alpha, const void* w_in,
                                      int64_t elems_in, int32_t n_mats, const void* const* src, void* const* dst,
                                      const int64_t* elems, float* sim, int32_t* nbr, void* scratch, void* stream) {
  if (n_experts <= 1 || top_K <= 0 || top_K >= n_experts || !w_in || elems_in <= 0 || n_mats < 0 || !nbr || !scratch)
    return SPES_EINVAL;
  if (dtype != SPES_F32 && dtype != SPES_BF16) return SPES_EINVAL;
  if (n_mats > 0 && (!src || !dst || !elems)) return SPES_EINVAL;
  if (n_experts > kMaxExperts || elems_in % 8 || elems_in >= (1LL << 31)) return SPES_ESHAPE;
  if (!aligned16(w_in) || !aligned16(nbr) || !aligned16(scratch) || (sim && !aligned16(sim))) return SPES_EALIGN;
  for (int m = 0; m < n_mats; ++m) {
    if (!src[m] || !dst[m] || src[m] == dst[m] || elems[m] <= 0) return SPES_EINVAL;
    if (elems[m] % 8) return SPES_ESHAPE;
    if (!aligned16(src[m]) || !aligned16(dst[m])) return SPES_EALIGN;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int M = n_experts;
  const int ng = gram_groups(elems_in);
  const long kchunk = ((elems_in + ng - 1) / ng + 63) / 64 * 64;   // whole K-tiles per group
  if (dtype == SPES_BF16) {
    // Gram matrix of the flattened input projections: one streaming pass, a partial sum per chunk of the long contraction
    SPES_TRY(launch_gram_bf16(w_in, M, elems_in, ng, kchunk, static_cast<float*>(scratch), s));
  } else {
    GemmArgs g = blank();
    g.A[0] = w_in; g.a_ms = elems_in; g.a_ks = 1; g.a_elems = (long)n_experts * elems_in;
    g.B[0] = w_in; g.b_ns = elems_in; g.b_ks = 1; g.b_elems = (long)n_experts * elems_in;
    g.Kdim = (int)elems_in; g.kchunk = (int)kchunk; g.n_groups = ng;
    g.Mdim = M; g.Ndim = M;
    g.C[0] = scratch; g.c_ms = M; g.c_gs = (long)M * M; g.c_f32 = 1;
    SPES_TRY(launch_gemm_simt(dtype, dtype, kGroupedK, kEpiStore, g, s));
  }
  SPES_TRY(launch_sim_topk(static_cast<float*>(scratch), ng, M, top_K, sim, nbr, s));
  for (int m = 0; m < n_mats; ++m)
    SPES_TRY(launch_warmup_mix(dtype, M, elems[m], top_K, alpha, src[m], dst[m], nbr, s));
  return SPES_OK;
}

// Scratch of spes_expert_warmup_merge_static: the Gram partials of the largest supported problem.  Every GPU the
// library runs on holds its own copy for the life of the process.
constexpr size_t kStaticScratchBytes = (size_t)kMaxGramGroups * kMaxExperts * kMaxExperts * 4;   // 8 MiB
static __device__ __align__(256) unsigned char g_warmup_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;

// device address of g_warmup_scratch on the current device (the array's name is a host-side stand-in, not an address)
static int static_scratch(void** out) {
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {nullptr};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPES_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_warmup_scratch)) != hipSuccess || p == nullptr) return SPES_EHIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return SPES_OK;
}

SPES_API int spes_expert_warmup_merge_static(int32_t n_experts, int32_t dtype, int32_t top_K, float alpha, const void* w_in,
                                             int64_t elems_in, int32_t n_mats, const void* const* src, void* const* dst,
                                             const int64_t* elems, float* sim, int32_t* nbr, void* stream) {
  if (n_experts <= 0 || elems_in <= 0) return SPES_EINVAL;
  if (n_experts > kMaxExperts) return SPES_ESHAPE;
  if (spes_warmup_scratch_bytes(n_experts, elems_in) > kStaticScratchBytes) return SPES_ESHAPE;
  void* scratch = nullptr;
  SPES_TRY(static_scratch(&scratch));
  return spes_expert_warmup_merge(n_experts, dtype, top_K, alpha, w_in, elems_in, n_mats, src, dst, elems, sim, nbr, scratch,
                                  stream);
}

SPES_API int spes_ref_mfma_rate(const void* data, int32_t blocks, int32_t iters, float* sink, double* flop, void* stream) {
  if (!data || !sink || blocks <= 0 || iters <= 0 || blocks > (1 << 20)) return SPES_EINVAL;
  if (!aligned16(data) || !aligned16(sink)) return SPES_EALIGN;
  return launch_mfma_rate(data, blocks, iters, sink, flop, static_cast<hipStream_t>(stream));
}

SPES_API int spes_profile_enable(int32_t on) {
  if (on && !g_prof.created) {
    for (int w = 0; w < 2; ++w)
      for (int i = 0; i <= kMaxStages; ++i)
        if (hipEventCreate(&g_prof.ev[w][i]) != hipSuccess) return SPES_EHIP;
    g_prof.created = true;
  }
  g_prof.on = on != 0;
  g_prof.n[0] = g_prof.n[1] = 0;
  return SPES_OK;
}

SPES_API int spes_profile_read(int32_t which, float* ms, const char** names, int32_t cap) {
  if ((which != 0 && which != 1) || !ms || cap <= 0 || !g_prof.created) return SPES_EINVAL;
  const int n = g_prof.n[which] < cap ? g_prof.n[which] : cap;
  if (n == 0) return 0;
  if (hipEventSynchronize(g_prof.ev[which][g_prof.n[which]]) != hipSuccess) return SPES_EHIP;
  for (int i = 0; i < n; ++i) {
    if (hipEventElapsedTime(&ms[i], g_prof.ev[which][i], g_prof.ev[which][i + 1]) != hipSuccess) return SPES_EHIP;
    if (names) names[i] = g_prof.name[which][i];
  }
  return n;
}

SPES_API const char* spes_strerror(int code) {
  switch (code) {
    case SPES_OK: return "ok";
    case SPES_EINVAL: return "invalid argument (null pointer, non-positive size, top_k > n_experts or unknown dtype)";
    case SPES_ESHAPE: return "unsupported shape (n_experts > 64, a feature size not a multiple of 8, or too many rows/trainers)";
    case SPES_EALIGN: return "device pointer not 16-byte aligned";
    case SPES_EHIP: return "HIP kernel launch failed";
    default: return "unknown error";
  }
}

}  // extern "C"
