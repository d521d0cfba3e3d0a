// Host-side launchers of every kernel in the library (one translation unit each).
#pragma once
#include "common.h"
#include "gemm.h"

namespace spes {

// routing.hip
int routing_blocks(int R);
int launch_topk_gate(float* logits, int n_part, const float* bias, int T, int M, int k, int renorm, int* idx, float* gate,
                     int* idx_copy, float* gate_copy, float* lse, hipStream_t s);
int launch_routing_tables(const int* idx, const float* gate, int R, int M, int k, int* block_counts, int* expert_count,
                          int* offset, int* perm, int* inv, int* row_token, float* row_gate, int bm0, int* tab0, int bm1,
                          int* tab1, int max_tiles, float* aux, hipStream_t s);
int launch_gating_bwd(const float* logits, const float* lse, const int* idx, const float* gate, const float* dgate_part,
                      int n_part, long part_stride, const int* inv, float* dgate, int T, int M, int k, int renorm, const float* aux,
                      float* dlogits, bf16_t* dlogits_bf, hipStream_t s);
// losses[0] = load-balancing loss, losses[1] = router z-loss; aux = the gradient factors read by launch_gating_bwd
int launch_router_aux(const float* logits, const float* lse, const int* offset, int T, int M, int k, float lb_coef, float z_coef,
                      float grad_scale, float* part, float* losses, float* aux, hipStream_t s);

// movement.hip (dtype = spes_dtype of the storage type)
int launch_permute(int dtype, const void* x, const int* inv, int k, void* xp, int T, int d, hipStream_t s);
int launch_combine(int dtype, const void* yp, const int* inv, const float* gate, void* y, int T, int d, int k, hipStream_t s);
int launch_dx_gather(int dtype, const void* dxp, const int* inv, const float* dlogits, const void* w_router, const void* dxr,
                     void* dx, int T, int d, int k, int M, hipStream_t s);

// dyp[inv[t*k+j],:] = gate[t,j] * dy[t,:], dgate[t,j] = <dy[t,:], yp[inv[t*k+j],:]> (movement.hip)
int launch_grad_scatter(int dtype, const void* dy, const void* yp, const int* inv, const float* gate, void* dyp, float* dgate,
                        int T, int d, int k, hipStream_t s);

// out[i] (+)= sum_p partial[p*n + i], p ascending (movement.hip)
int launch_reduce_partials(const float* partial, int n_partial, long n, float* out, int accumulate, hipStream_t s);

// merge.hip
int launch_sync_merge(int dtype, int n_experts, long elems, int n_nodes, const void* const* node_store, const int* slot,
                      const float* node_weight, void* dst, int* trainer_count, hipStream_t s);
int launch_gram_bf16(const void* w, int M, long elems, int n_groups, long kchunk, float* partial, hipStream_t s);
int launch_sim_topk(float* partial, int n_partial, int M, int K, float* sim, int* nbr, hipStream_t s);
int launch_warmup_mix(int dtype, int M, long elems, int K, float alpha, const void* src, void* dst, const int* nbr, hipStream_t s);

// optim.hip: AdamW on the experts whose mask byte is set; compact fp32 state, one slot per such expert in ascending id
int launch_masked_adamw(int dtype, int n_experts, long elems, void* param, const unsigned char* mask, float* master, float* m,
                        float* v, const float* grad, float lr, float beta1, float beta2, float eps, float wd, int step,
                        float grad_scale, hipStream_t s);

// upcycle.hip: out[e] = dense + noise on the selected share of the elements (thr = selected 256ths); gather / scatter
// of the rows of the experts whose mask byte is set between the full store and a contiguous buffer
int launch_upcycle_init(int dtype, int n_experts, long elems, const void* dense, unsigned thr, float sigma,
                        unsigned long long seed, unsigned long long stream_id, void* out, hipStream_t s);
int launch_expert_pack(int dtype, int n_experts, long elems, void* store, const unsigned char* mask, void* packed, int to_store,
                       hipStream_t s);

// reference.hip: register-resident MFMA loop (blocks x 4 wavefronts x iters x 64 MFMAs of 16x16x32); *flop = operations launched
int launch_mfma_rate(const void* data, int blocks, int iters, float* sink, double* flop, hipStream_t s);

}  // namespace spes
