// Host-side launchers of the HIP kernels.  Each returns a hipError_t from the launch.
#pragma once

#include "common.h"

namespace unipool {

// ---- router.hip -------------------------------------------------------------------
// Per-token NormRouter score, top-k, gates and block-partial statistics from logits.
hipError_t launch_route_score_topk(const unipool_shape& s, const float* logits, int32_t* topk_idx,
                                   float* topk_gate, int32_t* counts, float* psum,
                                   int32_t* cnt_part, float* psum_part, hipStream_t st);
// Per-token backward of the score: writes dz (act dtype) and d_sigma.
hipError_t launch_route_finalize(const unipool_shape& s, const int32_t* cnt_part, const float* psum_part,
                                 int32_t* counts, float* psum, hipStream_t st);
hipError_t launch_route_bwd_dz(const unipool_shape& s, const float* logits, const int32_t* topk_idx,
                               const float* dgate, const float* aux_coef, void* dz,
                               float* dsigma_part, float* d_sigma, hipStream_t st);

// ---- permute.hip ------------------------------------------------------------------
hipError_t launch_permute(const unipool_shape& s, const void* x, const int32_t* topk_idx,
                          const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                          int32_t* row_of_slot, int32_t* slot_of_row, int32_t* chunk_hist,
                          hipStream_t st);

// ---- combine.hip ------------------------------------------------------------------
hipError_t launch_combine(const unipool_shape& s, const void* y_perm, const int32_t* row_of_slot,
                          const float* gate, void* out, hipStream_t st);
hipError_t launch_combine_bwd(const unipool_shape& s, const void* dout, const void* y_perm,
                              const int32_t* row_of_slot, const float* gate, void* dy_perm,
                              float* dgate, hipStream_t st);

// ---- aux_loss.hip -----------------------------------------------------------------
hipError_t launch_pool_aux_loss(const unipool_shape& s, const int32_t* counts, const float* psum,
                                const float* fbar_in, int32_t* pool_counts, float* fbar_out,
                                float* loss, float* aux_coef, hipStream_t st);

// ---- analysis.hip -----------------------------------------------------------------
int c_blocks(int n);     // partial sums the c estimate needs for n draws
hipError_t launch_estimate_c(int E, int k, const float* samples, int n, float* part_sum,
                             int32_t* part_used, float* c_out, int32_t* used_out, hipStream_t st);
hipError_t launch_distinct_experts(const int32_t* const* idx_layers, int L, int T, int k,
                                   int32_t* distinct, int32_t* part_sum, float* mean_out, hipStream_t st);

// ---- router_fused.hip: logits on the matrix cores, scores, top-k and block statistics in one kernel -----
bool router_fused_supported(const unipool_shape& s);
hipError_t router_fused(const unipool_shape& s, const void* x, const void* w, float* z, int32_t* topk_idx,
                        float* topk_gate, int32_t* cnt_part, float* psum_part, hipStream_t st);

// ---- gemm_naive.hip: one thread per output element; any shape, both dtypes ---------
hipError_t naive_logits(const unipool_shape& s, const void* x, const void* w, float* z, hipStream_t st);
// slot_of_row != nullptr: x_perm is the un-permuted x and row r reads token slot_of_row[r] / k of it
hipError_t naive_ffn_fwd(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                         const void* wgu, const void* wd, void* a, void* b, void* h, void* y,
                         hipStream_t st, const int32_t* slot_of_row = nullptr);
hipError_t naive_ffn_gate_up(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                            const void* wgu, void* a, void* b, void* h, hipStream_t st,
                            const int32_t* slot_of_row = nullptr);
hipError_t naive_ffn_dgrad(const unipool_shape& s, const void* dy, const void* a, const void* b,
                           const int32_t* offsets, const void* wgu, const void* wd, void* dx,
                           void* d_act, hipStream_t st);
hipError_t naive_ffn_wgrad(const unipool_shape& s, int n_layers, const void* const* x_perm_l,
                           const void* const* d_act_l, const void* const* h_l,
                           const void* const* dy_l, const int32_t* const* offsets_l,
                           float* dwgu, float* dwd, int accumulate, hipStream_t st);
hipError_t naive_route_bwd_mm(const unipool_shape& s, const void* x, const void* w, const void* dz,
                              float* dw, void* dx, int dx_accumulate, hipStream_t st);

// ---- gemm_mfma.hip: bf16 MFMA grouped GEMMs -----------------------------------------
bool mfma_ffn_supported(const unipool_shape& s);
bool mfma_router_supported(const unipool_shape& s);
hipError_t mfma_logits(const unipool_shape& s, const void* x, const void* w, float* z,
                       int32_t* tile_meta, hipStream_t st);
hipError_t mfma_ffn_fwd(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                        const void* wgu, const void* wd, void* a, void* b, void* h, void* y,
                        int32_t* tile_meta, hipStream_t st, const int32_t* slot_of_row = nullptr);
hipError_t mfma_ffn_gate_up(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                           const void* wgu, void* a, void* b, void* h, int32_t* tile_meta,
                           hipStream_t st, const int32_t* slot_of_row = nullptr);
hipError_t mfma_ffn_dgrad(const unipool_shape& s, const void* dy, const void* a, const void* b,
                          const int32_t* offsets, const void* wgu, const void* wd, void* dx,
                          void* d_act, int32_t* tile_meta, hipStream_t st);
hipError_t mfma_ffn_wgrad(const unipool_shape& s, int n_layers, const void* const* x_perm_l,
                          const void* const* d_act_l, const void* const* h_l,
                          const void* const* dy_l, const int32_t* const* offsets_l,
                          float* dwgu, float* dwd, int accumulate, const void* zeros,
                          hipStream_t st);
hipError_t mfma_route_bwd_mm(const unipool_shape& s, const void* x, const void* w, const void* dz,
                             float* dw, void* dx, int dx_accumulate, int32_t* tile_meta,
                             float* wpart, const void* zeros, hipStream_t st);

// ---- small utilities (api.hip) ---------------------------------------------------------
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_set_ptrs(void** table, const void* p0, const void* p1, const void* p2,
                           const void* p3, const void* p4, hipStream_t st);

}  // namespace unipool
