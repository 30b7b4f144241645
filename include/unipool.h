/*
 * unipool.h -- C ABI of the shared-pool Mixture-of-Experts layer (UniPool),
 * forward and backward, for one AMD MI355X (gfx950).
 *
 * The layer (paper Sec. 4.1, Eq. 2):  FFN_l(x) = sum_{i in Top-k(r_l(x))} g_{l,i}(x) e_i(x),
 * where the experts e_1..e_M form ONE pool shared by all L layers, every layer has
 * its own NormRouter r_l (Sec. 4.3, Eq. 7), and a pool-level auxiliary loss balances
 * expert usage summed over the layers (Sec. 4.2, Eq. 4-6; App. G (pool auxiliary loss derivation)).
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; tensors are
 *     row-major and contiguous, last index fastest.  The library allocates nothing
 *     and keeps no state: weights, gradients, counts and fbar belong to the caller.
 *   - Scratch memory comes from the caller's workspace `ws` (device pointer, at least
 *     unipool_workspace_bytes() bytes, 256-byte aligned).  Calls that share a
 *     workspace must be ordered on one stream.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  No call synchronises with the host or copies to it.
 *   - Every function returns 0 on success or a negative UNIPOOL_E* code.  Arguments
 *     are validated before anything is launched; on error nothing has been written.
 *     unipool_last_error() gives a message for the calling thread's last failure.
 *   - Same inputs give bitwise the same outputs (no floating-point atomics).
 *   - dtype UNIPOOL_F32: every floating tensor is float.
 *     dtype UNIPOOL_BF16: tensors marked "act" below are bfloat16; logits, scores,
 *     gates, statistics and all weight gradients are float; products accumulate in
 *     float.  In this mode d_model and d_ff must be multiples of 64.
 *   - Index tensors are int32.  S = T*k is the number of (token, slot) pairs.
 *   - Limits: 1 <= k <= 8, k <= E <= 512, T*k < 2^31, sigma > 0.
 *
 * Weight storage (Linear convention, [out_features, in_features]):
 *   w_router  [E, d_model]            z = W h                        (Sec. 4.3)
 *   w_gate_up [E, 2*d_ff, d_model]    rows [0, d_ff) of expert e are W_gate,e,
 *                                     rows [d_ff, 2 d_ff) are W_up,e
 *   w_down    [E, d_model, d_ff]      e(x) = W_down ( silu(W_gate x) * (W_up x) )
 * Weight gradients have the same shapes, in float.
 */
#ifndef UNIPOOL_H
#define UNIPOOL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define UNIPOOL_OK          0
#define UNIPOOL_EINVAL     -1   /* NULL/invalid argument, unsupported shape or alignment */
#define UNIPOOL_EWORKSPACE -2   /* workspace missing or too small */
#define UNIPOOL_ELAUNCH    -3   /* the HIP runtime reported an error */

#define UNIPOOL_F32  0
#define UNIPOOL_BF16 1

/* Router kinds.  NORM is the paper's NormRouter (Sec. 4.3, Eq. 7).  SOFTMAX is the router of the comparison
 * rows (Sec. 4.1, Eq. 1 and Sec. 4.2, Eq. 3; ablation "softmax router" of Sec. 5.4): score p_i = exp(z_i) / sum_j exp(z_j),
 * selection of the k largest logits as for NORM, gate = p of the selected expert (no renormalisation over the
 * top-k), and the auxiliary losses take p as the routing probability.  sigma, c and eps are not used. */
#define UNIPOOL_ROUTER_NORM    0
#define UNIPOOL_ROUTER_SOFTMAX 1

typedef struct unipool_shape {
    int32_t T;          /* tokens in this layer call */
    int32_t d_model;    /* d */
    int32_t d_ff;       /* f, hidden width of one expert */
    int32_t E;          /* pool size M */
    int32_t k;          /* experts per token */
    int32_t L;          /* layers sharing the pool (used by unipool_pool_aux_loss only) */
    int32_t dtype;      /* UNIPOOL_F32 or UNIPOOL_BF16 */
    float sigma;        /* NormRouter scale of THIS layer (learnable, init 1; Eq. 7) */
    float c;            /* NormRouter calibration constant (App. H (NormRouter Monte Carlo initialization)); a plain input */
    float eps;          /* NormRouter epsilon, added outside the norm (Eq. 7) */
    float alpha_pool;   /* pool auxiliary loss coefficient (Eq. 5) */
    int32_t router;     /* UNIPOOL_ROUTER_NORM or UNIPOOL_ROUTER_SOFTMAX (unipool_route, unipool_route_bwd) */
} unipool_shape;

/* Bytes of workspace that is enough for every entry point at this shape. */
size_t unipool_workspace_bytes(const unipool_shape* shape);

/* Message for the last error returned on the calling thread (never NULL). */
const char* unipool_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int unipool_version(void);

/*
 * Which kernels a shape gets.  In bfloat16 mode the contractions run on the matrix cores (MFMA); shapes those
 * kernels do not cover still give correct results, on plain one-thread-per-output kernels that are far slower:
 * the router logits and the router backward when E is not a multiple of 8, and everything in float mode.
 * Returns a bit mask: bit 0 the expert GEMMs use MFMA kernels, bit 1 the router contractions do, bit 2 the
 * router runs as one fused kernel (logits, scores, top-k, statistics: d_model a multiple of 128, E a multiple
 * of 8 and at most 512).  Negative on an invalid shape.
 */
#define UNIPOOL_FAST_EXPERTS      1
#define UNIPOOL_FAST_ROUTER       2
#define UNIPOOL_FAST_ROUTER_FUSED 4
int unipool_fast_path(const unipool_shape* shape);

/*
 * Router of one layer (Sec. 4.3, Eq. 7 and the top-k paragraph).
 *   z = x W^T (float accumulate);  n = ||z||_2;  s_i = sigma c max(0, z_i/(n+eps));
 *   topk_idx[t, :] = the k experts with the largest logits, in descending order,
 *   exact ties to the lower index;  topk_gate[t, j] = s_{t, topk_idx[t,j]} (raw score).
 *   counts[i] = number of (t, j) with topk_idx[t,j] == i;  psum[i] = sum_t s_{t,i} over
 *   ALL experts (the statistics f and P of Sec. 4.2 before normalisation).
 *   With shape->router == UNIPOOL_ROUTER_SOFTMAX the score is s_i = softmax(z)_i instead.
 * in : x [T, d] act;  w_router [E, d] act
 * out: topk_idx [T, k] int32;  topk_gate [T, k] float;  logits [T, E] float (saved
 *      for the backward pass; may be NULL);  counts [E] int32;  psum [E] float.
 * counts and psum are overwritten, not accumulated.
 */
int unipool_route(const unipool_shape* shape, const void* x, const void* w_router,
                  int32_t* topk_idx, float* topk_gate, float* logits,
                  int32_t* counts, float* psum,
                  void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the router (derivative of Eq. 7 and of z = W h; App. G (pool auxiliary loss derivation): the pool
 * loss reaches parameters only through the scores).
 *   ds_{t,i} = aux_coef[i] (all i; omitted if aux_coef is NULL) + dgate[t,j] for i = topk_idx[t,j]
 *   d_sigma  = sum_{t,i} ds_{t,i} c max(0, zhat_{t,i});  dzhat = ds sigma c [zhat > 0]
 *   dz_j     = dzhat_j/(n+eps) - z_j <dzhat, z> / (n (n+eps)^2)
 *   d_w_router = dz^T x;   dx += dz W  (dx_accumulate != 0) or dx = dz W.
 *   UNIPOOL_ROUTER_SOFTMAX:  dz_j = p_j (ds_j - <ds, p>),  d_sigma = 0.
 *   In bfloat16 mode dz is rounded to bfloat16 before the two products.
 * in : x, w_router as in unipool_route;  logits [T, E] float from unipool_route;
 *      topk_idx [T, k];  dgate [T, k] float;  aux_coef [E] float or NULL.
 * out: d_w_router [E, d] float (overwritten);  d_sigma [1] float (overwritten);
 *      dx [T, d] act (accumulated into or overwritten, see dx_accumulate).
 */
int unipool_route_bwd(const unipool_shape* shape, const void* x, const void* w_router,
                      const float* logits, const int32_t* topk_idx, const float* dgate,
                      const float* aux_coef, float* d_w_router, float* d_sigma,
                      void* dx, int dx_accumulate,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * Dispatch: expert-contiguous copy of the tokens (the grouping a grouped GEMM needs;
 * Table 7 only says that grouped GEMM is used, the row order is this library's).
 *   expert_offsets = exclusive prefix sum of counts, expert_offsets[E] = S;
 *   the rows of expert e are expert_offsets[e] .. expert_offsets[e+1]-1 and hold the
 *   tokens that selected e in ascending token order;
 *   row_of_slot[t, j] = row of token t for its j-th expert;  slot_of_row[row] = t*k + j;
 *   x_perm[row_of_slot[t,j], :] = x[t, :].
 * in : x [T, d] act;  topk_idx [T, k];  counts [E] (from unipool_route)
 * out: x_perm [S, d] act;  expert_offsets [E+1];  row_of_slot [T, k];  slot_of_row [S].
 * x_perm may be NULL (x is then not read): only the three index tensors are made, for a caller that
 * runs the experts on gathered rows (unipool_expert_ffn_fwd_gather).
 */
int unipool_permute(const unipool_shape* shape, const void* x, const int32_t* topk_idx,
                    const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                    int32_t* row_of_slot, int32_t* slot_of_row,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * unipool_permute for callers that cannot allocate or size a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same inputs, outputs, kernels and
 * results as unipool_permute, but the per-chunk histograms live in a static device array inside the
 * library (2 MiB per GPU, held until the process ends) instead of the caller's workspace.
 * Limit: ceil(T/64) * E <= 524288; larger shapes return UNIPOOL_EINVAL (use unipool_permute).
 * The call allocates nothing; its first call on a device looks up the array's device address.
 * All calls on one GPU share that array: calls that overlap on one GPU (different streams or
 * threads) race; order them on one stream.  Nothing of an earlier call is read by a later one.
 */
int unipool_permute_static(const unipool_shape* shape, const void* x, const int32_t* topk_idx,
                           const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                           int32_t* row_of_slot, int32_t* slot_of_row, void* stream);

/*
 * Pool experts on their row groups (Eq. 2's e_i; SwiGLU FFN, Table 6 caption).
 * For every expert e with rows R_e:  A = X_e W_gate,e^T;  B = X_e W_up,e^T;
 *   H = silu(A) * B;  Y = H W_down,e^T.   Experts without rows cost nothing.
 * in : x_perm [S, d] act;  expert_offsets [E+1];  w_gate_up, w_down (see top).
 * out: act_a, act_b, act_h [S, f] act (saved for the backward pass);  y_perm [S, d] act.
 */
int unipool_expert_ffn_fwd(const unipool_shape* shape, const void* x_perm,
                           const int32_t* expert_offsets, const void* w_gate_up,
                           const void* w_down, void* act_a, void* act_b, void* act_h,
                           void* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * unipool_expert_ffn_fwd with the dispatch fused into the first GEMM: the rows of expert e are read straight
 * from the un-permuted x through slot_of_row (row r of the group order is token slot_of_row[r] / k), so no
 * x_perm has to exist.  Meant for forward-only use; the weight gradient of the backward pass reads x_perm as
 * a materialised operand.  Results are bit-identical to unipool_expert_ffn_fwd on the permuted copy.
 * in : x [T, d] act;  slot_of_row [S], expert_offsets [E+1] (from unipool_permute);  weights as above.
 * out: act_a, act_b, act_h [S, f] act;  y_perm [S, d] act.
 */
int unipool_expert_ffn_fwd_gather(const unipool_shape* shape, const void* x, const int32_t* slot_of_row,
                                  const int32_t* expert_offsets, const void* w_gate_up, const void* w_down,
                                  void* act_a, void* act_b, void* act_h, void* y_perm,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * First half of unipool_expert_ffn_fwd alone, for training with activation recomputation
 * (App. D (hyperparameter details): activation checkpointing with MoE layer recompute): a caller that
 * did not keep A and B of a layer runs this before unipool_expert_ffn_bwd.  Same arithmetic as
 * in the forward pass, so the three tensors come out bit-identical to the forward's.
 * in : x_perm [S, d] act;  expert_offsets [E+1];  w_gate_up (see top).
 * out: act_a, act_b, act_h [S, f] act.
 */
int unipool_expert_ffn_recompute(const unipool_shape* shape, const void* x_perm,
                                 const int32_t* expert_offsets, const void* w_gate_up,
                                 void* act_a, void* act_b, void* act_h,
                                 void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the pool experts for one layer.
 *   dH = dY W_down;  dA = dH * B * silu'(A);  dB = dH * silu(A);
 *   dX_perm = dA W_gate + dB W_up;
 *   d_w_down[e]    += dY_e^T H_e;   d_w_gate_up[e] += [dA_e | dB_e]^T X_e.
 * The pool is shared: every layer adds into the same float gradient buffers, which
 * the caller zeroes once per step (Sec. 3: each expert gathers gradients of L layers).
 * Experts without rows leave their gradient untouched.
 * in : dy_perm [S, d] act;  x_perm, act_a, act_b, act_h, expert_offsets, weights as above.
 * out: dx_perm [S, d] act;  d_act [S, 2f] act = [dA | dB] (also scratch for the weight
 *      gradient);  d_w_gate_up [E, 2f, d] float and d_w_down [E, d, f] float, accumulated.
 *      d_w_gate_up and d_w_down may both be NULL: then only dx_perm and d_act are made
 *      (the weight gradient can be taken later by unipool_expert_wgrad).
 */
int unipool_expert_ffn_bwd(const unipool_shape* shape, const void* dy_perm, const void* x_perm,
                           const void* act_a, const void* act_b, const void* act_h,
                           const int32_t* expert_offsets, const void* w_gate_up,
                           const void* w_down, void* dx_perm, void* d_act,
                           float* d_w_gate_up, float* d_w_down,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Weight gradient of the pool for n_layers layer calls at once.  Because the pool is
 * shared, the rows an expert received in different layers extend one reduction:
 *   d_w_gate_up[e] (+)= sum_l [dA|dB]^(l)_e^T X^(l)_e;   d_w_down[e] (+)= sum_l dY^(l)_e^T H^(l)_e.
 * The result equals n_layers calls of unipool_expert_ffn_bwd's accumulation.
 * in : n_layers in [1, 256]; device arrays of n_layers device pointers each: x_perm_l, d_act_l, act_h_l,
 *      dy_perm_l (tensors as in unipool_expert_ffn_bwd) and expert_offsets_l ([E+1] each).
 * out: d_w_gate_up, d_w_down float; accumulate != 0 adds to them, 0 overwrites them
 *      (experts with no rows in any layer are then set to zero).
 */
int unipool_expert_wgrad(const unipool_shape* shape, int n_layers,
                         const void* const* x_perm_l, const void* const* d_act_l,
                         const void* const* act_h_l, const void* const* dy_perm_l,
                         const int32_t* const* expert_offsets_l,
                         float* d_w_gate_up, float* d_w_down, int accumulate,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * Gate-weighted combine (Eq. 2):  out[t] = sum_j gate[t,j] * y_perm[row_of_slot[t,j]],
 * summed in slot order with float accumulation.  gate == NULL means unit gates, which
 * is the backward of unipool_permute (dX[t] = sum_j dX_perm[row_of_slot[t,j]]).
 * in : y_perm [S, d] act;  row_of_slot [T, k];  gate [T, k] float or NULL
 * out: out [T, d] act.
 */
int unipool_combine(const unipool_shape* shape, const void* y_perm, const int32_t* row_of_slot,
                    const float* gate, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the combine:  dy_perm[row_of_slot[t,j]] = gate[t,j] * dout[t];
 *                           dgate[t,j] = <dout[t], y_perm[row_of_slot[t,j]]>.
 * in : dout [T, d] act;  y_perm [S, d] act;  row_of_slot [T, k];  gate [T, k] float
 * out: dy_perm [S, d] act;  dgate [T, k] float.
 */
int unipool_combine_bwd(const unipool_shape* shape, const void* dout, const void* y_perm,
                        const int32_t* row_of_slot, const float* gate, void* dy_perm,
                        float* dgate, void* ws, size_t ws_bytes, void* stream);

/*
 * Pool-level auxiliary loss over the L layers that share the pool (Sec. 4.2).
 *   pool_counts[i] = sum_l counts[l,i];   fbar_out[i] = pool_counts[i] / (L T k)   (Eq. 4)
 *   fbar = fbar_in if given (one-step-behind statistic of App. G (pool auxiliary loss derivation)) else fbar_out
 *   loss = alpha_pool M sum_i fbar_i Pbar_i,  Pbar_i = (1/(L T)) sum_l psum[l,i]   (Eq. 5)
 *   aux_coef[i] = alpha_pool M fbar_i / (L T)  = d loss / d s^(l)_{t,i}             (Eq. 6)
 * fbar is a constant for differentiation (App. G (pool auxiliary loss derivation)).
 * in : counts [L, E] int32;  psum [L, E] float;  fbar_in [E] float or NULL
 * out: pool_counts [E] int32;  fbar_out [E] float;  loss [1] float;  aux_coef [E] float.
 */
int unipool_pool_aux_loss(const unipool_shape* shape, const int32_t* counts, const float* psum,
                          const float* fbar_in, int32_t* pool_counts, float* fbar_out,
                          float* loss, float* aux_coef, void* ws, size_t ws_bytes, void* stream);

/*
 * Monte-Carlo estimate of the NormRouter calibration constant c (App. H (NormRouter Monte Carlo initialization), Alg. 1) from draws
 * the caller supplies: for every row x of samples, y = relu(x / ||x||_2), the k largest
 * components of y, 1 / their 2-norm; c is the mean over the rows.  A row without a positive
 * component has an all-zero top-k part and is left out (the paper does not treat 1/0);
 * samples_used tells how many rows entered.  Float arithmetic, fixed summation order
 * (bitwise repeatable); the final mean is taken in double.
 * in : samples [n_samples, E] float (device), meant to be N(0, 1) draws;  1 <= k <= min(8, E);
 *      E <= 512.
 * out: c_out [1] float;  samples_used [1] int32.
 * workspace: at least 2 * roundup256(4 * ceil(n_samples / 64)) bytes, 256-byte aligned.
 */
int unipool_estimate_c(int E, int k, const float* samples, int n_samples, float* c_out,
                       int32_t* samples_used, void* ws, size_t ws_bytes, void* stream);

/*
 * Distinct pool experts per token (App. E (distinct-expert accounting)): U(t) = number of different experts token t
 * selects over n_layers layers that route into one pool (all k selections of a layer count;
 * the paper states it for top-1), and its mean over the tokens.
 * in : topk_idx_l: device array of n_layers device pointers, each to a [T, k] int32 tensor
 *      (as written by unipool_route).
 * out: distinct [T] int32;  mean_distinct [1] float.
 */
int unipool_distinct_experts(const unipool_shape* shape, int n_layers, const void* const* topk_idx_l,
                             int32_t* distinct, float* mean_distinct,
                             void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* UNIPOOL_H */
