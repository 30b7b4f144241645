// Plain contractions, one thread per output element.  They serve float mode (whose
// configurations are tiny) and bfloat16 shapes the MFMA kernels do not cover.  Sums run in
// float in index order.
#include "kernels.h"

namespace unipool {

namespace {

__device__ __forceinline__ int expert_of_row(const int32_t* offsets, int E, int row) {
    int lo = 0, hi = E;                      // offsets[lo] <= row < offsets[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] <= row) lo = mid; else hi = mid;
    }
    return lo;
}

template <typename TA>
__global__ void logits_kernel(const TA* __restrict__ x, const TA* __restrict__ w, int T, int d,
                              int E, float* __restrict__ z) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)T * E) return;
    const int t = (int)(id / E), e = (int)(id % E);
    float acc = 0.f;
    for (int c = 0; c < d; c++) acc += to_f32(x[(size_t)t * d + c]) * to_f32(w[(size_t)e * d + c]);
    z[id] = acc;
}

template <typename TA>
__global__ void gate_up_kernel(const TA* __restrict__ xp, const int32_t* __restrict__ offsets,
                               const TA* __restrict__ wgu, int S, int d, int f, int E,
                               TA* __restrict__ a, TA* __restrict__ b, TA* __restrict__ h,
                               const int32_t* __restrict__ slot_of_row, int k) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)S * f) return;
    const int row = (int)(id / f), n = (int)(id % f);
    const int e = expert_of_row(offsets, E, row);
    const TA* wg = wgu + ((size_t)e * 2 * f + n) * d;
    const TA* wu = wgu + ((size_t)e * 2 * f + f + n) * d;
    // gathered dispatch: row r of the group order is token slot_of_row[r] / k of the un-permuted input
    const size_t xrow = slot_of_row ? (size_t)(slot_of_row[row] / k) : (size_t)row;
    float av = 0.f, bv = 0.f;
    for (int c = 0; c < d; c++) {
        const float xv = to_f32(xp[xrow * d + c]);
        av += xv * to_f32(wg[c]);
        bv += xv * to_f32(wu[c]);
    }
    a[id] = from_f32<TA>(av);
    b[id] = from_f32<TA>(bv);
    h[id] = from_f32<TA>(silu_f(av) * bv);
}

template <typename TA>
__global__ void down_kernel(const TA* __restrict__ h, const int32_t* __restrict__ offsets,
                            const TA* __restrict__ wd, int S, int d, int f, int E,
                            TA* __restrict__ y) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)S * d) return;
    const int row = (int)(id / d), c = (int)(id % d);
    const int e = expert_of_row(offsets, E, row);
    const TA* w = wd + ((size_t)e * d + c) * f;
    float acc = 0.f;
    for (int n = 0; n < f; n++) acc += to_f32(h[(size_t)row * f + n]) * to_f32(w[n]);
    y[id] = from_f32<TA>(acc);
}

template <typename TA>
__global__ void dh_kernel(const TA* __restrict__ dy, const TA* __restrict__ a,
                          const TA* __restrict__ b, const int32_t* __restrict__ offsets,
                          const TA* __restrict__ wd, int S, int d, int f, int E,
                          TA* __restrict__ d_act) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)S * f) return;
    const int row = (int)(id / f), n = (int)(id % f);
    const int e = expert_of_row(offsets, E, row);
    float dh = 0.f;
    for (int c = 0; c < d; c++)
        dh += to_f32(dy[(size_t)row * d + c]) * to_f32(wd[((size_t)e * d + c) * f + n]);
    const float av = to_f32(a[id]), bv = to_f32(b[id]);
    const float sg = logistic_f(av);
    d_act[(size_t)row * 2 * f + n] = from_f32<TA>(dh * bv * sg * (1.0f + av * (1.0f - sg)));
    d_act[(size_t)row * 2 * f + f + n] = from_f32<TA>(dh * av * sg);
}

template <typename TA>
__global__ void dx_kernel(const TA* __restrict__ d_act, const int32_t* __restrict__ offsets,
                          const TA* __restrict__ wgu, int S, int d, int f, int E,
                          TA* __restrict__ dx) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)S * d) return;
    const int row = (int)(id / d), c = (int)(id % d);
    const int e = expert_of_row(offsets, E, row);
    float acc = 0.f;
    for (int n = 0; n < 2 * f; n++)
        acc += to_f32(d_act[(size_t)row * 2 * f + n]) * to_f32(wgu[((size_t)e * 2 * f + n) * d + c]);
    dx[id] = from_f32<TA>(acc);
}

// out[e][i][j] (+)= sum over layers and over the rows of e:  P[row][i] * Q[row][j]
template <typename TA>
__global__ void ptq_kernel(int n_layers, const void* const* __restrict__ p_l,
                           const void* const* __restrict__ q_l,
                           const int32_t* const* __restrict__ off_l, int E, int mdim, int ndim,
                           int accumulate, float* __restrict__ out) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)E * mdim * ndim) return;
    const int e = (int)(id / ((size_t)mdim * ndim));
    const int i = (int)((id / ndim) % mdim), j = (int)(id % ndim);
    float acc = 0.f;
    int rows = 0;
    for (int l = 0; l < n_layers; l++) {
        const TA* p = (const TA*)p_l[l];
        const TA* q = (const TA*)q_l[l];
        const int r0 = off_l[l][e], r1 = off_l[l][e + 1];
        rows += r1 - r0;
        for (int r = r0; r < r1; r++)
            acc += to_f32(p[(size_t)r * mdim + i]) * to_f32(q[(size_t)r * ndim + j]);
    }
    if (accumulate) {
        if (rows > 0) out[id] += acc;
    } else {
        out[id] = acc;
    }
}

template <typename TA>
__global__ void route_dw_kernel(const TA* __restrict__ dz, const TA* __restrict__ x, int T, int d,
                                int E, float* __restrict__ dw) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)E * d) return;
    const int e = (int)(id / d), c = (int)(id % d);
    float acc = 0.f;
    for (int t = 0; t < T; t++) acc += to_f32(dz[(size_t)t * E + e]) * to_f32(x[(size_t)t * d + c]);
    dw[id] = acc;
}

template <typename TA>
__global__ void route_dx_kernel(const TA* __restrict__ dz, const TA* __restrict__ w, int T, int d,
                                int E, int accumulate, TA* __restrict__ dx) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)T * d) return;
    const int t = (int)(id / d), c = (int)(id % d);
    float acc = accumulate ? to_f32(dx[id]) : 0.f;
    for (int e = 0; e < E; e++) acc += to_f32(dz[(size_t)t * E + e]) * to_f32(w[(size_t)e * d + c]);
    dx[id] = from_f32<TA>(acc);
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

}  // namespace

#define DISPATCH(TA_EXPR)                                   \
    if (s.dtype == UNIPOOL_BF16) { typedef bf16 TA; TA_EXPR; } \
    else { typedef float TA; TA_EXPR; }

hipError_t naive_logits(const unipool_shape& s, const void* x, const void* w, float* z, hipStream_t st) {
    DISPATCH((logits_kernel<TA><<<blocks_for((size_t)s.T * s.E), 256, 0, st>>>(
        (const TA*)x, (const TA*)w, s.T, s.d_model, s.E, z)));
    return hipGetLastError();
}

hipError_t naive_ffn_fwd(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                         const void* wgu, const void* wd, void* a, void* b, void* h, void* y,
                         hipStream_t st, const int32_t* slot_of_row) {
    const int S = s.T * s.k;
    DISPATCH((gate_up_kernel<TA><<<blocks_for((size_t)S * s.d_ff), 256, 0, st>>>(
        (const TA*)x_perm, offsets, (const TA*)wgu, S, s.d_model, s.d_ff, s.E, (TA*)a, (TA*)b, (TA*)h, slot_of_row, s.k)));
    DISPATCH((down_kernel<TA><<<blocks_for((size_t)S * s.d_model), 256, 0, st>>>(
        (const TA*)h, offsets, (const TA*)wd, S, s.d_model, s.d_ff, s.E, (TA*)y)));
    return hipGetLastError();
}

hipError_t naive_ffn_gate_up(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                            const void* wgu, void* a, void* b, void* h, hipStream_t st,
                            const int32_t* slot_of_row) {
    const int S = s.T * s.k;
    DISPATCH((gate_up_kernel<TA><<<blocks_for((size_t)S * s.d_ff), 256, 0, st>>>(
        (const TA*)x_perm, offsets, (const TA*)wgu, S, s.d_model, s.d_ff, s.E, (TA*)a, (TA*)b, (TA*)h, slot_of_row, s.k)));
    return hipGetLastError();
}

hipError_t naive_ffn_dgrad(const unipool_shape& s, const void* dy, const void* a, const void* b,
                           const int32_t* offsets, const void* wgu, const void* wd, void* dx,
                           void* d_act, hipStream_t st) {
    const int S = s.T * s.k;
    DISPATCH((dh_kernel<TA><<<blocks_for((size_t)S * s.d_ff), 256, 0, st>>>(
        (const TA*)dy, (const TA*)a, (const TA*)b, offsets, (const TA*)wd, S, s.d_model, s.d_ff, s.E,
        (TA*)d_act)));
    DISPATCH((dx_kernel<TA><<<blocks_for((size_t)S * s.d_model), 256, 0, st>>>(
        (const TA*)d_act, offsets, (const TA*)wgu, S, s.d_model, s.d_ff, s.E, (TA*)dx)));
    return hipGetLastError();
}

hipError_t naive_ffn_wgrad(const unipool_shape& s, int n_layers, const void* const* x_perm_l,
                           const void* const* d_act_l, const void* const* h_l,
                           const void* const* dy_l, const int32_t* const* offsets_l,
                           float* dwgu, float* dwd, int accumulate, hipStream_t st) {
    // d_w_gate_up[e][n][c] = sum d_act[row][n] x_perm[row][c];  d_w_down[e][c][n] = sum dy[row][c] h[row][n]
    DISPATCH((ptq_kernel<TA><<<blocks_for((size_t)s.E * 2 * s.d_ff * s.d_model), 256, 0, st>>>(
        n_layers, d_act_l, x_perm_l, offsets_l, s.E, 2 * s.d_ff, s.d_model, accumulate, dwgu)));
    DISPATCH((ptq_kernel<TA><<<blocks_for((size_t)s.E * s.d_model * s.d_ff), 256, 0, st>>>(
        n_layers, dy_l, h_l, offsets_l, s.E, s.d_model, s.d_ff, accumulate, dwd)));
    return hipGetLastError();
}

hipError_t naive_route_bwd_mm(const unipool_shape& s, const void* x, const void* w, const void* dz,
                              float* dw, void* dx, int dx_accumulate, hipStream_t st) {
    DISPATCH((route_dw_kernel<TA><<<blocks_for((size_t)s.E * s.d_model), 256, 0, st>>>(
        (const TA*)dz, (const TA*)x, s.T, s.d_model, s.E, dw)));
    DISPATCH((route_dx_kernel<TA><<<blocks_for((size_t)s.T * s.d_model), 256, 0, st>>>(
        (const TA*)dz, (const TA*)w, s.T, s.d_model, s.E, dx_accumulate, (TA*)dx)));
    return hipGetLastError();
}

}  // namespace unipool
