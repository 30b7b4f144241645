// Gate-weighted combine of the expert outputs (paper Eq. 2) and its backward.
// One wavefront per token; rows move in 16-byte chunks; sums are taken in float in slot order.
#include "kernels.h"

namespace unipool {

namespace {

template <typename TA> struct Vec;   // elements per 16-byte chunk
template <> struct Vec<float> { static constexpr int n = 4; };
template <> struct Vec<bf16> { static constexpr int n = 8; };

template <typename TA, int N>
__device__ __forceinline__ void load_chunk(const TA* p, float (&v)[N]) {
    const uint4 raw = *reinterpret_cast<const uint4*>(p);
    const TA* e = reinterpret_cast<const TA*>(&raw);
#pragma unroll
    for (int i = 0; i < N; i++) v[i] = to_f32(e[i]);
}

template <typename TA, int N>
__device__ __forceinline__ void store_chunk(TA* p, const float (&v)[N]) {
    uint4 raw;
    TA* e = reinterpret_cast<TA*>(&raw);
#pragma unroll
    for (int i = 0; i < N; i++) e[i] = from_f32<TA>(v[i]);
    *reinterpret_cast<uint4*>(p) = raw;
}

// K = top-k as a compile-time constant: the loops over the k copies of a token unroll, so the rows of the
// copies sit in registers and their k loads per chunk are in flight together (with k as a run-time bound
// the loads of the copies go out one after the other, each waiting for the one before).
template <typename TA, int K>
__global__ __launch_bounds__(256) void combine_kernel(const TA* __restrict__ y_perm,
                                                      const int32_t* __restrict__ row_of_slot,
                                                      const float* __restrict__ gate, int T, int d,
                                                      TA* __restrict__ out) {
    constexpr int N = Vec<TA>::n;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[K];
    float g[K];
#pragma unroll
    for (int j = 0; j < K; j++) {
        rows[j] = row_of_slot[(size_t)t * K + j];
        g[j] = gate ? gate[(size_t)t * K + j] : 1.0f;
    }
    const int chunks = (d % N == 0) ? d / N : 0;   // misaligned rows take the scalar path
    for (int c = lane; c < chunks; c += 64) {
        float v[K][N];
#pragma unroll
        for (int j = 0; j < K; j++) load_chunk<TA, N>(y_perm + (size_t)rows[j] * d + (size_t)c * N, v[j]);
        float acc[N];
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < K; j++)
#pragma unroll
            for (int i = 0; i < N; i++) acc[i] += g[j] * v[j][i];
        store_chunk<TA, N>(out + (size_t)t * d + (size_t)c * N, acc);
    }
    // tail elements when d is not a multiple of the chunk width
    for (int c = chunks * N + lane; c < d; c += 64) {
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < K; j++) acc += g[j] * to_f32(y_perm[(size_t)rows[j] * d + c]);
        out[(size_t)t * d + c] = from_f32<TA>(acc);
    }
}

template <typename TA, int K>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const TA* __restrict__ dout, const TA* __restrict__ y_perm,
    const int32_t* __restrict__ row_of_slot, const float* __restrict__ gate, int T, int d,
    TA* __restrict__ dy_perm, float* __restrict__ dgate) {
    constexpr int N = Vec<TA>::n;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int chunks = (d % N == 0) ? d / N : 0;   // misaligned rows take the scalar path
    int rows[K];
    float g[K], dot[K];
#pragma unroll
    for (int j = 0; j < K; j++) {
        rows[j] = row_of_slot[(size_t)t * K + j];
        g[j] = gate[(size_t)t * K + j];
        dot[j] = 0.f;
    }
    // a chunk of the token's dout row is read once and meets the same chunk of all k expert outputs
    for (int c = lane; c < chunks; c += 64) {
        float dv[N], yv[K][N];
        load_chunk<TA, N>(dout + (size_t)t * d + (size_t)c * N, dv);
#pragma unroll
        for (int j = 0; j < K; j++) load_chunk<TA, N>(y_perm + (size_t)rows[j] * d + (size_t)c * N, yv[j]);
#pragma unroll
        for (int j = 0; j < K; j++) {
            float o[N];
#pragma unroll
            for (int i = 0; i < N; i++) {
                dot[j] += dv[i] * yv[j][i];
                o[i] = g[j] * dv[i];
            }
            store_chunk<TA, N>(dy_perm + (size_t)rows[j] * d + (size_t)c * N, o);
        }
    }
    for (int c = chunks * N + lane; c < d; c += 64) {
        const float dv = to_f32(dout[(size_t)t * d + c]);
#pragma unroll
        for (int j = 0; j < K; j++) {
            dot[j] += dv * to_f32(y_perm[(size_t)rows[j] * d + c]);
            dy_perm[(size_t)rows[j] * d + c] = from_f32<TA>(g[j] * dv);
        }
    }
#pragma unroll
    for (int j = 0; j < K; j++) {
        const float s = wave_sum(dot[j]);
        if (lane == 0) dgate[(size_t)t * K + j] = s;
    }
}

}  // namespace

hipError_t launch_combine(const unipool_shape& s, const void* y_perm, const int32_t* row_of_slot,
                          const float* gate, void* out, hipStream_t st) {
    const int nblocks = cdiv(s.T, 4);
    with_top_k(s.k, [&](auto kc) {
        constexpr int K = decltype(kc)::value;
        if (s.dtype == UNIPOOL_BF16)
            combine_kernel<bf16, K><<<nblocks, 256, 0, st>>>((const bf16*)y_perm, row_of_slot, gate, s.T, s.d_model,
                                                             (bf16*)out);
        else
            combine_kernel<float, K><<<nblocks, 256, 0, st>>>((const float*)y_perm, row_of_slot, gate, s.T, s.d_model,
                                                              (float*)out);
    });
    return hipGetLastError();
}

hipError_t launch_combine_bwd(const unipool_shape& s, const void* dout, const void* y_perm,
                              const int32_t* row_of_slot, const float* gate, void* dy_perm,
                              float* dgate, hipStream_t st) {
    const int nblocks = cdiv(s.T, 4);
    with_top_k(s.k, [&](auto kc) {
        constexpr int K = decltype(kc)::value;
        if (s.dtype == UNIPOOL_BF16)
            combine_bwd_kernel<bf16, K><<<nblocks, 256, 0, st>>>((const bf16*)dout, (const bf16*)y_perm, row_of_slot,
                                                                 gate, s.T, s.d_model, (bf16*)dy_perm, dgate);
        else
            combine_bwd_kernel<float, K><<<nblocks, 256, 0, st>>>((const float*)dout, (const float*)y_perm,
                                                                  row_of_slot, gate, s.T, s.d_model,
                                                                  (float*)dy_perm, dgate);
    });
    return hipGetLastError();
}

}  // namespace unipool
