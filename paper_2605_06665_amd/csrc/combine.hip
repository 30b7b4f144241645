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

template <typename TA>
__global__ __launch_bounds__(256) void combine_kernel(const TA* __restrict__ y_perm,
                                                      const int32_t* __restrict__ row_of_slot,
                                                      const float* __restrict__ gate, int T, int d,
                                                      int k, TA* __restrict__ out) {
    constexpr int N = Vec<TA>::n;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[kMaxK];
    float g[kMaxK];
    for (int j = 0; j < k; j++) {
        rows[j] = row_of_slot[(size_t)t * k + j];
        g[j] = gate ? gate[(size_t)t * k + j] : 1.0f;
    }
    const int chunks = (d % N == 0) ? d / N : 0;   // misaligned rows take the scalar path
    for (int c = lane; c < chunks; c += 64) {
        float acc[N];
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = 0.f;
        for (int j = 0; j < k; j++) {
            float v[N];
            load_chunk<TA, N>(y_perm + (size_t)rows[j] * d + (size_t)c * N, v);
#pragma unroll
            for (int i = 0; i < N; i++) acc[i] += g[j] * v[i];
        }
        store_chunk<TA, N>(out + (size_t)t * d + (size_t)c * N, acc);
    }
    // tail elements when d is not a multiple of the chunk width
    for (int c = chunks * N + lane; c < d; c += 64) {
        float acc = 0.f;
        for (int j = 0; j < k; j++) acc += g[j] * to_f32(y_perm[(size_t)rows[j] * d + c]);
        out[(size_t)t * d + c] = from_f32<TA>(acc);
    }
}

template <typename TA>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const TA* __restrict__ dout, const TA* __restrict__ y_perm,
    const int32_t* __restrict__ row_of_slot, const float* __restrict__ gate, int T, int d, int k,
    TA* __restrict__ dy_perm, float* __restrict__ dgate) {
    constexpr int N = Vec<TA>::n;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int chunks = (d % N == 0) ? d / N : 0;   // misaligned rows take the scalar path
    for (int j = 0; j < k; j++) {
        const int row = row_of_slot[(size_t)t * k + j];
        const float g = gate[(size_t)t * k + j];
        float dot = 0.f;
        for (int c = lane; c < chunks; c += 64) {
            float dv[N], yv[N], o[N];
            load_chunk<TA, N>(dout + (size_t)t * d + (size_t)c * N, dv);
            load_chunk<TA, N>(y_perm + (size_t)row * d + (size_t)c * N, yv);
#pragma unroll
            for (int i = 0; i < N; i++) {
                dot += dv[i] * yv[i];
                o[i] = g * dv[i];
            }
            store_chunk<TA, N>(dy_perm + (size_t)row * d + (size_t)c * N, o);
        }
        for (int c = chunks * N + lane; c < d; c += 64) {
            const float dv = to_f32(dout[(size_t)t * d + c]);
            dot += dv * to_f32(y_perm[(size_t)row * d + c]);
            dy_perm[(size_t)row * d + c] = from_f32<TA>(g * dv);
        }
        dot = wave_sum(dot);
        if (lane == 0) dgate[(size_t)t * k + j] = dot;
    }
}

}  // namespace

hipError_t launch_combine(const unipool_shape& s, const void* y_perm, const int32_t* row_of_slot,
                          const float* gate, void* out, hipStream_t st) {
    const int nblocks = cdiv(s.T, 4);
    if (s.dtype == UNIPOOL_BF16)
        combine_kernel<bf16><<<nblocks, 256, 0, st>>>((const bf16*)y_perm, row_of_slot, gate, s.T,
                                                      s.d_model, s.k, (bf16*)out);
    else
        combine_kernel<float><<<nblocks, 256, 0, st>>>((const float*)y_perm, row_of_slot, gate, s.T,
                                                       s.d_model, s.k, (float*)out);
    return hipGetLastError();
}

hipError_t launch_combine_bwd(const unipool_shape& s, const void* dout, const void* y_perm,
                              const int32_t* row_of_slot, const float* gate, void* dy_perm,
                              float* dgate, hipStream_t st) {
    const int nblocks = cdiv(s.T, 4);
    if (s.dtype == UNIPOOL_BF16)
        combine_bwd_kernel<bf16><<<nblocks, 256, 0, st>>>((const bf16*)dout, (const bf16*)y_perm,
                                                          row_of_slot, gate, s.T, s.d_model, s.k,
                                                          (bf16*)dy_perm, dgate);
    else
        combine_bwd_kernel<float><<<nblocks, 256, 0, st>>>((const float*)dout, (const float*)y_perm,
                                                           row_of_slot, gate, s.T, s.d_model, s.k,
                                                           (float*)dy_perm, dgate);
    return hipGetLastError();
}

}  // namespace unipool
