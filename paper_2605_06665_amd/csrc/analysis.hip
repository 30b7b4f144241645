// Analysis observables of the paper, on the device:
//   * Monte-Carlo estimate of the NormRouter constant c from given normal draws (App. H (NormRouter Monte Carlo initialization), Alg. 1);
//   * U(x), the number of distinct pool experts a token selects over the L layers (App. E (distinct-expert accounting)).
#include "kernels.h"

namespace unipool {

namespace {

constexpr int kCBlockRows = 64;       // draws per block: 4 wavefronts x 16 draws

// One group of GS lanes per draw, lane s holds components s, s + GS, ...  Per draw:
// y = relu(x / ||x||), the k largest components of y, 1 / their 2-norm.  Block partial sums leave
// in a fixed order; draws whose top-k part is all zero are dropped.
template <int GS, int VPL>
__global__ __launch_bounds__(256) void c_terms_kernel(const float* __restrict__ samples, int n, int E,
                                                      int k, float* __restrict__ part_sum,
                                                      int32_t* __restrict__ part_used) {
    constexpr int TPW = 64 / GS;
    __shared__ float lds_s[4];
    __shared__ int lds_u[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / GS, sl = lane % GS;
    float acc = 0.f;
    int used = 0;
    for (int tt = 0; tt < 16; tt += TPW) {
        const int r = blockIdx.x * kCBlockRows + wave * 16 + tt + grp;
        const float* xr = samples + (size_t)min(r, n - 1) * E;
        float x[VPL];
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            const int e = sl + GS * i;
            x[i] = e < E ? xr[e] : 0.f;
            ss += x[i] * x[i];
        }
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        const float inv = 1.0f / sqrtf(ss);
        unsigned taken = 0;
        float top2 = 0.f;                       // sum of squares of the k largest y
        for (int j = 0; j < k; j++) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < VPL; i++) {
                const int e = sl + GS * i;
                const bool ok = (e < E) && !((taken >> i) & 1u);
                if (ok && (x[i] > bv || bi == 0x7fffffff)) { bv = x[i]; bi = e; }
            }
#pragma unroll
            for (int o = GS / 2; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, 64);
                const int oi = __shfl_xor(bi, o, 64);
                const bool take = oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
                if (take) { bv = ov; bi = oi; }
            }
            if (bi != 0x7fffffff && bi % GS == sl) taken |= 1u << (bi / GS);
            const float y = fmaxf(bv * inv, 0.f);           // bv is -inf once the draw has no more components
            if (bi != 0x7fffffff) top2 += y * y;
        }
        if (sl == 0 && r < n && top2 > 0.f) {
            acc += 1.0f / sqrtf(top2);
            used += 1;
        }
    }
    // over the groups of a wavefront, then over the wavefronts, in a fixed order
#pragma unroll
    for (int o = GS; o < 64; o <<= 1) {
        acc += __shfl_xor(acc, o, 64);
        used += __shfl_xor(used, o, 64);
    }
    if (lane == 0) { lds_s[wave] = acc; lds_u[wave] = used; }
    __syncthreads();
    if (threadIdx.x == 0) {
        part_sum[blockIdx.x] = ((lds_s[0] + lds_s[1]) + lds_s[2]) + lds_s[3];
        part_used[blockIdx.x] = lds_u[0] + lds_u[1] + lds_u[2] + lds_u[3];
    }
}

__global__ __launch_bounds__(256) void c_finalize_kernel(const float* __restrict__ part_sum,
                                                         const int32_t* __restrict__ part_used, int nb,
                                                         float* __restrict__ c_out,
                                                         int32_t* __restrict__ used_out) {
    __shared__ double rs[256];
    __shared__ int ru[256];
    const int t = threadIdx.x;
    double s = 0.0;
    int u = 0;
    for (int i = t; i < nb; i += 256) { s += (double)part_sum[i]; u += part_used[i]; }
    rs[t] = s;
    ru[t] = u;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (t < w) { rs[t] += rs[t + w]; ru[t] += ru[t + w]; }
        __syncthreads();
    }
    if (t == 0) {
        used_out[0] = ru[0];
        c_out[0] = ru[0] > 0 ? (float)(rs[0] / (double)ru[0]) : 0.f;
    }
}

// One thread per token: a 512-bit set of the experts selected at any layer.
__global__ __launch_bounds__(256) void distinct_kernel(const int32_t* const* __restrict__ idx_layers, int L,
                                                       int T, int k, int32_t* __restrict__ distinct,
                                                       int32_t* __restrict__ part_sum) {
    __shared__ int red[256];
    const int t = blockIdx.x * 256 + threadIdx.x;
    int u = 0;
    if (t < T) {
        unsigned mask[kMaxE / 32];
#pragma unroll
        for (int w = 0; w < kMaxE / 32; w++) mask[w] = 0u;
        for (int l = 0; l < L; l++) {
            const int32_t* row = idx_layers[l] + (size_t)t * k;
            for (int j = 0; j < k; j++) {
                const int e = row[j];
#pragma unroll
                for (int w = 0; w < kMaxE / 32; w++)
                    if (w == (e >> 5)) mask[w] |= 1u << (e & 31);
            }
        }
#pragma unroll
        for (int w = 0; w < kMaxE / 32; w++) u += __popc(mask[w]);
        distinct[t] = u;
    }
    red[threadIdx.x] = u;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) part_sum[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(256) void distinct_finalize_kernel(const int32_t* __restrict__ part_sum, int nb,
                                                                int T, float* __restrict__ mean_out) {
    __shared__ long long red[256];
    const int t = threadIdx.x;
    long long s = 0;
    for (int i = t; i < nb; i += 256) s += part_sum[i];
    red[t] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    if (t == 0) mean_out[0] = (float)((double)red[0] / (double)T);
}

}  // namespace

int c_blocks(int n) { return cdiv(n, kCBlockRows); }

hipError_t launch_estimate_c(int E, int k, const float* samples, int n, float* part_sum,
                             int32_t* part_used, float* c_out, int32_t* used_out, hipStream_t st) {
    const int nb = c_blocks(n);
    if (E <= 128) c_terms_kernel<16, 8><<<nb, 256, 0, st>>>(samples, n, E, k, part_sum, part_used);
    else if (E <= 256) c_terms_kernel<16, 16><<<nb, 256, 0, st>>>(samples, n, E, k, part_sum, part_used);
    else c_terms_kernel<32, 16><<<nb, 256, 0, st>>>(samples, n, E, k, part_sum, part_used);
    c_finalize_kernel<<<1, 256, 0, st>>>(part_sum, part_used, nb, c_out, used_out);
    return hipGetLastError();
}

hipError_t launch_distinct_experts(const int32_t* const* idx_layers, int L, int T, int k,
                                   int32_t* distinct, int32_t* part_sum, float* mean_out, hipStream_t st) {
    const int nb = cdiv(T, 256);
    distinct_kernel<<<nb, 256, 0, st>>>(idx_layers, L, T, k, distinct, part_sum);
    distinct_finalize_kernel<<<1, 256, 0, st>>>(part_sum, nb, T, mean_out);
    return hipGetLastError();
}

}  // namespace unipool
