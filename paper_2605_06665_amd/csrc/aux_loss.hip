// Pool-level auxiliary loss over the L layers that share the pool (paper Sec. 4.2, Eq. 4-6).
// One block; thread i owns expert i.  The usage counts of all layers are reduced on the device.
#include "kernels.h"

namespace unipool {

namespace {

__global__ __launch_bounds__(512) void pool_aux_loss_kernel(
    const int32_t* __restrict__ counts, const float* __restrict__ psum,
    const float* __restrict__ fbar_in, int L, int E, float inv_slots, float inv_tokens,
    float alpha_m, int32_t* __restrict__ pool_counts, float* __restrict__ fbar_out,
    float* __restrict__ loss, float* __restrict__ aux_coef) {
    __shared__ float red[512];
    const int i = threadIdx.x;
    float term = 0.f;
    if (i < E) {
        int c = 0;
        float p = 0.f;
        for (int l = 0; l < L; l++) {
            c += counts[(size_t)l * E + i];
            p += psum[(size_t)l * E + i];
        }
        const float fnow = (float)c * inv_slots;           // Eq. 4 with f = n / (T k)
        const float f = fbar_in ? fbar_in[i] : fnow;
        pool_counts[i] = c;
        fbar_out[i] = fnow;
        aux_coef[i] = alpha_m * f * inv_tokens;            // derivative of Eq. 6 w.r.t. a score
        term = f * (p * inv_tokens);                       // fbar_i * Pbar_i
    }
    red[i] = term;
    __syncthreads();
    for (int s = 256; s > 0; s >>= 1) {                    // fixed-shape tree: deterministic
        if (i < s) red[i] += red[i + s];
        __syncthreads();
    }
    if (i == 0) loss[0] = alpha_m * red[0];
}

}  // namespace

hipError_t launch_pool_aux_loss(const unipool_shape& s, const int32_t* counts, const float* psum,
                                const float* fbar_in, int32_t* pool_counts, float* fbar_out,
                                float* loss, float* aux_coef, hipStream_t st) {
    const float inv_slots = (float)(1.0 / ((double)s.L * s.T * s.k));
    const float inv_tokens = (float)(1.0 / ((double)s.L * s.T));
    pool_aux_loss_kernel<<<1, 512, 0, st>>>(counts, psum, fbar_in, s.L, s.E, inv_slots, inv_tokens,
                                            s.alpha_pool * (float)s.E, pool_counts, fbar_out, loss,
                                            aux_coef);
    return hipGetLastError();
}

}  // namespace unipool
