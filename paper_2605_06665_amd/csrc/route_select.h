// Router selection of one token by a group of GS lanes (paper Sec. 4.3, Eq. 7; softmax router of the
// comparison rows, Sec. 5.4): shared by the stand-alone top-k kernel and by the epilogue of the fused router
// GEMM, so that both take every decision and every sum in the same order.
#pragma once
#include "common.h"

namespace unipool {

// Lane s of the group holds the logits z[i] of experts s + GS*i (0 past E).  Adds the token's
// scores to the lane's running sums ps[], picks the k largest logits (ties: lower index), counts
// them in cnt[] (LDS, one word per expert) and writes index and gate (= score) of every pick.
// softmax = false: score_i = sigma_c max(0, z_i) / (||z|| + eps)   (NormRouter, Eq. 7)
// softmax = true : score_i = exp(z_i - max z) / sum_j exp(z_j - max z)
// `live` and `softmax` are uniform inside the group; a dead group takes part in the shuffles and writes nothing.
template <int GS, int VPL>
__device__ __forceinline__ void route_select(const float (&z)[VPL], int sl, int E, int k, float sigma_c,
                                             float eps, bool softmax, bool live, size_t t,
                                             int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, int* cnt,
                                             float (&ps)[VPL]) {
    float scale, zmax = 0.f;
    if (!softmax) {
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) ss += z[i] * z[i];
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        scale = sigma_c / (sqrtf(ss) + eps);
        if (live) {
#pragma unroll
            for (int i = 0; i < VPL; i++) ps[i] += fmaxf(z[i], 0.f) * scale;
        }
    } else {
        zmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < VPL; i++)
            if (sl + GS * i < E) zmax = fmaxf(zmax, z[i]);
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 64));
        float ex[VPL];
        float se = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            ex[i] = (sl + GS * i < E) ? expf(z[i] - zmax) : 0.f;
            se += ex[i];
        }
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
        scale = 1.0f / se;
        if (live) {
#pragma unroll
            for (int i = 0; i < VPL; i++) ps[i] += ex[i] * scale;
        }
    }
    unsigned taken = 0;
    for (int j = 0; j < k; j++) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            const int e = sl + GS * i;
            const bool ok = (e < E) && !((taken >> i) & 1u);
            if (ok && (z[i] > bv || bi == 0x7fffffff)) { bv = z[i]; bi = e; }
        }
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            const bool other_valid = oi != 0x7fffffff;
            const bool mine_valid = bi != 0x7fffffff;
            const bool take = other_valid && (!mine_valid || ov > bv || (ov == bv && oi < bi));
            if (take) { bv = ov; bi = oi; }
        }
        if (bi % GS == sl) {
            taken |= 1u << (bi / GS);
            if (live) {
                atomicAdd(&cnt[bi], 1);
                topk_idx[t * k + j] = bi;
                topk_gate[t * k + j] = softmax ? expf(bv - zmax) * scale : fmaxf(bv, 0.f) * scale;
            }
        }
    }
}

}  // namespace unipool
