// Router selection of one token by a group of GS lanes (paper Sec. 4.3, Eq. 7; softmax router of the
// comparison rows, Sec. 5.4): shared by the stand-alone top-k kernel and by the fused router
// kernel, so that both take every decision and every sum in the same order.
#pragma once
#include "common.h"

namespace unipool {

// All-reduce over a group of GS = 16 or 32 adjacent lanes without LDS traffic: two quad permutes, the mirror
// of half a row and of a row (each leaves every lane with the result of twice as many lanes), then for 32
// lanes the swap of odd and even rows.  Every lane of the wavefront must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E, kDppRowHalfMirror = 0x141, kDppRowMirror = 0x140;

template <int GS, class F>
__device__ __forceinline__ float group_reduce_f(float v, F f) {
    static_assert(GS == 16 || GS == 32, "a row of lanes or two");
    v = f(v, dpp_f<kDppQuadXor1>(v));
    v = f(v, dpp_f<kDppQuadXor2>(v));
    v = f(v, dpp_f<kDppRowHalfMirror>(v));
    v = f(v, dpp_f<kDppRowMirror>(v));
    if constexpr (GS == 32) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = f(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}
template <int GS>
__device__ __forceinline__ int group_min_i(int v) {
    static_assert(GS == 16 || GS == 32, "a row of lanes or two");
    v = min(v, dpp_i<kDppQuadXor1>(v));
    v = min(v, dpp_i<kDppQuadXor2>(v));
    v = min(v, dpp_i<kDppRowHalfMirror>(v));
    v = min(v, dpp_i<kDppRowMirror>(v));
    if constexpr (GS == 32) {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        v = min((int)r[0], (int)r[1]);
    }
    return v;
}

// Lane s of the group holds the logits z[i] of experts s + GS*i (anything past E).  Adds the token's
// scores to the lane's running sums ps[], picks the k largest logits (ties: lower index), counts
// them in cnt[] (LDS, one word per expert) and writes index and gate (= score) of every pick.
// softmax = false: score_i = sigma_c max(0, z_i) / (||z|| + eps)   (NormRouter, Eq. 7)
// softmax = true : score_i = exp(z_i - max z) / sum_j exp(z_j - max z)
// `live` and `softmax` are uniform inside the group; a dead group takes part in the exchanges and writes
// nothing.  Each round takes the largest logit left: its value by a maximum over the group, then the lowest
// expert index that holds this value by a minimum.  Logits are taken to be finite (they are sums of finite
// products); a row with fewer than k finite logits gets indices below E all the same, possibly repeated.
template <int GS, int VPL>
__device__ __forceinline__ void route_select(const float (&z)[VPL], int sl, int E, int k, float sigma_c,
                                             float eps, bool softmax, bool live, size_t t,
                                             int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, int* cnt,
                                             float (&ps)[VPL]) {
    const auto add = [](float a, float b) { return a + b; };
    const auto fmx = [](float a, float b) { return fmaxf(a, b); };
    float zz[VPL];                                   // logits still in the running; -inf: past E or taken
#pragma unroll
    for (int i = 0; i < VPL; i++) zz[i] = (sl + GS * i < E) ? z[i] : -INFINITY;
    float scale, zmax = 0.f;
    if (!softmax) {
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) ss += (sl + GS * i < E) ? z[i] * z[i] : 0.f;
        ss = group_reduce_f<GS>(ss, add);
        scale = sigma_c / (sqrtf(ss) + eps);
        if (live) {
#pragma unroll
            for (int i = 0; i < VPL; i++) ps[i] += fmaxf(zz[i], 0.f) * scale;
        }
    } else {
        zmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < VPL; i++) zmax = fmaxf(zmax, zz[i]);
        zmax = group_reduce_f<GS>(zmax, fmx);
        float ex[VPL];
        float se = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            ex[i] = (sl + GS * i < E) ? expf(z[i] - zmax) : 0.f;
            se += ex[i];
        }
        se = group_reduce_f<GS>(se, add);
        scale = 1.0f / se;
        if (live) {
#pragma unroll
            for (int i = 0; i < VPL; i++) ps[i] += ex[i] * scale;
        }
    }
    for (int j = 0; j < k; j++) {
        float bv = zz[0];
#pragma unroll
        for (int i = 1; i < VPL; i++) bv = fmaxf(bv, zz[i]);
        bv = group_reduce_f<GS>(bv, fmx);
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = VPL - 1; i >= 0; i--)
            if (zz[i] == bv) bi = sl + GS * i;
        bi = group_min_i<GS>(bi);
        bi = min(bi, E - 1);                          // only a row without k finite logits gets here past E
        const int mine = bi - sl;                     // GS * i on the lane that holds the pick
#pragma unroll
        for (int i = 0; i < VPL; i++)
            if (mine == GS * i) zz[i] = -INFINITY;
        if (live && (bi % GS) == sl) {
            atomicAdd(&cnt[bi], 1);
            topk_idx[t * k + j] = bi;
            topk_gate[t * k + j] = softmax ? expf(bv - zmax) * scale : fmaxf(bv, 0.f) * scale;
        }
    }
}

}  // namespace unipool
