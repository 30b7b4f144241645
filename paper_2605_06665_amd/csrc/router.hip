// NormRouter per-token kernels (paper Sec. 4.3, Eq. 7): score, top-k, gates, layer
// statistics, and the backward of the score.  One 64-lane wavefront owns one token at a
// time; lane j holds the logits of experts j, j+64, ... (at most 8 per lane, E <= 512).
#include "kernels.h"
#include "route_select.h"

namespace unipool {

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kTokPerWave = kRouterTokensPerBlock / kWavesPerBlock;

// Statistics and selection for the tokens of one block.  A group of GS lanes owns one token at a
// time (64 / GS tokens per wavefront in flight); lane s of the group holds the logits of experts
// s, s + GS, ... (VPL of them, E <= GS * VPL).  Partial sums leave the block in a fixed order, so the
// final reduction over blocks is deterministic.
template <int GS, int VPL>
__global__ __launch_bounds__(256) void route_score_topk_kernel(
    const float* __restrict__ logits, int T, int E, int k, float sigma_c, float eps, int softmax,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate,
    int32_t* __restrict__ cnt_part, float* __restrict__ psum_part) {
    constexpr int TPW = 64 / GS;                       // tokens per wavefront at a time
    static_assert(VPL <= 32 && kTokPerWave % TPW == 0, "taken-mask width; whole rounds per wavefront");
    __shared__ float lds_ps[kWavesPerBlock][kMaxE];
    __shared__ int lds_cnt[kMaxE];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int grp = lane / GS, sl = lane % GS;
    for (int i = threadIdx.x; i < kMaxE; i += 256) lds_cnt[i] = 0;
    __syncthreads();

    float ps[VPL];
#pragma unroll
    for (int i = 0; i < VPL; i++) ps[i] = 0.f;

    const int t0 = blockIdx.x * kRouterTokensPerBlock + wave * kTokPerWave + grp;
    float z[VPL], zn[VPL];
    auto fetch = [&](int t, float* dst) {
        const float* zr = logits + (size_t)min(t, T - 1) * E;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            const int e = sl + GS * i;
            dst[i] = (e < E) ? zr[e] : 0.f;
        }
    };
    fetch(t0, zn);
    for (int tt = 0; tt < kTokPerWave; tt += TPW) {
        const int t = t0 + tt;
#pragma unroll
        for (int i = 0; i < VPL; i++) z[i] = zn[i];
        if (tt + TPW < kTokPerWave) fetch(t + TPW, zn);          // the next token's logits, a round ahead
        route_select<GS, VPL>(z, sl, E, k, sigma_c, eps, softmax != 0, t < T, (size_t)t, topk_idx, topk_gate, lds_cnt, ps);
    }
    // score sums: over the token groups of the wavefront (fixed order), then over the wavefronts
#pragma unroll
    for (int i = 0; i < VPL; i++) {
#pragma unroll
        for (int o = GS; o < 64; o <<= 1) ps[i] += __shfl_xor(ps[i], o, 64);
        if (grp == 0 && sl + GS * i < kMaxE) lds_ps[wave][sl + GS * i] = ps[i];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        float v = lds_ps[0][e];
        v += lds_ps[1][e];
        v += lds_ps[2][e];
        v += lds_ps[3][e];
        psum_part[(size_t)blockIdx.x * E + e] = v;
        cnt_part[(size_t)blockIdx.x * E + e] = lds_cnt[e];
    }
}

// One block per expert: the block partials are summed by a fixed-shape tree (deterministic).
__global__ __launch_bounds__(256) void route_finalize_kernel(
    const int32_t* __restrict__ cnt_part, const float* __restrict__ psum_part, int nblocks, int E,
    int32_t* __restrict__ counts, float* __restrict__ psum) {
    __shared__ int rc[256];
    __shared__ float rp[256];
    const int e = blockIdx.x, t = threadIdx.x;
    int c = 0;
    float p = 0.f;
    for (int b = t; b < nblocks; b += 256) {
        c += cnt_part[(size_t)b * E + e];
        p += psum_part[(size_t)b * E + e];
    }
    rc[t] = c;
    rp[t] = p;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) {
            rc[t] += rc[t + s];
            rp[t] += rp[t + s];
        }
        __syncthreads();
    }
    if (t == 0) {
        counts[e] = rc[0];
        psum[e] = rp[0];
    }
}

// Backward of Eq. 7 per token, a group of GS lanes per token as in the forward selection:
// ds = aux_coef + dgate on the selected experts; dz = J^T ds with J the Jacobian of
// s = sigma c relu(z / (||z|| + eps)); d sigma = sum ds * s / sigma.
template <typename TA, int GS, int VPL>
__global__ __launch_bounds__(256) void route_bwd_dz_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ topk_idx,
    const float* __restrict__ dgate, const float* __restrict__ aux_coef, int T, int E, int k,
    float sigma, float c, float eps, int softmax, TA* __restrict__ dz, float* __restrict__ dsigma_part) {
    constexpr int TPW = 64 / GS;
    static_assert(kTokPerWave % TPW == 0, "whole rounds per wavefront");
    __shared__ float lds_ds[kWavesPerBlock];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int grp = lane / GS, sl = lane % GS;
    const auto add = [](float a, float b) { return a + b; };
    const auto fmx = [](float a, float b) { return fmaxf(a, b); };
    float coef[VPL];
#pragma unroll
    for (int i = 0; i < VPL; i++) {
        const int e = sl + GS * i;
        coef[i] = (aux_coef != nullptr && e < E) ? aux_coef[e] : 0.f;
    }
    float dsig = 0.f;
    const int t0 = blockIdx.x * kRouterTokensPerBlock + wave * kTokPerWave + grp;
    for (int tt = 0; tt < kTokPerWave; tt += TPW) {
        const int t = t0 + tt;
        const bool live = t < T;
        const int tc = min(t, T - 1);
        const float* zr = logits + (size_t)tc * E;
        float z[VPL], ds[VPL];
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            const int e = sl + GS * i;
            z[i] = (e < E) ? zr[e] : 0.f;
            ss += z[i] * z[i];
            ds[i] = coef[i];
        }
        ss = group_reduce_f<GS>(ss, add);
        // the k selections and their gate gradients are requested together, then applied in slot order
        int selv[kMaxK];
        float gdv[kMaxK];
#pragma unroll
        for (int j = 0; j < kMaxK; j++) {
            selv[j] = j < k ? topk_idx[(size_t)tc * k + j] : -1;
            gdv[j] = j < k ? dgate[(size_t)tc * k + j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < kMaxK; j++) {
#pragma unroll
            for (int i = 0; i < VPL; i++)
                if (selv[j] == sl + GS * i) ds[i] += gdv[j];
        }
        if (softmax) {
            // dz_j = p_j (ds_j - <ds, p>) with p = softmax(z); sigma takes no part
            float zmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < VPL; i++)
                if (sl + GS * i < E) zmax = fmaxf(zmax, z[i]);
            zmax = group_reduce_f<GS>(zmax, fmx);
            float pr[VPL];
            float se = 0.f;
#pragma unroll
            for (int i = 0; i < VPL; i++) {
                pr[i] = (sl + GS * i < E) ? expf(z[i] - zmax) : 0.f;
                se += pr[i];
            }
            se = group_reduce_f<GS>(se, add);
            const float inv_se = 1.0f / se;
            float dotp = 0.f;
#pragma unroll
            for (int i = 0; i < VPL; i++) {
                pr[i] *= inv_se;
                dotp += ds[i] * pr[i];
            }
            dotp = group_reduce_f<GS>(dotp, add);
            if (live) {
#pragma unroll
                for (int i = 0; i < VPL; i++) {
                    const int e = sl + GS * i;
                    if (e < E) dz[(size_t)t * E + e] = from_f32<TA>(pr[i] * (ds[i] - dotp));
                }
            }
            continue;
        }
        const float n = sqrtf(ss);
        const float inv = 1.0f / (n + eps);
        float dzh[VPL];
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; i++) {
            const float zh = z[i] * inv;
            if (live) dsig += ds[i] * c * fmaxf(zh, 0.f);
            dzh[i] = (zh > 0.f) ? ds[i] * sigma * c : 0.f;
            dot += dzh[i] * z[i];
        }
        dot = group_reduce_f<GS>(dot, add);
        const float back = (n > 0.f) ? dot * inv * inv / n : 0.f;
        if (live) {
#pragma unroll
            for (int i = 0; i < VPL; i++) {
                const int e = sl + GS * i;
                if (e < E) {
                    const float v = (n > 0.f) ? dzh[i] * inv - z[i] * back : 0.f;
                    dz[(size_t)t * E + e] = from_f32<TA>(v);
                }
            }
        }
    }
    dsig = wave_sum(dsig);
    if (lane == 0) lds_ds[wave] = dsig;
    __syncthreads();
    if (threadIdx.x == 0)
        dsigma_part[blockIdx.x] = ((lds_ds[0] + lds_ds[1]) + lds_ds[2]) + lds_ds[3];
}

__global__ __launch_bounds__(256) void dsigma_finalize_kernel(const float* __restrict__ part, int n,
                                                              float* __restrict__ out) {
    __shared__ float red[256];
    const int t = threadIdx.x;
    float v = 0.f;
    for (int i = t; i < n; i += 256) v += part[i];
    red[t] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    if (t == 0) out[0] = red[0];
}

}  // namespace

hipError_t launch_route_score_topk(const unipool_shape& s, const float* logits, int32_t* topk_idx,
                                   float* topk_gate, int32_t* counts, float* psum,
                                   int32_t* cnt_part, float* psum_part, hipStream_t st) {
    const int nblocks = cdiv(s.T, kRouterTokensPerBlock);
    // lanes per token and logits per lane by pool size
    if (s.E <= 128)
        route_score_topk_kernel<16, 8><<<nblocks, 256, 0, st>>>(logits, s.T, s.E, s.k, s.sigma * s.c, s.eps, s.router,
                                                                topk_idx, topk_gate, cnt_part, psum_part);
    else if (s.E <= 256)
        route_score_topk_kernel<16, 16><<<nblocks, 256, 0, st>>>(logits, s.T, s.E, s.k, s.sigma * s.c, s.eps, s.router,
                                                                 topk_idx, topk_gate, cnt_part, psum_part);
    else
        route_score_topk_kernel<32, 16><<<nblocks, 256, 0, st>>>(logits, s.T, s.E, s.k, s.sigma * s.c, s.eps, s.router,
                                                                 topk_idx, topk_gate, cnt_part, psum_part);
    route_finalize_kernel<<<s.E, 256, 0, st>>>(cnt_part, psum_part, nblocks, s.E, counts, psum);
    return hipGetLastError();
}

hipError_t launch_route_finalize(const unipool_shape& s, const int32_t* cnt_part, const float* psum_part,
                                 int32_t* counts, float* psum, hipStream_t st) {
    route_finalize_kernel<<<s.E, 256, 0, st>>>(cnt_part, psum_part, cdiv(s.T, kRouterTokensPerBlock), s.E,
                                               counts, psum);
    return hipGetLastError();
}

hipError_t launch_route_bwd_dz(const unipool_shape& s, const float* logits, const int32_t* topk_idx,
                               const float* dgate, const float* aux_coef, void* dz,
                               float* dsigma_part, float* d_sigma, hipStream_t st) {
    const int nblocks = cdiv(s.T, kRouterTokensPerBlock);
#define UNIPOOL_DZ(TA, GS, VPL)                                                                        \
    route_bwd_dz_kernel<TA, GS, VPL><<<nblocks, 256, 0, st>>>(logits, topk_idx, dgate, aux_coef, s.T, s.E, \
                                                              s.k, s.sigma, s.c, s.eps, s.router, (TA*)dz, dsigma_part)
    if (s.dtype == UNIPOOL_BF16) {
        if (s.E <= 128) UNIPOOL_DZ(bf16, 16, 8);
        else if (s.E <= 256) UNIPOOL_DZ(bf16, 16, 16);
        else UNIPOOL_DZ(bf16, 32, 16);
    } else {
        if (s.E <= 128) UNIPOOL_DZ(float, 16, 8);
        else if (s.E <= 256) UNIPOOL_DZ(float, 16, 16);
        else UNIPOOL_DZ(float, 32, 16);
    }
#undef UNIPOOL_DZ
    dsigma_finalize_kernel<<<1, 256, 0, st>>>(dsigma_part, nblocks, d_sigma);
    return hipGetLastError();
}

}  // namespace unipool
