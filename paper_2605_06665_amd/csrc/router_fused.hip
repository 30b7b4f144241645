// Router of one layer in one kernel (paper Sec. 4.3, Eq. 7 and the top-k paragraph): logits z = x W^T on the
// matrix cores, then scores, top-k, gates and the per-block statistics, for bfloat16 inputs and pools of
// up to 512 experts.
//
// The router is a memory-bound product: x is read once (2 T d bytes), the router matrix is small (E d
// bfloat16, at most 1 MiB) and stays in the caches, and the float logits go out once.  So x does not pass
// through LDS at all:
//   * A workgroup owns 64 or 128 consecutive tokens.  Four of its six wavefronts (one per SIMD) multiply: each
//     owns 16 or 32 tokens (NT = 1 or 2 fragments of 16 tokens) against ALL experts.  Its x fragments (16
//     tokens x 32 reduction indices, the MFMA B operand: lane l holds 8 consecutive indices of token l % 16)
//     come straight from global memory into registers, four or eight slices of 32 indices ahead, with no
//     barrier involved: per CU 16 to 32 KiB of x are in flight at any time.
//   * The router matrix passes through LDS in chunks of 64 (32 for pools beyond 256 experts) reduction
//     indices, three chunks deep.  The other two wavefronts do nothing but request the chunks with
//     direct-to-LDS loads and wait for them, so the wait counts of the two streams never meet (loads complete
//     in order per wavefront: in one wavefront a wait for a weight chunk would also wait for every x fragment
//     requested before it).  One barrier per chunk.  A weight fragment (16 experts x 32 indices, the A
//     operand) is read from LDS once per slice and wavefront, a group of fragments ahead of the MFMAs that
//     use them, and multiplied with the NT token fragments.
//   * After the last chunk the float logits of the workgroup's tokens are laid out in LDS (in the space of
//     the weight chunks), written to global memory as whole rows, and the selection code shared with the
//     stand-alone kernel runs on them in all six wavefronts: a group of 16 or 32 lanes per token.
// Measured at T = 32768, d_model = 1536, E = 192: 21 us for the product (x streams at 4.7 TB/s), 2 us for the
// copy of the logits, 10 us for the selection; the selection is bound by instruction issue (about 130
// instructions per pick for 16 logits per lane).
// Partial counts and score sums leave per block of 64 tokens; route_finalize adds them in a fixed order.
#include "gemm_common.h"
#include "route_select.h"

namespace unipool {

namespace {

constexpr int kRfConsumers = 4;        // wavefronts that multiply (one per SIMD)
constexpr int kRfProducers = 2;        // wavefronts that bring the weight chunks into LDS
constexpr int kRfWaves = kRfConsumers + kRfProducers;
constexpr int kRfThreads = kRfWaves * 64;
constexpr int kRfBuffers = 3;          // weight chunks in LDS
constexpr int kRfMaxE = 512;

// LDS: kRfBuffers weight chunks of E16 rows x BK indices; later the logits tile [TOK][E + 4] floats, then the
// score sums of the six wavefronts [6][E] and the selection counts of the 64-token blocks.
constexpr int rf_lds_bytes(int E16, int BK, int TOK) {
    const int ring = kRfBuffers * E16 * BK * 2;
    const int tile = TOK * (E16 + 4) * 4 + kRfWaves * E16 * 4 + (TOK / 64) * E16 * 4;
    return ring > tile ? ring : tile;
}

struct RouterArgs {
    const bf16* x;
    const bf16* w;
    float* logits;
    int32_t* topk_idx;
    float* topk_gate;
    int32_t* cnt_part;
    float* psum_part;
    int T, d, E, k;
    float sigma_c, eps;
    int softmax;
};

// NB16: 16-expert blocks (compile time: the accumulators are registers; even, so that the weight chunk is a
// whole number of loads); NT: token fragments per wavefront; BK: reduction indices per weight chunk.
// PD: slices of 32 indices that the x fragments run ahead (d_model is a multiple of 32 PD, so the main loop
// has no conditional code and the compiler's wait counts for the fragments stay exact).
template <int NB16, int NT, int BK, int PD>
__device__ __forceinline__ void rf_body(const RouterArgs& a, char* smem) {
    constexpr int TOK = kRfConsumers * 16 * NT;
    constexpr int E16 = NB16 * 16;
    constexpr int WBYTES = E16 * BK * 2;
    constexpr int SPC = BK / 32;                                          // slices per chunk
    constexpr int WIP = E16 * BK / 8 / (kRfProducers * 64);               // loads per producer lane and chunk
    static_assert(E16 * BK / 8 % (kRfProducers * 64) == 0 && WIP >= 1 && WIP < 60, "whole loads; wait count range");
    static_assert(PD % SPC == 0, "the x ring holds whole chunks");
    using WT = KTile<BK>;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    const int t0 = blockIdx.x * TOK;
    const int E = a.E, d = a.d;
    const int nk = d / BK;                       // weight chunks
    const int ns = d / 32;                       // slices
    const unsigned lds0 = lds_addr_of(smem);

    f32x4 acc[NT][NB16];
    if (wave >= kRfConsumers) {
        // ---- producers: chunk c -> buffer c % 3.  Chunk c+2 goes into the buffer of chunk c-1 once every
        // wavefront has passed the barrier of chunk c (nobody reads chunk c-1 any more).
        const int p = wave - kRfConsumers;
        const char* wsrc[WIP];
        unsigned wdst[WIP];
#pragma unroll
        for (int i = 0; i < WIP; i++) {
            const int q = (i * kRfProducers + p) * 64 + lane;             // 16-byte chunk of the tile
            const int row = q / WT::CPR;
            const int cc = (q % WT::CPR) ^ WT::swz(row);
            wsrc[i] = reinterpret_cast<const char*>(a.w + (size_t)min(row, E - 1) * d + cc * 8);
            wdst[i] = ((i * kRfProducers + p) * 64) * 16;
        }
        auto issue_w = [&](int c) {
#pragma unroll
            for (int i = 0; i < WIP; i++)
                glds16(wsrc[i] + (size_t)c * BK * 2, lds0 + (c % kRfBuffers) * WBYTES + wdst[i]);
        };
        issue_w(0);
        if (nk > 1) issue_w(1);
        for (int c = 0; c < nk; c++) {
            // chunk c has landed when at most the loads of chunk c+1 are outstanding (loads complete in order)
            if (c + 1 < nk) wait_vmcnt<WIP>();
            else wait_vmcnt<0>();
            lds_barrier();
            if (c + 2 < nk) issue_w(c + 2);
        }
    } else {
        // ---- consumers: x fragments straight from global memory, kRfPrefetch slices ahead.  These
        // wavefronts issue no other loads, so the compiler's own wait counts for the fragments are exact.
        const bf16* xrow[NT];
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
            xrow[nt] = a.x + (size_t)min(t0 + (wave * NT + nt) * 16 + l16, a.T - 1) * d + lg * 8;
        bf16x8 xq[PD][NT];                       // slice s lives in xq[s % PD]
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
#pragma unroll
            for (int nb = 0; nb < NB16; nb++) acc[nt][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        int koff[2];
        koff[0] = WT::off(l16, lg);
        koff[1] = SPC == 2 ? WT::off(l16, 4 + lg) : 0;
#pragma unroll
        for (int u = 0; u < PD; u++)
#pragma unroll
            for (int nt = 0; nt < NT; nt++) xq[u][nt] = *reinterpret_cast<const bf16x8*>(xrow[nt] + (size_t)u * 32);
        for (int s0 = 0; s0 < ns; s0 += PD) {
#pragma unroll
            for (int u = 0; u < PD; u++) {
                const int s = s0 + u;                             // slice; its fragments are in xq[u]
                const int c = s / SPC;
                if (u % SPC == 0) lds_barrier();                  // chunk c has landed (the producers waited for it)
                const char* wb = smem + (c % kRfBuffers) * WBYTES + koff[u % SPC];
                // weight fragments in groups of G, read one group ahead of the MFMAs that use them (a lone
                // wavefront per SIMD has nobody to hide its LDS latency behind)
                constexpr int G = NB16 % 4 == 0 ? 4 : 2, NG = NB16 / G;
                bf16x8 wf[2][G];
#pragma unroll
                for (int i = 0; i < G; i++) wf[0][i] = lds_read16(wb + (i * 16) * (BK * 2));
#pragma unroll
                for (int gq = 0; gq < NG; gq++) {
                    if (gq + 1 < NG) {
#pragma unroll
                        for (int i = 0; i < G; i++)
                            wf[(gq + 1) & 1][i] = lds_read16(wb + (((gq + 1) * G + i) * 16) * (BK * 2));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < G; i++)
#pragma unroll
                        for (int nt = 0; nt < NT; nt++)
                            acc[nt][gq * G + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[gq & 1][i], xq[u][nt],
                                                                                          acc[nt][gq * G + i], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // refill the slot with the slice PD ahead (past the end: the last slice again, never used)
                const int sn = min(s + PD, ns - 1);
#pragma unroll
                for (int nt = 0; nt < NT; nt++)
                    xq[u][nt] = *reinterpret_cast<const bf16x8*>(xrow[nt] + (size_t)sn * 32);
            }
        }
    }
    lds_barrier();                                                // every wavefront is done with the weight chunks

    // ---- logits of the workgroup's tokens into LDS (in the space of the weight chunks)
    const int ldz = E + 4;
    float* tile = reinterpret_cast<float*>(smem);
    float* lds_ps = tile + TOK * ldz;
    int* lds_cnt = reinterpret_cast<int*>(lds_ps + kRfWaves * E);
    for (int i = tid; i < (TOK / 64) * E; i += kRfThreads) lds_cnt[i] = 0;
    if (wave < kRfConsumers) {
        // acc[nt][nb][r] = z[token (wave NT + nt) 16 + l16][expert 16 nb + 4 lg + r]
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            float* trow = tile + ((wave * NT + nt) * 16 + l16) * ldz;
#pragma unroll
            for (int nb = 0; nb < NB16; nb++) {
                const int e = 16 * nb + 4 * lg;
                if (e < E)                                        // E is a multiple of 8, so e + 3 < E as well
                    *reinterpret_cast<float4*>(trow + e) =
                        make_float4(acc[nt][nb][0], acc[nt][nb][1], acc[nt][nb][2], acc[nt][nb][3]);
            }
        }
    }
    lds_barrier();
    // logits to global memory as whole rows (when the caller keeps them); all six wavefronts copy
    const int rows = min(TOK, a.T - t0);
    if (a.logits != nullptr) {
        const int c4n = E / 4;
        for (int id = tid; id < rows * c4n; id += kRfThreads) {
            const int r = id / c4n, c4 = id % c4n;
            // streaming store: the rows are read again only by the backward pass, and lines left dirty in
            // L2 would be written back after the last workgroup, when nothing overlaps the write any more
            const float4 v = *reinterpret_cast<const float4*>(tile + r * ldz + 4 * c4);
            const f32x4 q = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(a.logits + (size_t)(t0 + r) * E + 4 * c4));
        }
    }
    // ---- selection by all six wavefronts: the 64 / TPW steps of a 64-token block are split among the
    // WPB wavefronts of the block, a group of GS lanes per token
    constexpr int WPB = kRfWaves / (TOK / 64);        // wavefronts per 64-token block (3 or 6)
    {
        constexpr int GS = NB16 > 16 ? 32 : 16;       // lanes per token
        constexpr int VPL = E16 / GS < 8 ? 8 : E16 / GS;
        constexpr int TPW = 64 / GS;                  // tokens in flight per wavefront
        constexpr int STEPS = 64 / TPW;               // steps per 64-token block
        const int grp = lane / GS, sl = lane % GS;
        const int blk = wave / WPB, q = wave % WPB;
        float ps[VPL];
#pragma unroll
        for (int i = 0; i < VPL; i++) ps[i] = 0.f;
        for (int st = q * STEPS / WPB; st < (q + 1) * STEPS / WPB; st++) {
            const int lr = blk * 64 + st * TPW + grp;
            const float* zr = tile + min(lr, rows - 1) * ldz;
            float z[VPL];
#pragma unroll
            for (int i = 0; i < VPL; i++) {
                const int e = sl + GS * i;
                z[i] = (e < E) ? zr[e] : 0.f;
            }
            route_select<GS, VPL>(z, sl, E, a.k, a.sigma_c, a.eps, a.softmax != 0, lr < rows, (size_t)(t0 + lr),
                                  a.topk_idx, a.topk_gate, lds_cnt + blk * E, ps);
        }
#pragma unroll
        for (int i = 0; i < VPL; i++) {
#pragma unroll
            for (int o = GS; o < 64; o <<= 1) ps[i] += __shfl_xor(ps[i], o, 64);
            if (grp == 0 && sl + GS * i < E) lds_ps[wave * E + sl + GS * i] = ps[i];
        }
    }
    lds_barrier();
    // partial statistics of the 64-token blocks: the wavefronts of a block in ascending order
    const int nblocks = (a.T + 63) / 64;
    for (int id = tid; id < (TOK / 64) * E; id += kRfThreads) {
        const int b = id / E, e = id % E;
        const int blk = t0 / 64 + b;
        if (blk < nblocks && b * 64 < rows) {
            float v = lds_ps[(b * WPB) * E + e];
#pragma unroll
            for (int q = 1; q < WPB; q++) v += lds_ps[(b * WPB + q) * E + e];
            a.psum_part[(size_t)blk * E + e] = v;
            a.cnt_part[(size_t)blk * E + e] = lds_cnt[b * E + e];
        }
    }
}

// Two token fragments per wavefront and 64-index chunks for pools of up to 256 experts, one fragment and
// 32-index chunks beyond (the accumulators and the three weight chunks must fit registers and LDS).
template <int NT, int PD>
__global__ __launch_bounds__(kRfThreads) void router_fused_kernel(const RouterArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int nb16 = (a.E + 15) / 16;
#define UNIPOOL_RF_CASE(N, BK) \
    if (nb16 <= N) { rf_body<N, NT, BK, PD>(a, smem); return; }
    UNIPOOL_RF_CASE(2, 64) UNIPOOL_RF_CASE(4, 64) UNIPOOL_RF_CASE(6, 64) UNIPOOL_RF_CASE(8, 64)
    UNIPOOL_RF_CASE(12, 64) UNIPOOL_RF_CASE(16, 64)
    if constexpr (NT == 1) {
        UNIPOOL_RF_CASE(24, 32) UNIPOOL_RF_CASE(32, 32)
    }
#undef UNIPOOL_RF_CASE
}

}  // namespace

bool router_fused_supported(const unipool_shape& s) {
    return s.dtype == UNIPOOL_BF16 && s.d_model % 128 == 0 && s.E % 8 == 0 && s.E <= kRfMaxE;
}

// One 64-token block of partial statistics per 64 tokens: cnt_part / psum_part [ceil(T/64)][E].
hipError_t router_fused(const unipool_shape& s, const void* x, const void* w, float* z, int32_t* topk_idx,
                        float* topk_gate, int32_t* cnt_part, float* psum_part, hipStream_t st) {
    RouterArgs a = {};
    a.x = (const bf16*)x; a.w = (const bf16*)w; a.logits = z;
    a.topk_idx = topk_idx; a.topk_gate = topk_gate; a.cnt_part = cnt_part; a.psum_part = psum_part;
    a.T = s.T; a.d = s.d_model; a.E = s.E; a.k = s.k;
    a.sigma_c = s.sigma * s.c; a.eps = s.eps; a.softmax = s.router == UNIPOOL_ROUTER_SOFTMAX;
    // 128 tokens per workgroup (two token fragments per weight fragment read) where that still gives every CU
    // a workgroup and the accumulators fit (E <= 256); 64 tokens otherwise
    const bool two = s.E <= 256 && cdiv(s.T, 128) >= num_cus();
    const int tok = two ? 128 : 64;
    // the body the kernel picks pads the experts to its block count: size LDS for that
    const int nb16 = cdiv(s.E, 16);
    int nbody = 32;
    for (int n : {2, 4, 6, 8, 12, 16, 24, 32})
        if (nb16 <= n) { nbody = n; break; }
    const int lds = rf_lds_bytes(nbody * 16, nbody <= 16 ? 64 : 32, tok);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    auto launch = [&](auto kern, bool& attr_set) {
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        kern<<<cdiv(s.T, tok), kRfThreads, lds, st>>>(a);
        return hipGetLastError();
    };
    static bool set[3] = {false, false, false};
    // one token fragment: eight slices ahead where the reduction length allows; two fragments leave registers
    // for four
    if (two) return launch(router_fused_kernel<2, 4>, set[0]);
    const bool deep = s.d_model % 256 == 0;
    return deep ? launch(router_fused_kernel<1, 8>, set[1]) : launch(router_fused_kernel<1, 4>, set[2]);
}

}  // namespace unipool
