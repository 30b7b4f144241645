// bfloat16 grouped GEMMs on the CDNA4 matrix cores (v_mfma_f32_16x16x32_bf16), float accumulate.
//
// Two kernels cover every dense contraction of the layer:
//
//   gemm_xw  : C[rows of e, N] = X[rows of e, K] * W_e          (row-grouped; forward, dgrad, router)
//              X is K-contiguous.  W_e is either [N][K] (K-contiguous) or [K][N] (N-contiguous).
//   gemm_ptq : out[e][i][j] (+)= sum_rows P[row][i] * Q[row][j]  (reduction over the rows of e,
//              possibly chained over several layers; weight gradients)
//
// Common structure
//   * One workgroup of 8 wavefronts per CU, a 256 x 256 output tile, 128 accumulator registers per
//     lane; fragments have one register set each and are refilled in place as their last use passes.
//   * Operand tiles go global -> LDS directly (global_load_lds_dwordx4), several stages deep, one
//     barrier per stage.  The loads are issued through inline assembly so that the wait counts
//     are ours: the compiler would otherwise wait for every outstanding load before any LDS read.
//   * LDS tiles hold 16-byte chunks in XOR-swizzled positions; a direct-to-LDS load writes 64
//     consecutive chunks, so the swizzle is applied on the global address of each lane.
//   * Operands whose reduction index is the strided one in memory are read from LDS with pairs of
//     ds_read_b64_tr_b16, each of which hands a lane four consecutive reduction indices of one column.
//   * The weight fragment is the MFMA A operand and the activation fragment the B operand, so a
//     lane ends up with four consecutive output columns of one row: results are staged through
//     LDS and leave the CU as 16-byte row segments.
//   * Row groups come from a device-side tile table; nothing is read back to the host.  Tiles are
//     walked in a fixed order that keeps the tiles of one expert on one XCD (workgroup ids are dealt
//     round-robin to the 8 XCDs, each of which has its own L2), runs the two row tiles of an expert
//     side by side so that they share its weight tiles in L2, and lets a workgroup request the first
//     stages of its next tile before the epilogue of the current one.
#include "gemm_common.h"

namespace unipool {

namespace {

// Profiling builds (-DUNIPOOL_PHASE_TIMES) add up, per workgroup, the time the first wavefront
// spends in the three phases of a gemm_xw tile (100 MHz ticks): pipeline fill, K loop, epilogue; one row per
// workgroup and launch slot.
#ifdef UNIPOOL_PHASE_TIMES
__device__ unsigned long long g_phase_times[1024][8];
#define PHASE_STAMP(var) const long long var = wall_clock64()
#define PHASE_COMMIT(t0, t1, t2, t3)                                                         \
    if (threadIdx.x == 0 && blockIdx.x < 256) {                                              \
        unsigned long long* pt_ = g_phase_times[blockIdx.x + 256 * (g.launch_slot & 3)];     \
        pt_[0] += (unsigned long long)((t1) - (t0));                                         \
        pt_[1] += (unsigned long long)((t2) - (t1));                                         \
        pt_[2] += (unsigned long long)((t3) - (t2));                                         \
        pt_[3] += 1ull;                                                                      \
        pt_[4] += (unsigned long long)acc_wait_;                                             \
        pt_[5] += (unsigned long long)acc_bar_;                                              \
        pt_[6] += (unsigned long long)acc_cyc_;                                              \
    }
#define PHASE_CLOCK(var) const long long var = clock64()
#else
#define PHASE_STAMP(var)
#define PHASE_COMMIT(t0, t1, t2, t3)
#endif





__global__ __launch_bounds__(512) void build_tiles_kernel(const int32_t* __restrict__ offsets, int E,
                                                          int total_rows, int BM, int pad_even,
                                                          int32_t* __restrict__ meta, int32_t* __restrict__ pair_cnt) {
    if (pair_cnt != nullptr)
        for (int i = threadIdx.x; i < kPairCap; i += 512) pair_cnt[i] = 0;
    __shared__ __attribute__((aligned(16))) int lrows[512];   // rows per expert (0 past E)
    __shared__ __attribute__((aligned(16))) int lkey[512];    // place of an expert in the dealt order
    __shared__ int ltiles[512];           // tiles of the expert at a given place
    __shared__ int scan[2][512];
    const int t = threadIdx.x;
    int r0 = 0, r1 = 0;
    if (t < E) {
        r0 = offsets ? offsets[t] : 0;
        r1 = offsets ? offsets[t + 1] : total_rows;
    }
    const int nt = (r1 - r0 + BM - 1) / BM;
    // Every expert takes an even number of places in the list (the odd one out is an entry without
    // rows, which the workgroups skip): the kernels hand out the list in pairs of row tiles that run
    // side by side and share the weight tile through L2, and a pair must not straddle two experts.
    const int ns = pad_even ? (nt + 1) & ~1 : nt;
    lrows[t] = r1 - r0;
    __syncthreads();
    // Order of the experts in the tile list.  The persistent workgroups walk the list in a fixed
    // pattern (one eighth of it per XCD, dealt in rounds to the workgroups of the XCD), so the list
    // is laid out for them: experts sorted by rows, descending, are dealt to the eight parts in
    // serpentine order (0..7, 7..0, ...), which gives every XCD the same amount of work to within
    // one small expert and makes the tiles that run at the same time equally long.
    // (entries past E hold no rows and take no part; the loops read four experts per LDS access)
    const int E4 = (E + 3) / 4;
    const int rt = r1 - r0;
    int rank = 0;                         // experts with more rows (ties: lower index first)
    for (int o4 = 0; o4 < E4; o4++) {
        const int4 v = reinterpret_cast<const int4*>(lrows)[o4];
        const int o = 4 * o4;
        rank += (v.x > rt) || (v.x == rt && o < t);
        rank += (v.y > rt) || (v.y == rt && o + 1 < t);
        rank += (v.z > rt) || (v.z == rt && o + 2 < t);
        rank += (v.w > rt) || (v.w == rt && o + 3 < t);
    }
    const int lap = rank / kNumXcd, posn = rank % kNumXcd;
    const int part = (lap & 1) ? kNumXcd - 1 - posn : posn;
    const int place = t < E ? part * (512 / kNumXcd) + lap : 0x7fffffff;     // unique below E: lap < 64
    lkey[t] = place;
    ltiles[t] = 0;
    __syncthreads();
    int dense = 0;                        // experts placed before this one
    for (int o4 = 0; o4 < E4; o4++) {
        const int4 v = reinterpret_cast<const int4*>(lkey)[o4];
        dense += (v.x < place) + (v.y < place) + (v.z < place) + (v.w < place);
    }
    __syncthreads();
    if (t < E) ltiles[dense] = ns;
    __syncthreads();
    // exclusive prefix sum of the tiles in list order (inclusive Hillis-Steele scan over 512 entries)
    const int mine = ltiles[t];
    scan[0][t] = mine;
    __syncthreads();
    int cur = 0;
    for (int d = 1; d < 512; d <<= 1) {
        scan[cur ^ 1][t] = scan[cur][t] + (t >= d ? scan[cur][t - d] : 0);
        cur ^= 1;
        __syncthreads();
    }
    ltiles[t] = scan[cur][t] - mine;      // first tile of the expert at place t
    if (t == 0) meta[0] = scan[cur][511];
    __syncthreads();
    // The rows of an expert are cut into equal tiles (multiples of 16 rows, the MFMA's row count)
    // rather than into full tiles plus a remainder: tiles that share an expert's weights then take
    // equally long and stay in step, so the second reader of a weight tile still finds it in L2.
    if (t < E) {
        const int my_first = ltiles[dense];
        const int per = nt > 0 ? (((r1 - r0 + nt - 1) / nt + 15) / 16) * 16 : 0;
        for (int i = 0; i < ns; i++) {
            int32_t* m = meta + kTileBase + 4 * (my_first + i);
            m[0] = t;
            m[1] = r0 + i * per;
            m[2] = max(0, min(per, r1 - (r0 + i * per)));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// gemm_xw
// ---------------------------------------------------------------------------------------------
// One 256 x 256 output tile, eight wavefronts (two per SIMD).  Wavefront (wm, wn) owns the 64
// columns of group wn and every second 32-row strip starting at wm; both wavefronts of a column
// group sit on the same SIMD, so a SIMD always carries the same share of the tile, however many
// strips hold rows.  MTV = strips of THIS wavefront that hold rows (0..4), LH = only the upper 16
// rows of its last strip do; the body is instantiated per (MTV, LH) so that the K loop is
// straight-line code and absent rows have no MFMAs.
// The products are v_mfma_f32_16x16x32_bf16 (at the card's power limit this form sustains about a
// sixth more than 32x32x16): a strip is two 16-row halves, the 64 columns four 16-column blocks.


// pre: what the previous tile has already requested for this one (bit 0: X(0) and W(0), bit 1: W(1));
// g0: number of K stages this workgroup has run before this tile (the LDS buffers rotate on).
template <int BM, int BN, int BK, int NS, bool WK, int EPI, bool KTAIL, int MTV, bool LH>
__device__ __forceinline__ void xw_tile(const GemmArgs& g, char* smem, TileRef cur, TileRef nxt, int pre,
                                        int g0) {
    constexpr int NW = kXwWaves;
    constexpr int TN = 2;
    constexpr int XBYTES = BM * BK * 2;
    constexpr int WBYTES = BN * BK * 2;
    constexpr int XI = BM * BK / 8 / (NW * 64);   // direct-to-LDS loads per wavefront, X tile
    constexpr int WI = BN * BK / 8 / (NW * 64);
    constexpr int KS = BK / 32;                   // slices of 32 reduction indices per stage
    static_assert(KS == 2, "the stage body below is written for two slices");
    static_assert(BM == 256 && BN == 256 && NW == 8, "2 x 4 wavefronts, strips interleaved by 2");
    using XT = KTile<BK>;
    using WTK = KTile<BK>;
    using WTN = NTile16<BN>;

    // The per-MTV bodies are alternatives of one switch.  Their set-up code is identical, and if
    // the compiler merges it in front of the switch the merged values stay live across all the
    // bodies and spill; spill code is scratch traffic, whose wait counts would then serialise the
    // direct-to-LDS pipeline.  Making the inputs opaque here keeps every body self-contained.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    int expert = __builtin_amdgcn_readfirstlane(cur.expert);
    int row0 = __builtin_amdgcn_readfirstlane(cur.row0);
    int rows = __builtin_amdgcn_readfirstlane(cur.rows);
    int nt = __builtin_amdgcn_readfirstlane(cur.nt);
    pre = __builtin_amdgcn_readfirstlane(pre);
    g0 = __builtin_amdgcn_readfirstlane(g0);
    asm volatile("" : "+s"(expert), "+s"(row0), "+s"(rows), "+s"(nt), "+s"(pre), "+s"(g0));
    PHASE_STAMP(t_begin);
#ifdef UNIPOOL_PHASE_TIMES
    long long acc_wait_ = 0, acc_bar_ = 0, acc_cyc_ = 0;
#endif
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 3, wm = wave >> 2;
    const unsigned lds0 = lds_addr_of(smem);
    const int n0 = nt * BN;                 // first column of the tile (plain epilogues)
    const int f0 = nt * (BN / 2);           // first column per half (SWIGLU_FWD)

    // ---- per-lane source pointers of the direct-to-LDS loads ----------------------------------
    // Load i of a wavefront fills LDS chunks (i*NW + wave)*64 .. +63: 8 rows of 128 bytes.  Loads
    // past the tile's last row are left out (xload[i] false, wave-uniform): what the MFMAs then read
    // for those rows is stale, and it only reaches output rows that are never stored.
    const char* xsrc[XI];
    bool xload[XI];
    const char* wsrc[WI];
    const size_t wstep = WK ? (size_t)BK * 2 : (size_t)BK * g.ldw * 2;      // bytes per K step
    auto set_sources = [&](int t_expert, int t_row0, int t_rows, int t_nt) {
        const bf16* We = g.W + (long long)t_expert * g.w_stride;
        const int t_n0 = t_nt * BN, t_f0 = t_nt * (BN / 2);
#pragma unroll
        for (int i = 0; i < XI; i++) {
            const int q = (i * NW + wave) * 64 + lane;
            const int row = q / XT::CPR;
            const int cc = (q % XT::CPR) ^ XT::swz(row);
            int grow = t_row0 + min(row, t_rows - 1);
            if (g.gather != nullptr) grow = g.gather[grow] / g.gather_div;
            xsrc[i] = reinterpret_cast<const char*>(g.X + (size_t)grow * g.ldx + cc * 8);
            xload[i] = ((i * NW + wave) * 64 / XT::CPR) < ((t_rows + 7) & ~7);
        }
        if constexpr (WK) {
#pragma unroll
            for (int i = 0; i < WI; i++) {
                const int q = (i * NW + wave) * 64 + lane;
                const int row = q / WTK::CPR;
                const int cc = (q % WTK::CPR) ^ WTK::swz(row);
                int wrow;
                if constexpr (EPI == EPI_SWIGLU_FWD) {
                    const int half = row / (BN / 2);
                    wrow = half * g.up_rows + min(t_f0 + row % (BN / 2), g.N - 1);
                } else {
                    wrow = min(t_n0 + row, g.N - 1);
                }
                wsrc[i] = reinterpret_cast<const char*>(We + (size_t)wrow * g.ldw + cc * 8);
            }
        } else {
#pragma unroll
            for (int i = 0; i < WI; i++) {
                const int q = (i * NW + wave) * 64 + lane;
                const int krow = q / WTN::CPR;
                const int cc = (q % WTN::CPR) ^ WTN::swz(krow);
                const int col = min(t_n0 + cc * 8, g.N - 8);
                wsrc[i] = reinterpret_cast<const char*>(We + (size_t)krow * g.ldw + col);
            }
        }
    };
    set_sources(expert, row0, rows, nt);

    // acc[tm][mh][nb]: strip tm of this wavefront, 16-row half mh, 16-column block nb
    f32x4 acc[MTV > 0 ? MTV : 1][2][4];
#pragma unroll
    for (int tm = 0; tm < MTV; tm++)
#pragma unroll
        for (int mh = 0; mh < 2; mh++)
#pragma unroll
            for (int nb = 0; nb < 4; nb++) acc[tm][mh][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // LDS rows (K-contiguous W) or columns (N-contiguous W) of this wavefront's two fragments
    int wpos[TN];
    if constexpr (EPI == EPI_SWIGLU_FWD) {
        wpos[0] = wn * 32;
        wpos[1] = BN / 2 + wn * 32;
    } else {
        wpos[0] = wn * 64;
        wpos[1] = wn * 64 + 32;
    }

    const int nk = KTAIL ? (g.K + BK - 1) / BK : g.K / BK;
    // ---- software pipeline ----------------------------------------------------------------------
    // LDS holds NSX stages of the X tile and NSW stages of the W tile (BK reduction indices each).
    // While stage kt is multiplied, X(kt+1), W(kt+1) and W(kt+2) are landing, and from its meeting
    // point on X(kt+2) as well.  A stage is KS slices of 32 indices; every fragment has one register
    // set, and the LDS reads that refill it are interleaved one by one with the MFMAs (issue is in
    // order: a burst of LDS reads would hold back the MFMAs behind it).
    constexpr int NSX = NS, NSW = NS + 1;
    constexpr int WBASE = NSX * XBYTES;
    static_assert(NSX == 2 && NSW == 3, "buffer rotation and wait counts below");
    // Stage kt of this tile lives in X buffer (g0 + kt) mod 2 and W buffer (g0 + kt) mod 3: the
    // buffers rotate on from tile to tile, so the first stages of the next tile can be requested
    // while this tile's last stage and epilogue still hold theirs.
    const int x0 = g0 & 1, w0 = g0 % 3;
    auto xbuf = [&](int kt) { return (kt + x0) & 1; };
    auto wbuf = [&](int kt) { return (kt + w0) % 3; };
    // Fragments of one slice: W block nb (16 columns x 32 indices, the MFMA A operand) and X fragment
    // a (16 rows x 32 indices, the B operand: a < MTV the upper rows of strip a, a >= MTV the lower rows
    // of strip a - MTV), one register set each.  A slice is two halves; slot nb * MTV + tm of the first
    // takes the upper rows of the strips, slot nb * M2 + tm of the second the lower rows, so X[0 .. MTV)
    // and W[0..2] are free for the next slice's data during the second half, W[3] and the other X
    // fragments at its end.
    static_assert(!LH || MTV >= 2, "a lone strip is always computed whole");
    constexpr int M2 = MTV - (LH ? 1 : 0);          // strips whose lower 16 rows are computed
    constexpr int NXF = MTV + M2;
    constexpr int HM1 = 4 * MTV, HM2 = 4 * M2;      // MFMA slots of the two halves of a slice
    bf16x8 wfr[4], xfr[NXF > 0 ? NXF : 1];
    // per-lane part of the fragment addresses (rows that are multiples of 16 further down add whole rows)
    const int l16 = lane & 15, lg = lane >> 4;
    const int koff0 = XT::off(l16, lg), koff1 = XT::off(l16, 4 + lg);       // K-contiguous tiles, slice 0 / 1
    static_assert(XT::CPR == 8, "a slice is four 16-byte chunks of a 128-byte row");
    [[maybe_unused]] int noff[4];                                         // N-contiguous W
    if constexpr (!WK) {
#pragma unroll
        for (int nb = 0; nb < 4; nb++) noff[nb] = WTN::frag_off(wpos[nb >> 1] + 16 * (nb & 1), lane);
    }
    constexpr int ROWB = BK * 2;                                           // bytes per K-contiguous row
    auto load_w = [&](int kt, int ks, int nb) {
        const char* wb = smem + WBASE + wbuf(kt) * WBYTES;
        if constexpr (WK) {
            wfr[nb] = lds_read16(wb + (wpos[nb >> 1] + 16 * (nb & 1)) * ROWB + (ks ? koff1 : koff0));
        } else {
            const char* p = wb + ks * (32 * WTN::CPR * 16) + noff[nb];
            wfr[nb] = lds_read_tr8(p, p + 4 * WTN::CPR * 16);
        }
    };
    auto load_x = [&](int kt, int ks, int a) {
        const int tm = a < MTV ? a : a - MTV, mh = a < MTV ? 0 : 1;
        const char* xb = smem + xbuf(kt) * XBYTES;
        xfr[a] = lds_read16(xb + ((wm + 2 * tm) * 32 + 16 * mh) * ROWB + (ks ? koff1 : koff0));
    };
    auto mfma_one = [&](int a, int nb) {
        const int tm = a < MTV ? a : a - MTV, mh = a < MTV ? 0 : 1;
        acc[tm][mh][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[nb], xfr[a], acc[tm][mh][nb], 0, 0, 0);
    };
    // KTAIL: K is not a multiple of BK; chunks past K come from a page of zeros in both operands
    static_assert(!KTAIL || !WK, "the reduction tail is implemented for N-contiguous W only");
    int xk[KTAIL ? XI : 1], wk[KTAIL ? WI : 1];   // first reduction index of the lane's chunk / row
    if constexpr (KTAIL) {
#pragma unroll
        for (int i = 0; i < XI; i++) {
            const int q = (i * NW + wave) * 64 + lane;
            xk[i] = ((q % XT::CPR) ^ XT::swz(q / XT::CPR)) * 8;
        }
#pragma unroll
        for (int i = 0; i < WI; i++) wk[i] = ((i * NW + wave) * 64 + lane) / WTN::CPR;
    }
    // load i of stage kt of the tile the sources point at, into the buffer of stage kb of this tile
    auto issue_x = [&](int kt, int i, int kb) {
        if (!xload[i]) return;
        const char* src = xsrc[i] + (size_t)kt * BK * 2;
        if constexpr (KTAIL)
            if (kt * BK + xk[i] >= g.K) src = reinterpret_cast<const char*>(g.zeros);
        glds16(src, lds0 + xbuf(kb) * XBYTES + ((i * NW + wave) * 64) * 16);
    };
    auto issue_w = [&](int kt, int i, int kb) {
        const char* src = wsrc[i] + (size_t)kt * wstep;
        if constexpr (KTAIL)
            if (kt * BK + wk[i] >= g.K) src = reinterpret_cast<const char*>(g.zeros);
        glds16(src, lds0 + WBASE + wbuf(kb) * WBYTES + ((i * NW + wave) * 64) * 16);
    };
    // One stage.  The wavefronts meet between the halves of the second slice: stage kt+1 has landed,
    // nobody reads stage kt any more, and the second half, whose operands are in registers, covers the
    // first fragment loads of stage kt+1.  Loads go out two stages ahead, into the buffers that the
    // meeting points release: W(kt+2), whose buffer stage kt-1 held, during the MFMAs ahead of the
    // meeting (IW), X(kt+2), whose buffer is the one stage kt is reading, right behind it.  They are
    // spread between the MFMAs: a wavefront whose load finds the address unit's queue full stands
    // still, MFMAs included, so a burst of loads from all wavefronts at once would cost the matrix
    // cores the whole time the queue takes to drain.
    auto stage_body = [&](auto iw_c, int kt) {
        constexpr bool IW = decltype(iw_c)::value;
        constexpr int SL = 2 * HM1 + HM2;             // slots before the meeting point
        const bool ix = kt + 2 < nk;                  // X(kt+2) exists
        auto w_loads = [&](int slot) {
            if constexpr (IW) {
#pragma unroll
                for (int u = 0; u < WI; u++)
                    if (u * SL / WI == slot) issue_w(kt + 2, u, kt + 2);
            }
        };
        auto x_loads = [&](int slot) {
#pragma unroll
            for (int u = 0; u < XI; u++)
                if (u * HM2 / XI == slot && ix) issue_x(kt + 2, u, kt + 2);
        };
        if constexpr (SL == 0 && IW) {
#pragma unroll
            for (int u = 0; u < WI; u++) issue_w(kt + 2, u, kt + 2);
        }
        auto first_half = [&](int ks, int slot0) {
#pragma unroll
            for (int sl = 0; sl < HM1; sl++) {
                mfma_one(sl % MTV, sl / MTV);
                if (sl == 0) load_w(kt, ks, 3);                        // what the previous slice still held
                if (sl >= 1 && sl <= M2) load_x(kt, ks, MTV + sl - 1);
                w_loads(slot0 + sl);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto second_half = [&](int nkt, int nks, int slot0) {       // (nkt, nks): the slice that follows
#pragma unroll
            for (int sl = 0; sl < HM2; sl++) {
                mfma_one(MTV + sl % M2, sl / M2);
                if (sl < MTV) load_x(nkt, nks, sl);
                if (sl >= M2 && sl % M2 == 0) load_w(nkt, nks, sl / M2 - 1);
                if (slot0 >= 0) w_loads(slot0 + sl);
                else x_loads(sl);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        first_half(0, 0);
        second_half(kt, 1, HM1);
        first_half(1, HM1 + HM2);
        // X(kt+1) and W(kt+1) must have landed.  Loads complete in issue order, and the only ones
        // issued after those two batches are the W loads of stage kt+2.
#ifdef UNIPOOL_PHASE_TIMES
        PHASE_CLOCK(c0_);
#endif
        if (nk - 2 - kt >= 1) wait_vmcnt<WI>();
        else wait_vmcnt<0>();
#ifdef UNIPOOL_PHASE_TIMES
        PHASE_CLOCK(c1_);
#endif
        lds_barrier();
#ifdef UNIPOOL_PHASE_TIMES
        PHASE_CLOCK(c2_);
        acc_wait_ += c1_ - c0_;
        acc_bar_ += c2_ - c1_;
#endif
        if constexpr (HM2 == 0) {
            if (ix) {
#pragma unroll
                for (int u = 0; u < XI; u++) issue_x(kt + 2, u, kt + 2);
            }
        }
        second_half(kt + 1, 0, -1);                   // after the last stage: unused, in bounds
    };
    // prologue: X(0) W(0) X(1) W(1) W(2), less what the previous tile has requested already
    if (!(pre & 1)) {
#pragma unroll
        for (int i = 0; i < XI; i++) issue_x(0, i, 0);
#pragma unroll
        for (int i = 0; i < WI; i++) issue_w(0, i, 0);
    }
    if (nk > 1) {
#pragma unroll
        for (int i = 0; i < XI; i++) issue_x(1, i, 1);
        if (!(pre & 2)) {
#pragma unroll
            for (int i = 0; i < WI; i++) issue_w(1, i, 1);
        }
    }
    if (nk > 2) {
#pragma unroll
        for (int i = 0; i < WI; i++) issue_w(2, i, 2);
    }
    // stage 0 has landed when at most the two W batches of stages 1 and 2 are outstanding (the X
    // batch of stage 1, which may be shorter than XI loads, then has landed too: stricter than needed)
    if (nk >= NSW) wait_vmcnt<(NSW - 1) * WI>();
    else wait_vmcnt<0>();
    lds_barrier();
    PHASE_STAMP(t_filled);
#ifdef UNIPOOL_PHASE_TIMES
    PHASE_CLOCK(cl0_);
#endif
#pragma unroll
    for (int a = 0; a < MTV; a++) load_x(0, 0, a);
    if constexpr (MTV > 0) {
#pragma unroll
        for (int nb = 0; nb < 3; nb++) load_w(0, 0, nb);
    }
    {
        using T = std::integral_constant<bool, true>;
        using F = std::integral_constant<bool, false>;
        // stage 0: the prologue has issued X(1) and W(2) already
        stage_body(F{}, 0);
        int kt = 1;
        for (; kt + 2 < nk; kt++) stage_body(T{}, kt);
        for (; kt < nk; kt++) stage_body(F{}, kt);
    }
    lds_barrier();   // every wavefront is done with the operand tiles
    PHASE_STAMP(t_looped);
    // The buffers of the last stage become the staging space of the epilogue; the others take the
    // first stages of the next tile now, so that its pipeline is full when the epilogue ends.
    constexpr bool PREW1 = Staging<EPI>::PREW1;
    if constexpr (!KTAIL) {
        if (nxt.valid) {
            set_sources(nxt.expert, nxt.row0, nxt.rows, nxt.nt);
#pragma unroll
            for (int i = 0; i < XI; i++) issue_x(0, i, nk);
#pragma unroll
            for (int i = 0; i < WI; i++) issue_w(0, i, nk);
            if (PREW1 && nk > 1) {
#pragma unroll
                for (int i = 0; i < WI; i++) issue_w(1, i, nk + 1);
            }
        }
    }
#ifdef UNIPOOL_PHASE_TIMES
    PHASE_CLOCK(cl1_);
    acc_cyc_ = cl1_ - cl0_;
#endif

    // ---- epilogue ---------------------------------------------------------------------------------
    // acc[tm][mh][nb][r] = C[row (wm + 2 tm)*32 + 16 mh + lane%16][column 16 nb + 4*(lane/16) + r of the wavefront's 64]

    if constexpr (EPI == EPI_F32) {
        float* out = reinterpret_cast<float*>(g.out0);
#pragma unroll
        for (int tm = 0; tm < MTV; tm++)
#pragma unroll
            for (int mh = 0; mh < 2; mh++) {
                if (LH && tm == MTV - 1 && mh == 1) continue;
                const int r_in = (wm + 2 * tm) * 32 + 16 * mh + l16;
                if (r_in < rows) {
                    float* orow = out + (size_t)(row0 + r_in) * g.ldo;
#pragma unroll
                    for (int nb = 0; nb < 4; nb++)
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const int col = n0 + wpos[nb >> 1] + 16 * (nb & 1) + 4 * lg + r;
                            if (col < g.N) orow[col] = acc[tm][mh][nb][r];
                        }
                }
            }
    } else {
        using SG = Staging<EPI>;
        // Staging area of this wavefront: region 0 is the X buffer of the last stage, region 1 its W
        // buffer, region 2 (SwiGLU backward only) the W buffer that would otherwise hold W(1) of the
        // next tile.
        const int region = wave / SG::RW;
        const int rbase = region == 0 ? xbuf(nk - 1) * XBYTES
                                      : WBASE + (region == 1 ? wbuf(nk - 1) : wbuf(nk + 1)) * WBYTES;
        char* stg = smem + rbase + (wave % SG::RW) * SG::WSTG;
        xw_staged_epilogue<EPI, MTV, LH, true>(epi_args(g), AccArray<MTV>{acc}, stg, rows, row0, n0, f0, wm, 2, wn, lane);
    }
    PHASE_STAMP(t_end);
    PHASE_COMMIT(t_begin, t_filled, t_looped, t_end);
}

template <int BM, int BN, int BK, int NS, bool WK, int EPI, bool KTAIL>
__global__ __launch_bounds__(kXwThreads) void gemm_xw_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // ---- persistent workgroups, static schedule ------------------------------------------------
    // One workgroup per CU stays resident and walks a list of tiles that every wavefront can work
    // out by itself (no counter, no hand-over through LDS), so the next tile is known while the
    // current one runs and its first stages are requested before the epilogue.
    //   * Workgroup b belongs to XCD b mod 8 (workgroups are dealt round-robin to the XCDs; if a
    //     device dealt them otherwise, only the L2 locality below would suffer).  Each XCD has its own
    //     L2, so the tile list is cut into eight contiguous parts: the row tiles of an expert, which
    //     share the expert's weights, and its column tiles, which share its rows, stay on one L2.
    //   * Inside a part, round n gives the next P tiles to the P workgroups of the XCD, rotated by n,
    //     so that no workgroup keeps the same position inside the experts' tile groups.  The tile
    //     table lists the experts of a part in descending order of rows: the workgroups of an XCD
    //     work on tiles of nearly equal length at any time and end together.
    const bool flat = g.flat_rows > 0;
    const int n_mt = flat ? (g.flat_rows + g.flat_bm - 1) / g.flat_bm : g.tile_meta[0];
    const int G = flat ? 1 : g.group_m;
    const int per_group = G * g.n_tiles_n;
    const int total = ((n_mt + G - 1) / G) * per_group;
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    const int P = gridDim.x / kNumXcd;                 // workgroups per XCD (the grid is a multiple of 8)
    const int lt_end = min(total, (xcd + 1) * per_xcd);
    const int wm = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);        // wavefronts 4..7: odd strips
    const bool use_pairs = !flat && G == 2 && (per_group & 1) == 0 && g.pair_cnt != nullptr && total / 2 <= g.pair_cap;
    int round = 0;
    // the next tile of this workgroup that holds rows, or valid = 0 at the end of the list
    auto next_tile = [&]() {
        TileRef t = {0, 0, 0, 0, 0, -1};
        for (;;) {
            const int lt = xcd * per_xcd + round * P + (slot + round) % P;
            if (lt >= lt_end) return t;
            round++;
            const int grp = lt / per_group;
            const int rem = lt % per_group;
            const int mt = grp * G + rem % G;
            if (mt >= n_mt) continue;
            if (flat) {
                t.valid = 1;
                t.row0 = mt * g.flat_bm;
                t.rows = min(g.flat_bm, g.flat_rows - t.row0);
                t.nt = rem;
                return t;
            }
            const int rows = g.tile_meta[kTileBase + 4 * mt + 2];
            if (rows <= 0) continue;
            t.valid = 1;
            t.expert = g.tile_meta[kTileBase + 4 * mt];
            t.row0 = g.tile_meta[kTileBase + 4 * mt + 1];
            t.rows = rows;
            t.nt = rem / G;
            // partner: the other row tile of the pair, same column tile (list position lt ^ 1); the
            // test reads the same table entries on both sides, so either both wait or neither does
            if (use_pairs) {
                const int mt2 = mt ^ 1;
                if (mt2 < n_mt && g.tile_meta[kTileBase + 4 * mt2 + 2] > 0 &&
                    g.tile_meta[kTileBase + 4 * mt2] == t.expert)
                    t.pair = lt >> 1;
            }
            return t;
        }
    };
    const int nk = KTAIL ? (g.K + BK - 1) / BK : g.K / BK;
    TileRef cur = next_tile();
    int pre = 0, g0 = 0;
#ifdef UNIPOOL_PHASE_TIMES
    int tile_i_ = 0;
#endif
    while (cur.valid) {
        const TileRef nxt = next_tile();
#ifdef UNIPOOL_PHASE_TIMES
        if (threadIdx.x == 0 && (g.launch_slot & 3) == 1 && tile_i_ < 8)
            g_phase_times[768 + (blockIdx.x & 255)][tile_i_] = (unsigned long long)wall_clock64();
        tile_i_++;
#endif
        // Meet the partner (bounded wait: if it is far behind, go on alone and fetch the weights twice).
        if (cur.pair >= 0) {
            if (threadIdx.x == 0) {
                int32_t* c = g.pair_cnt + cur.pair;
                __hip_atomic_fetch_add(c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int spin = 0; spin < kPairSpins; spin++) {
                    if (__hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= 2) break;
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            lds_barrier();
        }
        // strips wm, wm+2, ... of this wavefront that hold rows, and whether the last of them is the
        // tile's last strip with rows in its upper half only; every body runs the same barriers
        const int strips = (cur.rows + 31) >> 5;
        const int mtv = max(0, (strips - wm + 1) >> 1);
        const bool lh = mtv >= 2 && wm + 2 * (mtv - 1) == strips - 1 && (((cur.rows + 15) >> 4) & 1) != 0;
        switch (2 * mtv + (lh ? 1 : 0)) {
            case 0: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 0, false>(g, smem, cur, nxt, pre, g0); break;
            case 2: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 1, false>(g, smem, cur, nxt, pre, g0); break;
            case 4: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 2, false>(g, smem, cur, nxt, pre, g0); break;
            case 5: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 2, true>(g, smem, cur, nxt, pre, g0); break;
            case 6: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 3, false>(g, smem, cur, nxt, pre, g0); break;
            case 7: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 3, true>(g, smem, cur, nxt, pre, g0); break;
            case 9: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 4, true>(g, smem, cur, nxt, pre, g0); break;
            default: xw_tile<BM, BN, BK, NS, WK, EPI, KTAIL, 4, false>(g, smem, cur, nxt, pre, g0); break;
        }
        lds_barrier();                // the staging space is free: the next tile may load into it
        pre = (!KTAIL && nxt.valid) ? ((Staging<EPI>::PREW1 && nk > 1) ? 3 : 1) : 0;
        g0 = (g0 + nk) % 6;           // the buffers repeat with period 2 and 3
        cur = nxt;
    }
}

// ---------------------------------------------------------------------------------------------
// gemm_ptq: out[e][i][j] (+)= sum_l sum_{row in group e of layer l} P_l[row][i] * Q_l[row][j]
// ---------------------------------------------------------------------------------------------
struct PtqArgs {
    int n_layers;
    const void* const* P;        // device arrays of device pointers
    const void* const* Q;
    const int32_t* const* off;
    int E, mdim, ndim;
    int m_tiles, n_tiles;
    float* out;
    long long out_stride;        // elements between experts
    int accumulate;
    const void* zeros;           // >= 16 readable zero bytes
};

template <int BK, int NS, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_ptq_kernel(const PtqArgs g) {
    // 256 x 256 float tile, 2 x 4 wavefronts of 128 x 64, v_mfma_f32_16x16x32_bf16 (at the card's power
    // limit it sustains about a sixth more than the 32x32x16 form): 8 x 4 accumulator blocks of 16 x 16.
    constexpr int BM = 256, BN = 256;
    constexpr int NT = 64 * NW;               // threads
    constexpr int WNC = NW / 2;               // wavefronts along n (two along m)
    constexpr int CW = BN / WNC;              // columns of a wavefront's block (128 rows)
    constexpr int NA = 8, NB = CW / 16;       // 16-wide fragments of P and of Q per wavefront
    static_assert(NW == 8 && BK == 32 && NB == 4, "one 32-deep slice per stage, 8 x 4 blocks per wavefront");
    constexpr int PBYTES = BK * BM * 2;
    constexpr int STAGE = 2 * PBYTES;
    constexpr int PI = BK * BM / 8 / NT;      // loads per wavefront per operand per stage
    constexpr int LPS = 2 * PI;
    using PT = NTile16<BM>;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int per_e = g.m_tiles * g.n_tiles;
    const int total = g.E * per_e;
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    if (slot >= per_xcd) return;
    const int lt = (blockIdx.x % kNumXcd) * per_xcd + slot;
    if (lt >= total) return;
    const int e = lt / per_e;
    // The 32 workgroups of an XCD run 32 consecutive tiles side by side and share their operand blocks
    // through L2: with the shorter tile axis running fastest the 32 tiles form the squarest block
    // (about 6 x 5 instead of 2 x 16), which needs the fewest distinct operand blocks.
    const int idx = lt % per_e;
    const int m0 = (g.m_tiles <= g.n_tiles ? idx % g.m_tiles : idx / g.n_tiles) * BM;
    const int n0 = (g.m_tiles <= g.n_tiles ? idx / g.m_tiles : idx % g.n_tiles) * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WNC, wn = wave % WNC;
#ifdef UNIPOOL_PHASE_TIMES
    const long long pt_begin = wall_clock64();
#endif
    const unsigned lds0 = lds_addr_of(smem);

    // Per-layer row range and operand pointers of expert e, fetched once into LDS: the K loop then
    // advances from layer to layer without global loads of its own (whose wait counts would also
    // wait for the operand loads in flight) and with wave-uniform control flow.
    __shared__ int lds_r0[kMaxPtqLayers], lds_r1[kMaxPtqLayers];
    __shared__ const bf16* lds_p[kMaxPtqLayers];
    __shared__ const bf16* lds_q[kMaxPtqLayers];
    for (int l = threadIdx.x; l < g.n_layers; l += NT) {
        lds_r0[l] = g.off[l][e];
        lds_r1[l] = g.off[l][e + 1];
        lds_p[l] = reinterpret_cast<const bf16*>(g.P[l]);
        lds_q[l] = reinterpret_cast<const bf16*>(g.Q[l]);
    }
    __syncthreads();
    // The rows of expert e in all the layers form one reduction, cut into K blocks of BK rows without
    // regard to the layers: a block may end one layer's range and begin the next one's, and only the
    // very last block is filled up with zero rows.
    int k_total = 0;
    for (int l = 0; l < g.n_layers; l++) k_total += max(0, __builtin_amdgcn_readfirstlane(lds_r1[l] - lds_r0[l]));
    const int nb = (k_total + BK - 1) / BK;
    float* otile = g.out + (long long)e * g.out_stride;
    if (nb == 0) {
        if (!g.accumulate) {
            for (int i = threadIdx.x; i < BM * BN; i += NT) {
                const int r = m0 + i / BN, c = n0 + i % BN;
                if (r < g.mdim && c < g.ndim) otile[(size_t)r * g.ndim + c] = 0.f;
            }
        }
        return;
    }

    // lane geometry of the direct-to-LDS loads: load i of a wavefront fills LDS slots
    // (i*NW + wave)*64 + lane, i.e. K row 2*NW*i + 2*wave + lane/32, chunk position lane%32.  The
    // swizzle depends on bits 0, 1 and 3 of the K row, which are the same for all i.
    static_assert((2 * NW) % 16 == 0, "the K rows of a lane's loads differ by multiples of 16");
    static_assert(2 * PI == 4, "four loads per K block");
    const int krow0 = 2 * wave + (lane >> 5);
    const int cc = (lane & 31) ^ PT::swz(krow0);
    const int pcol = min(m0 + cc * 8, g.mdim - 8);
    const int qcol = min(n0 + cc * 8, g.ndim - 8);

    // A K block that lies inside one layer's row range is loaded from a wave-uniform row address plus
    // these per-lane byte offsets (no vector arithmetic per load); a block that runs over the end of a
    // range finds, lane by lane, the layer and row of its K index, or the page of zeros past the end.
    const unsigned voff_p = ((unsigned)krow0 * (unsigned)g.mdim + (unsigned)pcol) * 2u;
    const unsigned voff_q = ((unsigned)krow0 * (unsigned)g.ndim + (unsigned)qcol) * 2u;

    // load cursor over the rows of expert e, layer after layer
    int ld_layer = -1, ld_r = 0, ld_end = 0;
    const bf16* ld_p = nullptr;
    const bf16* ld_q = nullptr;
    auto uniform_ptr = [](const bf16* p) {
        const unsigned long long v = (unsigned long long)p;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
        return reinterpret_cast<const bf16*>(((unsigned long long)hi << 32) | lo);
    };
    // The cursor also holds the next layer in which the expert has rows, fetched from LDS when the
    // cursor moves (once per layer): a block that straddles two layers then needs no LDS access.
    int nx_layer = -1, nx_r = 0, nx_end = 0;
    const bf16* nx_p = nullptr;
    const bf16* nx_q = nullptr;
    auto fetch_next = [&]() {
        nx_r = nx_end = 0;
        while (++nx_layer < g.n_layers) {
            nx_r = __builtin_amdgcn_readfirstlane(lds_r0[nx_layer]);
            nx_end = __builtin_amdgcn_readfirstlane(lds_r1[nx_layer]);
            if (nx_end > nx_r) {
                nx_p = uniform_ptr(lds_p[nx_layer]);
                nx_q = uniform_ptr(lds_q[nx_layer]);
                return;
            }
        }
        nx_layer = g.n_layers;
        nx_r = nx_end = 0;
    };
    fetch_next();
    auto next_layer = [&]() {     // the cursor moves to the next layer with rows (wave-uniform); false past the last
        if (nx_layer >= g.n_layers) return false;
        ld_layer = nx_layer;
        ld_r = nx_r;
        ld_end = nx_end;
        ld_p = nx_p;
        ld_q = nx_q;
        fetch_next();
        return true;
    };
    auto next_block = [&]() {     // put the cursor on the first row of the next K block
        while (ld_r >= ld_end)
            if (!next_layer()) break;
    };
    auto advance_block = [&]() {  // move the cursor BK rows on, from layer to layer
        int need = BK;
        for (;;) {
            const int n = min(ld_end - ld_r, need);
            if (n > 0) {
                ld_r += n;
                need -= n;
            }
            if (need == 0 || !next_layer()) break;
        }
    };
    // Per-lane source addresses of the LPS loads of the K block at the cursor (P rows for i < PI, Q
    // rows after), worked out in one place per block so that the load slots between the MFMAs hold
    // nothing but the load.
    const void* blk_src[2 * PI];
    auto block_sources = [&]() {
        if (__builtin_expect(ld_r + BK <= ld_end, 1)) {
#pragma unroll
            for (int i = 0; i < 2 * PI; i++) {
                const int rb = ld_r + 2 * NW * (i < PI ? i : i - PI);         // wave-uniform
                blk_src[i] = i < PI ? reinterpret_cast<const char*>(ld_p + (size_t)rb * g.mdim) + voff_p
                                    : reinterpret_cast<const char*>(ld_q + (size_t)rb * g.ndim) + voff_q;
            }
        } else {
            // K index j of this lane inside the block: in the rest of the cursor's layer, in the next
            // layer, or (the next layer being shorter than the block) further on
            const int rem = ld_end - ld_r, nrows = nx_end - nx_r;
#pragma unroll
            for (int i = 0; i < 2 * PI; i++) {
                const int j = 2 * NW * (i < PI ? i : i - PI) + krow0;
                const int dim = i < PI ? g.mdim : g.ndim, col = i < PI ? pcol : qcol;
                const void* src = g.zeros;
                if (j < rem) src = (i < PI ? ld_p : ld_q) + (size_t)(ld_r + j) * dim + col;
                else if (j - rem < nrows) src = (i < PI ? nx_p : nx_q) + (size_t)(nx_r + j - rem) * dim + col;
                int j0 = rem + nrows;
                for (int lay = nx_layer + 1; j0 < BK && lay < g.n_layers; lay++) {
                    const int r = __builtin_amdgcn_readfirstlane(lds_r0[lay]);
                    const int n = min(__builtin_amdgcn_readfirstlane(lds_r1[lay]) - r, BK - j0);
                    if (n <= 0) continue;
                    const bf16* base = uniform_ptr(i < PI ? lds_p[lay] : lds_q[lay]);
                    if (j >= j0 && j < j0 + n) src = base + (size_t)(r + j - j0) * dim + col;
                    j0 += n;
                }
                blk_src[i] = src;
            }
        }
    };
    auto issue_one = [&](int stage, int i) {
        const int ii = i < PI ? i : i - PI;
        glds16(blk_src[i], lds0 + stage * STAGE + (i < PI ? 0 : PBYTES) + ((ii * NW + wave) * 64) * 16);
    };

    f32x4 acc[NA][NB];
#pragma unroll
    for (int a = 0; a < NA; a++)
#pragma unroll
        for (int b = 0; b < NB; b++) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Fragments: P block a (rows of the output) and Q block b (columns), one register set each.  A
    // stage is 32 MFMA slots, slot 4b + a in each half (a = 0..3 in the first half, 4..7 in the
    // second), so P[0..3] and Q[0..2] become free for the next stage's data during the second half,
    // Q[3] and P[4..7] at its end; the wavefronts meet in the middle, where the next stage's data has
    // landed.
    static_assert(NS >= 2 && (NS - 1) * LPS < 64, "outstanding loads must fit the wait counter");
    bf16x8 pfr[NA], qfr[NB];
    int foff_p[NA], foff_q[NB];
#pragma unroll
    for (int a = 0; a < NA; a++) foff_p[a] = PT::frag_off(wm * 128 + a * 16, lane);
#pragma unroll
    for (int b = 0; b < NB; b++) foff_q[b] = PBYTES + PT::frag_off(wn * CW + b * 16, lane);
    constexpr int SECOND = 4 * PT::CPR * 16;          // bytes between the two reads of a fragment
    auto load_p = [&](int stage, int a) {
        const char* b_ = smem + stage * STAGE + foff_p[a];
        pfr[a] = lds_read_tr8(b_, b_ + SECOND);
    };
    auto load_q = [&](int stage, int b) {
        const char* b_ = smem + stage * STAGE + foff_q[b];
        qfr[b] = lds_read_tr8(b_, b_ + SECOND);
    };
    auto mfma_one = [&](int a, int b) {
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfr[a], qfr[b], acc[a][b], 0, 0, 0);
    };
#ifdef UNIPOOL_PHASE_TIMES
    long long pc_wait = 0, pc_bar = 0;
#endif
    // ISSUE: the loads of K block kb-1+NS go out during the first half of this stage, into the buffer
    // that stage kb-1 has released, spaced by three MFMAs (a burst of loads stalls the issuing
    // wavefronts, MFMAs included, until the address unit's queue has drained).
    auto stage_body = [&](auto issue_c, int kb) {
        constexpr bool ISSUE = decltype(issue_c)::value;
        const int stage = kb % NS, nstage = (kb + 1) % NS;
        static_assert(LPS == 4, "load slots below");
        if constexpr (ISSUE) {
            next_block();
            block_sources();
        }
#pragma unroll
        for (int s = 0; s < 16; s++) {
            mfma_one(s & 3, s >> 2);
            if (s == 0) load_q(stage, 3);                       // what the previous stage still held
            if (s >= 1 && s <= 4) load_p(stage, 3 + s);
            if constexpr (ISSUE) {
                if (s >= 5 && (s - 5) % 3 == 0) issue_one((kb + NS - 1) % NS, (s - 5) / 3);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (ISSUE) advance_block();
#ifdef UNIPOOL_PHASE_TIMES
        const long long pw0 = clock64();
#endif
        if (nb - 2 - kb >= NS - 2) wait_vmcnt<(NS - 2) * LPS>();
        else wait_vmcnt<0>();
#ifdef UNIPOOL_PHASE_TIMES
        const long long pw1 = clock64();
#endif
        __syncthreads();
#ifdef UNIPOOL_PHASE_TIMES
        pc_wait += pw1 - pw0;
        pc_bar += clock64() - pw1;
#endif
#pragma unroll
        for (int s = 0; s < 16; s++) {
            mfma_one(4 + (s & 3), s >> 2);
            if (s < 4) load_p(nstage, s);                       // after the last stage: unused, in bounds
            else if ((s & 3) == 0) load_q(nstage, (s >> 2) - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
#pragma unroll
    for (int s = 0; s < NS; s++)
        if (s < nb) {
            next_block();
            block_sources();
#pragma unroll
            for (int i = 0; i < LPS; i++) issue_one(s, i);
            advance_block();
        }
    if (nb > NS - 1) wait_vmcnt<(NS - 1) * LPS>();
    else wait_vmcnt<0>();
    __syncthreads();
#ifdef UNIPOOL_PHASE_TIMES
    const long long pt_filled = wall_clock64(), pc_filled = clock64();
#endif
#pragma unroll
    for (int a = 0; a < 4; a++) load_p(0, a);
#pragma unroll
    for (int b = 0; b < 3; b++) load_q(0, b);
    {
        stage_body(std::integral_constant<bool, false>{}, 0);       // nb >= 1 here
        int kb = 1;
        for (; kb - 1 + NS < nb; kb++) stage_body(std::integral_constant<bool, true>{}, kb);
        for (; kb < nb; kb++) stage_body(std::integral_constant<bool, false>{}, kb);
    }
#ifdef UNIPOOL_PHASE_TIMES
    const long long pt_looped = wall_clock64(), pc_looped = clock64();
#endif

    // acc[a][b][r] = out[i = m0 + wm*128 + a*16 + 4*(lane/16) + r][j = n0 + wn*CW + b*16 + lane%16]
    // The 128 x CW block of a wavefront leaves in four passes of 32 rows through a wave-private LDS
    // area (rows of CW floats + 4 of padding), so that every lane stores 16 bytes and a wavefront
    // instruction covers whole row segments of 4*CW bytes; when accumulating, the old values are
    // fetched in the same layout.
    __syncthreads();                          // every wavefront is done with the operand stages
    {
        constexpr int SLD = CW + 4;           // staging row stride in floats
        constexpr int LPR = CW / 4;           // lanes per row
        constexpr int RPI = 64 / LPR;         // rows per wavefront instruction
        float* stg = reinterpret_cast<float*>(smem) + wave * (32 * SLD);
        const int jw = n0 + wn * CW;          // first column of the wavefront's block
        const bool vec_ok = (g.ndim & 3) == 0 && (reinterpret_cast<size_t>(g.out) & 15) == 0;
#pragma unroll
        for (int a2 = 0; a2 < NA / 2; a2++) {
#pragma unroll
            for (int ah = 0; ah < 2; ah++)
#pragma unroll
                for (int b = 0; b < NB; b++)
#pragma unroll
                    for (int r = 0; r < 4; r++)
                        stg[(16 * ah + 4 * (lane >> 4) + r) * SLD + b * 16 + (lane & 15)] = acc[2 * a2 + ah][b][r];
            const int i_blk = m0 + wm * 128 + a2 * 32;
#pragma unroll 4
            for (int it = 0; it < 32 / RPI; it++) {
                const int row = it * RPI + lane / LPR;
                const int c4 = (lane % LPR) * 4;
                const int i = i_blk + row, j = jw + c4;
                if (i >= g.mdim || j >= g.ndim) continue;
                float4 v = *reinterpret_cast<const float4*>(stg + row * SLD + c4);
                float* dst = otile + (size_t)i * g.ndim + j;
                if (vec_ok) {                 // then j + 3 < ndim as well
                    if (g.accumulate) {
                        const float4 o = *reinterpret_cast<const float4*>(dst);
                        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                    }
                    *reinterpret_cast<float4*>(dst) = v;
                } else {
                    const float vv[4] = {v.x, v.y, v.z, v.w};
                    for (int q = 0; q < 4; q++)
                        if (j + q < g.ndim) dst[q] = (g.accumulate ? dst[q] : 0.f) + vv[q];
                }
            }
        }
    }
#ifdef UNIPOOL_PHASE_TIMES
    if (threadIdx.x == 0) {
        unsigned long long* pt_ = g_phase_times[512 + (blockIdx.x & 255)];
        atomicAdd(&pt_[0], (unsigned long long)(pt_filled - pt_begin));
        atomicAdd(&pt_[1], (unsigned long long)(pt_looped - pt_filled));
        atomicAdd(&pt_[2], (unsigned long long)(wall_clock64() - pt_looped));
        atomicAdd(&pt_[3], 1ull);
        atomicAdd(&pt_[4], (unsigned long long)pc_wait);
        atomicAdd(&pt_[5], (unsigned long long)pc_bar);
        atomicAdd(&pt_[6], (unsigned long long)(pc_looped - pc_filled));
        atomicAdd(&pt_[7], (unsigned long long)nb);
    }
#endif
}

// Set-up of the router weight gradient in one launch: row offsets of the token chunks, the pointer
// table of the reduction (P, Q, offsets) and the page of zeros that stands in for rows past a chunk.
__global__ __launch_bounds__(256) void route_bwd_prep_kernel(int T, int chunk_rows, int nchunks,
                                                             int32_t* __restrict__ off, void** table,
                                                             const void* p, const void* q,
                                                             uint32_t* __restrict__ zeros) {
    const int i = threadIdx.x;
    for (int c = i; c <= nchunks; c += 256) off[c] = min(T, c * chunk_rows);
    if (i < 64) zeros[i] = 0u;
    if (i == 0) {
        table[0] = const_cast<void*>(p);
        table[1] = const_cast<void*>(q);
        table[2] = off;
    }
}

__global__ void reduce_partials_kernel(const float* __restrict__ part, int nparts, size_t n,
                                       float* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float v = 0.f;
    for (int p = 0; p < nparts; p++) v += part[(size_t)p * n + i];
    out[i] = v;
}

// ---------------------------------------------------------------------------------------------
// launch helpers
// ---------------------------------------------------------------------------------------------
constexpr int kFlatBM = 128;     // row tiles of ungrouped matrices (router): a token count of 128 per CU fills the chip
constexpr int kBM = 256, kBN = 256, kBK = 64, kNS = 2;   // gemm_xw: 128-byte row segments per load
constexpr int kPtqBK = 32, kPtqNS = 4, kPtqWaves = 8;       // gemm_ptq
constexpr int kGemmLds = kNS * kBM * kBK * 2 + (kNS + 1) * kBN * kBK * 2;   // 2 X stages + 3 W stages = 160 KiB
constexpr int kPtqLds = kPtqNS * 2 * kPtqBK * 256 * 2;            // 128 KiB


template <bool WK, int EPI, bool KTAIL = false>
hipError_t run_xw(GemmArgs a, int max_row_tiles, hipStream_t st) {
    auto kern = gemm_xw_kernel<kBM, kBN, kBK, kNS, WK, EPI, KTAIL>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    a.group_m = 2;
    (void)max_row_tiles;
    const int grid = max(kNumXcd, num_cus() / kNumXcd * kNumXcd);
    kern<<<grid, kXwThreads, kGemmLds, st>>>(a);
    return hipGetLastError();
}

hipError_t run_ptq(const PtqArgs& a, hipStream_t st) {
    auto kern = gemm_ptq_kernel<kPtqBK, kPtqNS, kPtqWaves>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kPtqLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int total = a.E * a.m_tiles * a.n_tiles;
    const int grid = cdiv(total, kNumXcd) * kNumXcd;
    kern<<<grid, 64 * kPtqWaves, kPtqLds, st>>>(a);
    return hipGetLastError();
}

// the meeting counters live behind the largest possible tile table (total_rows / 256 + 2 E entries)
int32_t* pair_counters(int32_t* meta, int E, int total_rows) {
    return meta + kTileBase + 4 * (total_rows / kBM + 2 * E);
}

// Timing aid of debugging builds: UNIPOOL_W0=1 makes every expert read the weights of expert 0, so that the
// weight stream comes from the caches instead of HBM (same instructions, results meaningless).
long long debug_w_stride(long long w_stride) {
#ifdef UNIPOOL_DEBUG_SWITCHES
    static int v = -1;
    if (v < 0) {
        const char* e = getenv("UNIPOOL_W0");
        v = (e && e[0] == '1') ? 1 : 0;
    }
    return v == 1 ? 0 : w_stride;
#else
    return w_stride;
#endif
}

hipError_t build_tiles(const int32_t* offsets, int E, int total_rows, int32_t* meta, hipStream_t st) {
    build_tiles_kernel<<<1, 512, 0, st>>>(offsets, E, total_rows, kBM, 1, meta, pair_counters(meta, E, total_rows));
    return hipGetLastError();
}

}  // namespace

int num_cus() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess)
            n = p.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

bool mfma_ffn_supported(const unipool_shape& s) {
    // the tile table is built by one workgroup with a thread per expert; the weight-gradient kernel
    // keeps the per-layer row ranges of an expert in LDS
    return s.dtype == UNIPOOL_BF16 && s.d_model % 64 == 0 && s.d_ff % 64 == 0 && s.E <= kMaxTableExperts;
}

bool mfma_router_supported(const unipool_shape& s) {
    return s.dtype == UNIPOOL_BF16 && s.d_model % 64 == 0 && s.E % 8 == 0;
}

hipError_t mfma_logits(const unipool_shape& s, const void* x, const void* w, float* z,
                       int32_t* tile_meta, hipStream_t st) {
    GemmArgs a = {};
    a.X = (const bf16*)x; a.ldx = s.d_model;
    a.W = (const bf16*)w; a.w_stride = 0; a.ldw = s.d_model;
    a.K = s.d_model; a.N = s.E; a.n_tiles_n = cdiv(s.E, kBN);
    a.tile_meta = tile_meta; a.out0 = z; a.ldo = s.E;
    a.flat_rows = s.T; a.flat_bm = kFlatBM;
    return run_xw<true, EPI_F32>(a, cdiv(s.T, kBM), st);
}

hipError_t mfma_ffn_gate_up(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                           const void* wgu, void* a_out, void* b_out, void* h_out, int32_t* tile_meta,
                           hipStream_t st, const int32_t* slot_of_row) {
    const int S = s.T * s.k, d = s.d_model, f = s.d_ff;
    const int max_tiles = S / kBM + s.E;
    hipError_t e = build_tiles(offsets, s.E, S, tile_meta, st);
    if (e != hipSuccess) return e;
    GemmArgs a = {};
    a.X = (const bf16*)x_perm; a.ldx = d;
    a.W = (const bf16*)wgu; a.w_stride = debug_w_stride(2LL * f * d); a.ldw = d;
    a.K = d; a.N = f; a.n_tiles_n = cdiv(f, kBN / 2);
    a.tile_meta = tile_meta; a.out0 = a_out; a.out1 = b_out; a.out2 = h_out; a.ldo = f;
    a.up_rows = f;
    a.gather = slot_of_row; a.gather_div = s.k;
    return run_xw<true, EPI_SWIGLU_FWD>(a, max_tiles, st);
}

hipError_t mfma_ffn_fwd(const unipool_shape& s, const void* x_perm, const int32_t* offsets,
                        const void* wgu, const void* wd, void* a_out, void* b_out, void* h_out,
                        void* y, int32_t* tile_meta, hipStream_t st, const int32_t* slot_of_row) {
    const int S = s.T * s.k, d = s.d_model, f = s.d_ff;
    const int max_tiles = S / kBM + s.E;
    hipError_t e = mfma_ffn_gate_up(s, x_perm, offsets, wgu, a_out, b_out, h_out, tile_meta, st, slot_of_row);
    if (e != hipSuccess) return e;
    GemmArgs b = {};
    b.X = (const bf16*)h_out; b.ldx = f;
    b.W = (const bf16*)wd; b.w_stride = debug_w_stride((long long)d * f); b.ldw = f;
    b.K = f; b.N = d; b.n_tiles_n = cdiv(d, kBN);
    b.tile_meta = tile_meta; b.launch_slot = 1; b.out0 = y; b.ldo = d;
    if (b.K >= kPairMinK) { b.pair_cnt = pair_counters(tile_meta, s.E, S); b.pair_cap = kPairCap; }
    return run_xw<true, EPI_STORE>(b, max_tiles, st);
}

hipError_t mfma_ffn_dgrad(const unipool_shape& s, const void* dy, const void* a_in, const void* b_in,
                          const int32_t* offsets, const void* wgu, const void* wd, void* dx,
                          void* d_act, int32_t* tile_meta, hipStream_t st) {
    const int S = s.T * s.k, d = s.d_model, f = s.d_ff;
    const int max_tiles = S / kBM + s.E;
    hipError_t e = build_tiles(offsets, s.E, S, tile_meta, st);
    if (e != hipSuccess) return e;
    GemmArgs a = {};   // dH = dY W_down (W_down[e] is [d][f]: reduction index strided), then SwiGLU backward
    a.X = (const bf16*)dy; a.ldx = d;
    a.W = (const bf16*)wd; a.w_stride = debug_w_stride((long long)d * f); a.ldw = f;
    a.K = d; a.N = f; a.n_tiles_n = cdiv(f, kBN);
    a.tile_meta = tile_meta; a.out0 = d_act; a.ldo = 2 * f;
    a.aux_a = (const bf16*)a_in; a.aux_b = (const bf16*)b_in;
    e = run_xw<false, EPI_SWIGLU_BWD>(a, max_tiles, st);
    if (e != hipSuccess) return e;
    GemmArgs b = {};   // dX = [dA|dB] W_gate_up (W_gate_up[e] is [2f][d])
    b.X = (const bf16*)d_act; b.ldx = 2 * f;
    b.W = (const bf16*)wgu; b.w_stride = debug_w_stride(2LL * f * d); b.ldw = d;
    b.K = 2 * f; b.N = d; b.n_tiles_n = cdiv(d, kBN);
    b.tile_meta = tile_meta; b.launch_slot = 1; b.out0 = dx; b.ldo = d;
    if (b.K >= kPairMinK) { b.pair_cnt = pair_counters(tile_meta, s.E, S); b.pair_cap = kPairCap; }
    return run_xw<false, EPI_STORE>(b, max_tiles, st);
}

hipError_t mfma_ffn_wgrad(const unipool_shape& s, int n_layers, const void* const* x_perm_l,
                          const void* const* d_act_l, const void* const* h_l,
                          const void* const* dy_l, const int32_t* const* offsets_l,
                          float* dwgu, float* dwd, int accumulate, const void* zeros,
                          hipStream_t st) {
    const int d = s.d_model, f = s.d_ff;
    PtqArgs a = {};    // d_w_gate_up[e][n][c] = sum d_act[row][n] * x_perm[row][c]
    a.n_layers = n_layers; a.P = d_act_l; a.Q = x_perm_l; a.off = offsets_l;
    a.E = s.E; a.mdim = 2 * f; a.ndim = d; a.m_tiles = cdiv(2 * f, 256); a.n_tiles = cdiv(d, 256);
    a.out = dwgu; a.out_stride = 2LL * f * d; a.accumulate = accumulate; a.zeros = zeros;
    hipError_t e = run_ptq(a, st);
    if (e != hipSuccess) return e;
    PtqArgs b = {};    // d_w_down[e][c][n] = sum dy[row][c] * h[row][n]
    b.n_layers = n_layers; b.P = dy_l; b.Q = h_l; b.off = offsets_l;
    b.E = s.E; b.mdim = d; b.ndim = f; b.m_tiles = cdiv(d, 256); b.n_tiles = cdiv(f, 256);
    b.out = dwd; b.out_stride = (long long)d * f; b.accumulate = accumulate; b.zeros = zeros;
    return run_ptq(b, st);
}

hipError_t mfma_route_bwd_mm(const unipool_shape& s, const void* x, const void* w, const void* dz,
                             float* dw, void* dx, int dx_accumulate, int32_t* tile_meta,
                             float* wpart, const void* zeros, hipStream_t st) {
    const int d = s.d_model, E = s.E, T = s.T;
    // d_w_router = dz^T x: the token axis is cut into chunks whose partial products are summed in
    // a fixed order.
    // as many chunks as give every CU one output tile in a single round
    const int tiles_per_chunk = cdiv(E, 256) * cdiv(d, 256);
    const int nchunks = max(1, min(min(kRouteBwdSplit, cdiv(T, 256)), num_cus() / tiles_per_chunk));
    const int chunk_rows = cdiv(cdiv(T, nchunks), 32) * 32;
    const int used = cdiv(T, chunk_rows);
    // the pointer table and the chunk offsets live behind the tile table
    int32_t* off = tile_meta;                       // [used + 1]
    void** tab = reinterpret_cast<void**>(tile_meta + 1024);
    route_bwd_prep_kernel<<<1, 256, 0, st>>>(T, chunk_rows, used, off, tab, dz, x,
                                             reinterpret_cast<uint32_t*>(const_cast<void*>(zeros)));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    PtqArgs a = {};
    a.n_layers = 1;
    a.P = (const void* const*)(tab + 0); a.Q = (const void* const*)(tab + 1);
    a.off = (const int32_t* const*)(tab + 2);
    a.E = used; a.mdim = E; a.ndim = d; a.m_tiles = cdiv(E, 256); a.n_tiles = cdiv(d, 256);
    a.out = wpart; a.out_stride = (long long)E * d; a.accumulate = 0; a.zeros = zeros;
    e = run_ptq(a, st);
    if (e != hipSuccess) return e;
    const size_t n = (size_t)E * d;
    reduce_partials_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(wpart, used, n, dw);
    // dx (+)= dz W   (W is [E][d]: reduction index strided)
    GemmArgs b = {};
    // 256-row tiles where they still give every CU a tile: the short reduction (E indices) makes the pipeline
    // fill of a tile as long as its loop, and a taller tile pays it once for twice the rows
    b.flat_rows = T; b.flat_bm = (cdiv(T, kBM) * cdiv(d, kBN) >= num_cus()) ? kBM : kFlatBM;
    b.X = (const bf16*)dz; b.ldx = E;
    b.W = (const bf16*)w; b.w_stride = 0; b.ldw = d;
    b.K = E; b.N = d; b.n_tiles_n = cdiv(d, kBN);
    b.tile_meta = tile_meta; b.out0 = dx; b.ldo = d; b.add = dx_accumulate; b.zeros = zeros;
    if (E % kBK != 0) return run_xw<false, EPI_STORE, true>(b, cdiv(T, kBM), st);
    return run_xw<false, EPI_STORE>(b, cdiv(T, kBM), st);
}

}  // namespace unipool

#ifdef UNIPOOL_PHASE_TIMES
// Copies the phase sums to the host ([1024][8] values) and clears them.
extern "C" int unipool_debug_phase_times(unsigned long long* out) {
    hipError_t e = hipMemcpyFromSymbol(out, HIP_SYMBOL(unipool::g_phase_times), sizeof(unsigned long long) * 8192);
    if (e != hipSuccess) return (int)e;
    static unsigned long long zeros[8192];
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(unipool::g_phase_times), zeros, sizeof(zeros));
}
#endif
