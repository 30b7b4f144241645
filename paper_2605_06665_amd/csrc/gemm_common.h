// Shared pieces of the bfloat16 MFMA GEMM kernels: arguments, tile table layout, direct-to-LDS loads,
// LDS tile layouts with their swizzles, and the staged epilogues of the row-grouped GEMM.
#pragma once
#include <type_traits>

#include "kernels.h"

namespace unipool {

struct GemmArgs {
    const bf16* X;
    int ldx;
    const bf16* W;
    long long w_stride;   // elements between experts
    int ldw;
    int K, N;             // reduction length; number of output columns (per half for SWIGLU_FWD)
    int n_tiles_n;
    int32_t* tile_meta;
    int launch_slot;      // ordinal of the launch inside its entry point (profiling builds file phase times by it)
    void* out0;
    void* out1;
    void* out2;
    int ldo;
    int add;              // EPI_STORE: add to the destination
    const bf16* aux_a;
    const bf16* aux_b;
    int up_rows;          // EPI_SWIGLU_FWD: row offset of the up projection inside W_e (= d_ff)
    int group_m;          // row tiles walked together
    const void* zeros;    // >= 16 readable zero bytes (reduction tail of KTAIL kernels)
    // gathered rows: row r of the grouped order is row gather[r] / gather_div of X (null: row r itself)
    const int32_t* gather;
    int gather_div;
    // ungrouped matrices (router): flat_rows > 0 replaces the tile table by row tiles of flat_bm rows
    int flat_rows, flat_bm;
    // Meeting point of the two workgroups that run the two row tiles of an expert side by side (one
    // zeroed counter per pair of list positions, or null): they start their tiles together, so the
    // weight tile one of them fetches is still in L2 when the other asks for it.
    int32_t* pair_cnt;
    int pair_cap;
};

struct TileRef {
    int valid, expert, row0, rows, nt;
    int pair;       // index of the meeting counter shared with the partner tile, or -1
};

int num_cus();

namespace {

constexpr int EPI_STORE = 0;       // bf16 store (optionally added to the destination)
constexpr int EPI_SWIGLU_FWD = 1;  // tile = [gate | up] columns; writes A, B, H = silu(A)*B
constexpr int EPI_SWIGLU_BWD = 2;  // acc = dH; reads A, B; writes dA | dB
constexpr int EPI_F32 = 3;         // float store

constexpr int kNumXcd = 8;

constexpr int kMaxPtqLayers = 256;   // layers chained in one weight-gradient reduction


// ---------------------------------------------------------------------------------------------
// low-level helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void glds16(const void* gptr, unsigned lds_addr) {
    // 64 lanes x 16 bytes -> LDS[lds_addr + 16*lane]; lds_addr must be wave-uniform.
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(base)
                 : "memory", "m0");
}

__device__ __forceinline__ void glds16_s(const void* sbase, unsigned voff, unsigned lds_addr) {
    // as glds16, the source address given as a wave-uniform base plus a 32-bit byte offset per lane
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_addr);
    // (the base is wave-uniform by contract; reading the first lane keeps it in scalar registers where the
    // compiler cannot prove that, and costs nothing where it can)
    const unsigned long long sb = (unsigned long long)sbase;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)sb);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(sb >> 32));
    const void* ub = reinterpret_cast<const void*>(((unsigned long long)hi << 32) | lo);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(ub), "s"(base)
                 : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    // gfx9 encoding: vmcnt[3:0] -> bits 3:0, vmcnt[5:4] -> bits 15:14; other counters untouched
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Workgroup barrier that orders LDS traffic only: earlier LDS operations of the wavefront are
// complete, outstanding global stores and loads are left in flight (__syncthreads() would wait for
// every global store the compiler knows of, i.e. for the whole epilogue of a tile to reach memory).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const char*)p;
}

__device__ __forceinline__ bf16x8 lds_read16(const char* p) {
    return *reinterpret_cast<const bf16x8*>(p);
}

__device__ __forceinline__ bf16x8 lds_read_tr8(const char* p0, const char* p1) {
    typedef __attribute__((address_space(3))) short4v* lp;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p0);
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p1);
    union { short4v s[2]; bf16x8 v; } u;
    u.s[0] = lo;
    u.s[1] = hi;
    return u.v;
}

// K-contiguous tile: rows of BK elements, CPR = BK/8 chunks per row.
template <int BK> struct KTile {
    static constexpr int CPR = BK / 8;
    static constexpr int RP = 256 / (BK * 2);   // rows per 256 bytes
    __device__ static __forceinline__ int swz(int row) { return (row / RP) & (CPR - 1); }
    // byte offset of logical chunk cc of row
    __device__ static __forceinline__ int off(int row, int cc) {
        return (row * CPR + (cc ^ swz(row))) * 16;
    }
};

// N-contiguous tile: BK rows of BC elements, CPR = BC/8 chunks per row (>= 16), read for
// v_mfma_f32_16x16x32_bf16: a fragment is 16 columns x 32 reduction
// indices; lane l ends with column l%16 and indices 8*(l/16) .. +7.  Two transposing reads (K rows
// krow and krow+4) of the 4 x 16 block that a group of 16 lanes addresses.  The swizzle keeps the four
// K rows of a group and the groups 8 rows apart in different banks.
template <int BC> struct NTile16 {
    static constexpr int CPR = BC / 8;
    __device__ static __forceinline__ int swz(int krow) { return ((krow & 3) << 2) | (((krow >> 3) & 1) << 1); }
    __device__ static __forceinline__ int off(int krow, int col) {
        return (krow * CPR + ((col >> 3) ^ swz(krow))) * 16 + (col & 7) * 2;
    }
    // byte offset of the first read of the fragment at columns col0 .. col0+15, reduction indices 0..31;
    // the second read is 4 K rows (4 * CPR * 16 bytes) further on
    __device__ static __forceinline__ int frag_off(int col0, int lane) {
        return off(8 * (lane >> 4) + ((lane & 15) >> 2), col0 + 4 * (lane & 3));
    }
};

// four floats to four bfloat16 (round to nearest even); converting pairs as vectors lets the compiler
// use one packed conversion per pair instead of a conversion, a shift and an OR per value
__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
    typedef __attribute__((ext_vector_type(2))) float f32x2v;
    typedef __attribute__((ext_vector_type(2))) bf16 bf16x2v;
    union { bf16x2v h[2]; uint2 u; } p;
    p.h[0] = __builtin_convertvector(f32x2v{a, b}, bf16x2v);
    p.h[1] = __builtin_convertvector(f32x2v{c, d}, bf16x2v);
    return p.u;
}

// ---------------------------------------------------------------------------------------------
// tile table: [0] = number of entries; entry i at kTileBase + 4i: expert, first row, rows in tile
// (0 for the entry that pads an expert to an even number of places)
// ---------------------------------------------------------------------------------------------
constexpr int kTileBase = 64;
constexpr int kMaxTableExperts = 512;   // build_tiles_kernel: one thread per expert
constexpr int kPairSpins = 48;      // polls of the partner's arrival, roughly a microsecond apart
constexpr int kPairCap = 2048;      // meeting counters behind the tile table
constexpr int kPairMinK = 4096;     // tiles this long are worth the meeting (its cost: a few microseconds)

constexpr int kXwWaves = 8;       // wavefronts of a gemm_xw workgroup (256 x 256 tiles)
constexpr int kXwThreads = kXwWaves * 64;


// Wavefronts that share one staging region of 32 KiB in the epilogue, per epilogue kind: the staging
// areas live in the operand buffers the last stage has released.  Kinds whose eight areas fit two
// regions leave a third buffer free, which then takes the next tile's W(1) ahead of time.
template <int EPI> struct Staging {
    static constexpr int SC = EPI == EPI_SWIGLU_FWD ? 96 : 64;   // columns per staging row
    static constexpr int SROW = SC * 2 + 16;                    // row stride in bytes
    static constexpr int WSTG = (EPI == EPI_SWIGLU_BWD ? 2 : 1) * 32 * SROW;   // bytes per wavefront
    static constexpr int RW = 32768 / WSTG < kXwWaves ? 32768 / WSTG : kXwWaves;
    static constexpr int REGIONS = (EPI == EPI_F32) ? 0 : (kXwWaves + RW - 1) / RW;
    static constexpr bool PREW1 = REGIONS <= 2;
    static_assert(REGIONS <= 3, "three operand buffers are free in the epilogue");
};

// compile-time loop: f(std::integral_constant<int, I>{}) for I = 0 .. N-1
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Accumulators held in a register array acc[strip][16-row half][16-column block].
template <int MTV> struct AccArray {
    f32x4 (&acc)[MTV > 0 ? MTV : 1][2][4];
    template <int TM> __device__ __forceinline__ void strip(f32x4 (&s)[2][4]) const {
#pragma unroll
        for (int mh = 0; mh < 2; mh++)
#pragma unroll
            for (int nb = 0; nb < 4; nb++) s[mh][nb] = acc[TM][mh][nb];
    }
};

// ---------------------------------------------------------------------------------------------
// Staged epilogues of the row-grouped GEMM (EPI_STORE, EPI_SWIGLU_FWD, EPI_SWIGLU_BWD).
// A.strip<tm>(s) hands over the accumulators of strip tm:
// s[mh][nb][r] = C[row (strip_first + strip_step tm)*32 + 16 mh + lane%16]
//                 [column 16 nb + 4*(lane/16) + r of the wavefront's 64 columns];
// MTV = strips of this wavefront that hold rows, LH = only the upper 16 rows of its last strip do.
// Results pass through the wave-private staging area stg and leave as 16-byte row segments.
// CAN_ADD: EPI_STORE may add to the destination (g.add); the old values of all strips then take
// 16 registers per strip, so kernels with many strips per wavefront compile it out.
// ---------------------------------------------------------------------------------------------
// What the staged epilogues need of the launch arguments, by value (a handful of scalars the compiler keeps in
// registers; a reference to the whole argument block has ended up in scratch memory in large kernels).
struct EpiArgs {
    void* out0;
    void* out1;
    void* out2;
    const bf16* aux_a;
    const bf16* aux_b;
    int N, ldo, add;
};
__device__ __forceinline__ EpiArgs epi_args(const GemmArgs& a) {
    return EpiArgs{a.out0, a.out1, a.out2, a.aux_a, a.aux_b, a.N, a.ldo, a.add};
}

template <int EPI, int MTV, bool LH, bool CAN_ADD, typename AccT>
__device__ __forceinline__ void xw_staged_epilogue(const EpiArgs g, const AccT& A,
                                                   char* stg, int rows, int row0, int n0, int f0,
                                                   int strip_first, int strip_step, int wn, int lane) {
    using SG = Staging<EPI>;
    constexpr int SROW = SG::SROW;                  // staging row stride in bytes
    constexpr int CPRS = SG::SC / 8;                // 16-byte chunks per staging row
    const int l16 = lane & 15, lg = lane >> 4;
    // SWIGLU_BWD stages the saved activations A and B of a strip in two areas of 32 x 64 values:
    // they are fetched as whole 128-byte row segments (one request per cache line instead of one
    // per 16 bytes in the accumulator layout), a strip ahead, picked up from LDS in the
    // accumulator layout, and replaced in place by dA and dB, which leave as row segments again.
    [[maybe_unused]] char* stgb = stg + 32 * SROW;
    [[maybe_unused]] uint4 av0, av1, av2, av3, bv0, bv1, bv2, bv3;
    // the 64 columns of a wavefront are inside N or outside as a whole (N is a multiple of 64)
    [[maybe_unused]] const bool cols_ok = n0 + wn * 64 < g.N;
#define UNIPOOL_LOAD_AB1(TMX, IT)                                                                  \
{                                                                                              \
    const int r_ = min((strip_first + strip_step * (TMX)) * 32 + (IT) * 8 + (lane >> 3), rows - 1);              \
    const size_t o_ = (size_t)(row0 + r_) * g.N + n0 + wn * 64 + (lane & 7) * 8;               \
    av##IT = *reinterpret_cast<const uint4*>(g.aux_a + o_);                                    \
    bv##IT = *reinterpret_cast<const uint4*>(g.aux_b + o_);                                    \
}
#define UNIPOOL_LOAD_AB(TMX)                                                                       \
UNIPOOL_LOAD_AB1(TMX, 0) UNIPOOL_LOAD_AB1(TMX, 1) UNIPOOL_LOAD_AB1(TMX, 2) UNIPOOL_LOAD_AB1(TMX, 3)
    if constexpr (EPI == EPI_SWIGLU_BWD && MTV > 0) {
        if (cols_ok) { UNIPOOL_LOAD_AB(0) }
    }
    // EPI_STORE adding to the destination: the old values of all strips are requested up front,
    // in the layout the row segments leave in, so that their latency is paid once per tile.
    [[maybe_unused]] uint4 oldv[CAN_ADD && MTV > 0 ? MTV : 1][4];
    if constexpr (EPI == EPI_STORE && CAN_ADD) {
        if (g.add) {
#pragma unroll
            for (int tm = 0; tm < MTV; tm++)
#pragma unroll
                for (int it = 0; it < 4; it++) {
                    const int id = it * 64 + lane;
                    const int rr = min((strip_first + strip_step * tm) * 32 + id / CPRS, rows - 1);
                    const int col = min(n0 + wn * 64 + (id % CPRS) * 8, g.N - 8);
                    oldv[tm][it] = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16*>(g.out0) +
                                                                   (size_t)(row0 + rr) * g.ldo + col);
                }
        }
    }
    static_for<0, MTV>([&](auto tm_c) __attribute__((always_inline)) {
        constexpr int tm = decltype(tm_c)::value;
        const int strip0 = (strip_first + strip_step * tm) * 32;     // first row of the strip inside the tile
        f32x4 acc_s[2][4];
        A.template strip<tm>(acc_s);
        // -- registers -> staging rows
        if constexpr (EPI == EPI_STORE) {
#pragma unroll
            for (int mh = 0; mh < (LH && tm == MTV - 1 ? 1 : 2); mh++)
#pragma unroll
                for (int nb = 0; nb < 4; nb++) {
                    const int c = 16 * nb + 4 * lg;
                    *reinterpret_cast<uint2*>(stg + (16 * mh + l16) * SROW + c * 2) =
                        pack4(acc_s[mh][nb][0], acc_s[mh][nb][1], acc_s[mh][nb][2], acc_s[mh][nb][3]);
                }
        } else if constexpr (EPI == EPI_SWIGLU_FWD) {
#pragma unroll
            for (int q = 0; q < (LH && tm == MTV - 1 ? 2 : 4); q++) {
                const int mh = q >> 1, nbg = q & 1;       // blocks nbg and 2 + nbg: gate and up of the same columns
                const int c = 16 * nbg + 4 * lg;
                char* srow = stg + (16 * mh + l16) * SROW;
                float a[4], b[4], h[4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    a[i] = acc_s[mh][nbg][i];
                    b[i] = acc_s[mh][2 + nbg][i];
                    h[i] = silu_f(a[i]) * b[i];
                }
                *reinterpret_cast<uint2*>(srow + c * 2) = pack4(a[0], a[1], a[2], a[3]);
                *reinterpret_cast<uint2*>(srow + (32 + c) * 2) = pack4(b[0], b[1], b[2], b[3]);
                *reinterpret_cast<uint2*>(srow + (64 + c) * 2) = pack4(h[0], h[1], h[2], h[3]);
            }
        } else {   // EPI_SWIGLU_BWD
            if (cols_ok) {
                const int so = (lane >> 3) * SROW + (lane & 7) * 16;
                *reinterpret_cast<uint4*>(stg + so) = av0;
                *reinterpret_cast<uint4*>(stgb + so) = bv0;
                *reinterpret_cast<uint4*>(stg + so + 8 * SROW) = av1;
                *reinterpret_cast<uint4*>(stgb + so + 8 * SROW) = bv1;
                *reinterpret_cast<uint4*>(stg + so + 16 * SROW) = av2;
                *reinterpret_cast<uint4*>(stgb + so + 16 * SROW) = bv2;
                *reinterpret_cast<uint4*>(stg + so + 24 * SROW) = av3;
                *reinterpret_cast<uint4*>(stgb + so + 24 * SROW) = bv3;
                if (tm + 1 < MTV) { UNIPOOL_LOAD_AB(tm + 1) }
            }
#pragma unroll
            for (int mh = 0; mh < (LH && tm == MTV - 1 ? 1 : 2); mh++)
#pragma unroll
                for (int nb = 0; nb < 4; nb++) {
                    const int c = 16 * nb + 4 * lg;                 // column inside the wave's 64
                    float da[4] = {0.f, 0.f, 0.f, 0.f}, db[4] = {0.f, 0.f, 0.f, 0.f};
                    // a lane overwrites exactly the eight bytes of A and of B it has read
                    uint2* pa = reinterpret_cast<uint2*>(stg + (16 * mh + l16) * SROW + c * 2);
                    uint2* pb = reinterpret_cast<uint2*>(stgb + (16 * mh + l16) * SROW + c * 2);
                    if (cols_ok) {
                        union { uint2 u; bf16 h[4]; } a4, b4;
                        a4.u = *pa;
                        b4.u = *pb;
#pragma unroll
                        for (int i = 0; i < 4; i++) {
                            const float a = (float)a4.h[i], b = (float)b4.h[i];
                            const float dh = acc_s[mh][nb][i];
                            const float sg = logistic_f(a);
                            da[i] = dh * b * sg * (1.0f + a * (1.0f - sg));
                            db[i] = dh * a * sg;
                        }
                    }
                    *pa = pack4(da[0], da[1], da[2], da[3]);
                    *pb = pack4(db[0], db[1], db[2], db[3]);
                }
        }
        // -- staging rows -> global, 16 bytes per lane
        constexpr int NCH = (EPI == EPI_SWIGLU_BWD ? 2 : 1) * CPRS;     // chunks per output row
#pragma unroll
        for (int it = 0; it < 32 * NCH / 64; it++) {
            const int id = it * 64 + lane;
            const int srow = id / NCH;
            const int ch = id % NCH;
            const int rr = strip0 + srow;
            if (rr >= rows) continue;
            const size_t grow = (size_t)(row0 + rr);
            if constexpr (EPI == EPI_STORE) {
                const uint4 v = *reinterpret_cast<const uint4*>(stg + srow * SROW + ch * 16);
                const int col = n0 + wn * 64 + ch * 8;
                if (col < g.N) {
                    bf16* dst = reinterpret_cast<bf16*>(g.out0) + grow * g.ldo + col;
                    if (CAN_ADD && g.add) {
                        union { uint4 u; bf16 h[8]; } o, n;
                        o.u = oldv[tm][it];
                        n.u = v;
#pragma unroll
                        for (int i = 0; i < 8; i++) n.h[i] = (bf16)((float)o.h[i] + (float)n.h[i]);
                        *reinterpret_cast<uint4*>(dst) = n.u;
                    } else {
                        *reinterpret_cast<uint4*>(dst) = v;
                    }
                }
            } else if constexpr (EPI == EPI_SWIGLU_FWD) {
                const uint4 v = *reinterpret_cast<const uint4*>(stg + srow * SROW + ch * 16);
                const int which = ch >> 2;
                const int col = f0 + wn * 32 + (ch & 3) * 8;
                if (col < g.N) {
                    bf16* base = reinterpret_cast<bf16*>(which == 0 ? g.out0 : (which == 1 ? g.out1 : g.out2));
                    *reinterpret_cast<uint4*>(base + grow * g.ldo + col) = v;
                }
            } else {
                const int which = ch >> 3;
                const uint4 v = *reinterpret_cast<const uint4*>((which ? stgb : stg) + srow * SROW + (ch & 7) * 16);
                const int col = n0 + wn * 64 + (ch & 7) * 8;
                if (col < g.N) {
                    bf16* dst = reinterpret_cast<bf16*>(g.out0) + grow * g.ldo + which * g.N + col;
                    *reinterpret_cast<uint4*>(dst) = v;
                }
            }
        }
    });
#undef UNIPOOL_LOAD_AB
#undef UNIPOOL_LOAD_AB1
}

}  // namespace

}  // namespace unipool
