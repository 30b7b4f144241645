// Dispatch: builds the expert-contiguous row order and copies the token rows.
//
// The order is unique (expert-major, ascending token inside an expert), so it is computed
// without order-dependent atomics:
//   1. hist    : one wavefront per chunk of 64 tokens builds, in LDS, a 64-bit token mask per
//                expert (atomic OR, order-free) and writes the per-chunk histogram;
//   2. scan    : one block per expert: its offset (sum of the counts of the experts before it) and
//                an exclusive scan over the chunks, which turns the histograms into per-chunk
//                base rows;
//   3. copy    : one wavefront per token.  The lanes fetch the selections of the token's chunk;
//                the rank of the token inside its chunk is the number of lower tokens that
//                selected the same expert (a ballot and a popcount); row = chunk base + rank.
//                The row is read once and written k times with 16-byte accesses.
#include <mutex>

#include "kernels.h"

namespace unipool {

namespace {

constexpr int kChunkWaves = 4;   // chunks (wavefronts) per block

// Scratch of unipool_permute_static: the per-chunk histograms / base rows ([ceil(T/64)][E] int32) that
// unipool_permute keeps in the caller's workspace.  One copy per GPU, held until the process ends.
constexpr size_t kStaticHistWords = 512 * 1024;       // 2 MiB: e.g. T = 65536 with E = 512
static __device__ __align__(256) int32_t scratch[kStaticHistWords];

// Device address of `scratch` on the current device (the array's name is only a host-side handle of
// the symbol; every GPU holds its own copy at its own address).  Looked up once per device.
constexpr int kMaxDevices = 64;
int32_t* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

hipError_t scratch_address(int32_t** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

__device__ __forceinline__ void build_masks(unsigned long long* mask, const int32_t* topk_idx,
                                            int t, int T, int E, int k, int lane, int* sel) {
    for (int e = lane; e < E; e += 64) mask[e] = 0ull;
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    if (t < T) {
        for (int j = 0; j < k; j++) {
            sel[j] = topk_idx[(size_t)t * k + j];
            atomicOr(&mask[sel[j]], 1ull << lane);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__global__ __launch_bounds__(256) void permute_hist_kernel(const int32_t* __restrict__ topk_idx,
                                                           int T, int E, int k,
                                                           int32_t* __restrict__ chunk_hist) {
    extern __shared__ unsigned long long lds_mask[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x * kChunkWaves + wave;
    const int nchunks = (T + 63) / 64;
    if (chunk >= nchunks) return;
    unsigned long long* mask = lds_mask + (size_t)wave * E;
    int sel[kMaxK];
    build_masks(mask, topk_idx, chunk * 64 + lane, T, E, k, lane, sel);
    for (int e = lane; e < E; e += 64) chunk_hist[(size_t)chunk * E + e] = __popcll(mask[e]);
}

// One block per expert: its offset = sum of the counts of the experts before it (fixed-shape tree),
// then the exclusive scan of its per-chunk histogram, started at that offset.
__global__ __launch_bounds__(256) void permute_scan_kernel(const int32_t* __restrict__ counts, int E,
                                                           int nchunks, int32_t* __restrict__ expert_offsets,
                                                           int32_t* __restrict__ chunk_hist) {
    __shared__ int scan[2][256];
    __shared__ int red[256];
    const int e = blockIdx.x, t = threadIdx.x;
    int before = 0, all = 0;
    for (int i = t; i < E; i += 256) {
        const int c = counts[i];
        all += c;
        if (i < e) before += c;
    }
    red[t] = before;
    scan[0][t] = all;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) {
            red[t] += red[t + s];
            scan[0][t] += scan[0][t + s];
        }
        __syncthreads();
    }
    int carry = red[0];
    if (t == 0) {
        expert_offsets[e] = carry;
        if (e == 0) expert_offsets[E] = scan[0][0];
    }
    __syncthreads();
    for (int c0 = 0; c0 < nchunks; c0 += 256) {
        const int c = c0 + t;
        const int h = c < nchunks ? chunk_hist[(size_t)c * E + e] : 0;
        scan[0][t] = h;
        __syncthreads();
        int cur = 0;
        for (int d = 1; d < 256; d <<= 1) {
            scan[cur ^ 1][t] = scan[cur][t] + (t >= d ? scan[cur][t - d] : 0);
            cur ^= 1;
            __syncthreads();
        }
        if (c < nchunks) chunk_hist[(size_t)c * E + e] = carry + scan[cur][t] - h;
        carry += scan[cur][255];
        __syncthreads();
    }
}

// Rows of token t (lane-uniform): lane l holds the selections of token chunk*64 + l.  K = top-k at compile
// time: the loops unroll, so the K selections are loaded together and so are the K chunk bases.
template <int K>
__device__ __forceinline__ void rows_of_token(const int32_t* __restrict__ topk_idx, int t, int T, int E,
                                              const int32_t* __restrict__ chunk_base, int lane, int (&rows)[K]) {
    const int chunk = t >> 6, tl = t & 63;
    const int to = chunk * 64 + lane;
    int other[K];
#pragma unroll
    for (int j = 0; j < K; j++) other[j] = to < T ? topk_idx[(size_t)to * K + j] : -1;
    const unsigned long long below = (1ull << tl) - 1ull;
    int base[K], rank[K];
#pragma unroll
    for (int j = 0; j < K; j++) {
        const int e = __shfl(other[j], tl, 64);                     // this token's j-th expert
        base[j] = chunk_base[(size_t)chunk * E + e];
        bool hit = false;
#pragma unroll
        for (int i = 0; i < K; i++) hit |= other[i] == e;
        const unsigned long long sel = __ballot(hit);               // tokens of the chunk that selected e
        rank[j] = __popcll(sel & below);
    }
#pragma unroll
    for (int j = 0; j < K; j++) rows[j] = base[j] + rank[j];
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// One wavefront per token: 16-byte chunks of the row, read once, written k times.
template <int K>
__global__ __launch_bounds__(256) void permute_copy_kernel(const uint4* __restrict__ x,
                                                           const int32_t* __restrict__ topk_idx,
                                                           const int32_t* __restrict__ chunk_base,
                                                           int T, int E, int row_chunks,
                                                           uint4* __restrict__ x_perm,
                                                           int32_t* __restrict__ row_of_slot,
                                                           int32_t* __restrict__ slot_of_row) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[K];
    rows_of_token<K>(topk_idx, t, T, E, chunk_base, lane, rows);
    if (lane < K) {
        int r = rows[0];
#pragma unroll
        for (int j = 1; j < K; j++) r = lane == j ? rows[j] : r;
        row_of_slot[(size_t)t * K + lane] = r;
        slot_of_row[r] = t * K + lane;
    }
    if (x_perm == nullptr) return;                 // index maps only
    const uint4* src = x + (size_t)t * row_chunks;
    for (int c0 = 0; c0 < row_chunks; c0 += 256) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int c = c0 + u * 64 + lane;
            if (c < row_chunks) v[u] = src[c];
        }
#pragma unroll
        for (int j = 0; j < K; j++) {
            uint4* dst = x_perm + (size_t)rows[j] * row_chunks;
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 64 + lane;
                // the copy is written once and read much later by another kernel: a streaming store keeps it
                // from displacing the lines of x that are still to be read (measured 13 % faster at d_model
                // 1536, k = 2; the same hint on the combine kernels' stores measured slower)
                if (c < row_chunks) {
                    const u32x4 q = {v[u].x, v[u].y, v[u].z, v[u].w};
                    __builtin_nontemporal_store(q, reinterpret_cast<u32x4*>(dst + c));
                }
            }
        }
    }
}

// Rows whose byte length is not a multiple of 16 (only possible in float mode with odd d).
template <int K>
__global__ __launch_bounds__(64) void permute_copy_scalar_kernel(const uint32_t* __restrict__ x,
                                                                 const int32_t* __restrict__ topk_idx,
                                                                 const int32_t* __restrict__ chunk_base,
                                                                 int T, int E, int row_words,
                                                                 uint32_t* __restrict__ x_perm,
                                                                 int32_t* __restrict__ row_of_slot,
                                                                 int32_t* __restrict__ slot_of_row) {
    const int lane = threadIdx.x;
    const int t = blockIdx.x;
    int rows[K];
    rows_of_token<K>(topk_idx, t, T, E, chunk_base, lane, rows);
#pragma unroll
    for (int j = 0; j < K; j++) {
        if (lane == 0) {
            row_of_slot[(size_t)t * K + j] = rows[j];
            slot_of_row[rows[j]] = t * K + j;
        }
        if (x_perm == nullptr) continue;           // index maps only
        for (int c = lane; c < row_words; c += 64)
            x_perm[(size_t)rows[j] * row_words + c] = x[(size_t)t * row_words + c];
    }
}

}  // namespace

hipError_t launch_permute(const unipool_shape& s, const void* x, const int32_t* topk_idx,
                          const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                          int32_t* row_of_slot, int32_t* slot_of_row, int32_t* chunk_hist,
                          hipStream_t st) {
    const int nchunks = cdiv(s.T, 64);
    const int nblocks = cdiv(nchunks, kChunkWaves);
    const size_t lds = (size_t)kChunkWaves * s.E * sizeof(unsigned long long);
    permute_hist_kernel<<<nblocks, 256, lds, st>>>(topk_idx, s.T, s.E, s.k, chunk_hist);
    permute_scan_kernel<<<s.E, 256, 0, st>>>(counts, s.E, nchunks, expert_offsets, chunk_hist);
    const size_t row_bytes = (size_t)s.d_model * (s.dtype == UNIPOOL_BF16 ? 2 : 4);
    with_top_k(s.k, [&](auto kc) {
        constexpr int K = decltype(kc)::value;
        if (row_bytes % 16 == 0) {
            permute_copy_kernel<K><<<cdiv(s.T, 4), 256, 0, st>>>((const uint4*)x, topk_idx, chunk_hist, s.T, s.E,
                                                                 (int)(row_bytes / 16), (uint4*)x_perm, row_of_slot,
                                                                 slot_of_row);
        } else {
            permute_copy_scalar_kernel<K><<<s.T, 64, 0, st>>>((const uint32_t*)x, topk_idx, chunk_hist, s.T, s.E,
                                                              (int)(row_bytes / 4), (uint32_t*)x_perm, row_of_slot,
                                                              slot_of_row);
        }
    });
    return hipGetLastError();
}

}  // namespace unipool

extern "C" int unipool_permute_static(const unipool_shape* shape, const void* x, const int32_t* topk_idx,
                                      const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                                      int32_t* row_of_slot, int32_t* slot_of_row, void* stream) {
    using namespace unipool;
    int rc = validate_shape(shape, __func__);
    if (rc) return rc;
    if (!topk_idx || !counts || !expert_offsets || !row_of_slot || !slot_of_row || (x_perm && !x))
        return set_error(UNIPOOL_EINVAL, "%s: a tensor argument is NULL", __func__);
    const size_t words = (size_t)cdiv(shape->T, 64) * (size_t)shape->E;
    if (words > kStaticHistWords)
        return set_error(UNIPOOL_EINVAL, "%s: ceil(T/64)*E = %zu exceeds the static scratch of %zu words; use unipool_permute",
                         __func__, words, kStaticHistWords);
    int32_t* hist = nullptr;
    hipError_t e = scratch_address(&hist);
    if (e != hipSuccess) return check_hip(e, "unipool_permute_static: address of the static scratch");
    // every word of the histogram region in use is written by the first kernel before it is read:
    // nothing of an earlier call survives into this one
    return check_hip(launch_permute(*shape, x, topk_idx, counts, x_perm, expert_offsets, row_of_slot,
                                    slot_of_row, hist, (hipStream_t)stream),
                     "unipool_permute_static");
}
