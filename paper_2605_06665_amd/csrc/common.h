// Shared declarations of the UniPool HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "unipool.h"

namespace unipool {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWave = 64;
constexpr int kMaxE = 512;
constexpr int kMaxK = 8;

// ---- error reporting (host) ------------------------------------------------
int set_error(int code, const char* fmt, ...);
int check_hip(hipError_t e, const char* what);
// Range and alignment checks every entry point runs on its shape before anything is launched.
int validate_shape(const unipool_shape* s, const char* fn);

// ---- top-k as a compile-time constant (host) --------------------------------
// The per-token kernels loop over the k copies of a token; with k known at compile time these loops unroll,
// the rows of the copies sit in registers and their loads are in flight together.
// Calls f with k as a compile-time constant (1 <= k <= kMaxK, checked at the boundary).
template <class F>
inline void with_top_k(int k, F f) {
    static_assert(kMaxK == 8, "one case per admissible k");
    switch (k) {
        case 1: f(std::integral_constant<int, 1>{}); break;
        case 2: f(std::integral_constant<int, 2>{}); break;
        case 3: f(std::integral_constant<int, 3>{}); break;
        case 4: f(std::integral_constant<int, 4>{}); break;
        case 5: f(std::integral_constant<int, 5>{}); break;
        case 6: f(std::integral_constant<int, 6>{}); break;
        case 7: f(std::integral_constant<int, 7>{}); break;
        default: f(std::integral_constant<int, 8>{}); break;
    }
}

// ---- scalar conversions (device) --------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE

// 1 / (1 + e^-a) with the hardware reciprocal (1 ulp) instead of an IEEE division
__device__ __forceinline__ float logistic_f(float a) { return __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }
__device__ __forceinline__ float silu_f(float a) { return a * logistic_f(a); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---- workspace layout ---------------------------------------------------------
// The workspace is cut into fixed regions, all 256-byte aligned, sized from the shape.
struct WsLayout {
    size_t zeros;          // 256 bytes of zeros (address for masked direct-to-LDS loads)
    size_t tile_meta;      // int32: [0] number of row tiles, then 3 ints per tile
    size_t chunk_hist;     // int32 [ceil(T/64)][E]   permute: per-64-token histograms/bases
    size_t psum_part;      // float [router blocks][E] partial score sums
    size_t dsigma_part;    // float [router blocks]
    size_t dz;             // act   [T][E]  router backward logits gradient
    size_t ptr_tab;        // 5 device pointers for the single-layer weight gradient
    size_t wpart;          // float [split][E][d]  router weight gradient partials
    size_t total;
};
WsLayout ws_layout(const unipool_shape& s);

constexpr int kRouterTokensPerBlock = 64;   // tokens per block in the per-token router kernels
constexpr int kRouteBwdSplit = 64;          // max row chunks of the router weight-gradient reduction

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

}  // namespace unipool
