// C ABI of the UniPool library: argument checks, workspace carving and kernel dispatch.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "kernels.h"

namespace unipool {

namespace {
thread_local char g_err[512] = "no error";

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }
}  // namespace
size_t align_up_256(size_t v) { return (v + 255) & ~(size_t)255; }
namespace {

// Debugging builds (-DUNIPOOL_DEBUG_SWITCHES) read two switches from the environment; a regular build has
// none and keeps no state.  UNIPOOL_FORCE_NAIVE=1 sends bfloat16 contractions to the plain
// one-thread-per-element kernels; UNIPOOL_UNFUSED_ROUTER=1 keeps the logits GEMM and the selection in
// separate kernels.
#ifdef UNIPOOL_DEBUG_SWITCHES
bool env_switch(const char* name) {
    const char* e = getenv(name);
    return e && e[0] == '1';
}
bool force_naive() {
    static const bool v = env_switch("UNIPOOL_FORCE_NAIVE");
    return v;
}
bool unfused_router() {
    static const bool v = env_switch("UNIPOOL_UNFUSED_ROUTER");
    return v;
}
#else
constexpr bool force_naive() { return false; }
constexpr bool unfused_router() { return false; }
#endif

__global__ void fill_zero_kernel(uint32_t* p, size_t words) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

__global__ void set_ptrs_kernel(void** table, const void* p0, const void* p1, const void* p2,
                                const void* p3, const void* p4) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        table[0] = const_cast<void*>(p0);
        table[1] = const_cast<void*>(p1);
        table[2] = const_cast<void*>(p2);
        table[3] = const_cast<void*>(p3);
        table[4] = const_cast<void*>(p4);
    }
}
}  // namespace

int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return UNIPOOL_OK;
    return set_error(UNIPOOL_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    const size_t words = bytes / 4;
    if (words == 0) return hipSuccess;
    fill_zero_kernel<<<(unsigned)((words + 255) / 256), 256, 0, st>>>((uint32_t*)p, words);
    return hipGetLastError();
}

hipError_t launch_set_ptrs(void** table, const void* p0, const void* p1, const void* p2,
                           const void* p3, const void* p4, hipStream_t st) {
    set_ptrs_kernel<<<1, 64, 0, st>>>(table, p0, p1, p2, p3, p4);
    return hipGetLastError();
}

WsLayout ws_layout(const unipool_shape& s) {
    WsLayout w;
    const size_t T = (size_t)s.T, E = (size_t)s.E, d = (size_t)s.d_model;
    const size_t S = T * (size_t)s.k;
    const size_t rblocks = (T + kRouterTokensPerBlock - 1) / kRouterTokensPerBlock;
    const size_t act = s.dtype == UNIPOOL_BF16 ? 2 : 4;
    size_t o = 0;
    w.zeros = o;       o += 256;
    w.tile_meta = o;   o += align_up((4096 + 4 * (S / 256 + 2 * E + T / 128 + 16)) * sizeof(int32_t));
    w.chunk_hist = o;  o += align_up(((T + 63) / 64) * E * sizeof(int32_t));
    w.psum_part = o;   o += align_up(rblocks * E * sizeof(float));
    w.dsigma_part = o; o += align_up(rblocks * E * sizeof(int32_t));   // also holds count partials
    w.dz = o;          o += align_up(T * E * (act > 4 ? act : 4));     // logits (float) or dz
    w.ptr_tab = o;     o += 256;
    w.wpart = o;       o += align_up((size_t)kRouteBwdSplit * E * d * sizeof(float));
    w.total = o;
    return w;
}

int validate_shape(const unipool_shape* s, const char* fn) {
    if (!s) return set_error(UNIPOOL_EINVAL, "%s: shape is NULL", fn);
    if (s->dtype != UNIPOOL_F32 && s->dtype != UNIPOOL_BF16)
        return set_error(UNIPOOL_EINVAL, "%s: dtype %d is neither UNIPOOL_F32 nor UNIPOOL_BF16", fn, s->dtype);
    if (s->T < 1 || s->d_model < 1 || s->d_ff < 1)
        return set_error(UNIPOOL_EINVAL, "%s: T, d_model, d_ff must be positive (T=%d d=%d f=%d)", fn, s->T,
                         s->d_model, s->d_ff);
    if (s->E < 1 || s->E > kMaxE) return set_error(UNIPOOL_EINVAL, "%s: E=%d outside [1, %d]", fn, s->E, kMaxE);
    if (s->k < 1 || s->k > kMaxK || s->k > s->E)
        return set_error(UNIPOOL_EINVAL, "%s: k=%d outside [1, min(%d, E=%d)]", fn, s->k, kMaxK, s->E);
    if ((long long)s->T * s->k >= (1LL << 31))
        return set_error(UNIPOOL_EINVAL, "%s: T*k does not fit int32", fn);
    if (s->dtype == UNIPOOL_BF16 && (s->d_model % 64 != 0 || s->d_ff % 64 != 0))
        return set_error(UNIPOOL_EINVAL, "%s: bfloat16 mode needs d_model and d_ff to be multiples of 64 (d=%d f=%d)",
                         fn, s->d_model, s->d_ff);
    if (s->router != UNIPOOL_ROUTER_NORM && s->router != UNIPOOL_ROUTER_SOFTMAX)
        return set_error(UNIPOOL_EINVAL, "%s: router %d is neither UNIPOOL_ROUTER_NORM nor UNIPOOL_ROUTER_SOFTMAX", fn,
                         s->router);
    if (!(s->sigma > 0.f)) return set_error(UNIPOOL_EINVAL, "%s: sigma must be positive", fn);
    if (!(s->eps >= 0.f)) return set_error(UNIPOOL_EINVAL, "%s: eps must be non-negative", fn);
    return UNIPOOL_OK;
}

namespace {

int need_ws(const unipool_shape* s, void* ws, size_t ws_bytes, const char* fn) {
    if (!ws) return set_error(UNIPOOL_EWORKSPACE, "%s: workspace is NULL", fn);
    if (((uintptr_t)ws & 255) != 0) return set_error(UNIPOOL_EWORKSPACE, "%s: workspace is not 256-byte aligned", fn);
    const size_t need = ws_layout(*s).total;
    if (ws_bytes < need)
        return set_error(UNIPOOL_EWORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, ws_bytes, need);
    return UNIPOOL_OK;
}

#define REQUIRE_PTR(p)                                                                  \
    if (!(p)) return unipool::set_error(UNIPOOL_EINVAL, "%s: argument %s is NULL", __func__, #p)
#define PROLOGUE()                                                            \
    {                                                                         \
        int rc_ = unipool::validate_shape(shape, __func__);                         \
        if (rc_) return rc_;                                                  \
    }
#define NEED_WS()                                                             \
    {                                                                         \
        int rc_ = unipool::need_ws(shape, ws, ws_bytes, __func__);            \
        if (rc_) return rc_;                                                  \
    }

}  // namespace
}  // namespace unipool

using namespace unipool;

extern "C" {

size_t unipool_workspace_bytes(const unipool_shape* shape) {
    if (validate_shape(shape, __func__) != UNIPOOL_OK) return 0;
    return ws_layout(*shape).total;
}

const char* unipool_last_error(void) { return g_err; }

int unipool_version(void) { return 200; }

int unipool_fast_path(const unipool_shape* shape) {
    PROLOGUE();
    return (mfma_ffn_supported(*shape) ? UNIPOOL_FAST_EXPERTS : 0) | (mfma_router_supported(*shape) ? UNIPOOL_FAST_ROUTER : 0) |
           (router_fused_supported(*shape) ? UNIPOOL_FAST_ROUTER_FUSED : 0);
}

int unipool_route(const unipool_shape* shape, const void* x, const void* w_router,
                  int32_t* topk_idx, float* topk_gate, float* logits, int32_t* counts, float* psum,
                  void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(x); REQUIRE_PTR(w_router); REQUIRE_PTR(topk_idx); REQUIRE_PTR(topk_gate);
    REQUIRE_PTR(counts); REQUIRE_PTR(psum);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    char* base = (char*)ws;
    hipStream_t st = (hipStream_t)stream;
    float* z = logits ? logits : (float*)(base + w.dz);
    hipError_t e;
    if (router_fused_supported(*shape) && !force_naive() && !unfused_router()) {
        // logits, scores, top-k and block statistics in one kernel; then the sum over the blocks
        int32_t* cnt_part = (int32_t*)(base + w.dsigma_part);
        float* psum_part = (float*)(base + w.psum_part);
        e = router_fused(*shape, x, w_router, z, topk_idx, topk_gate, cnt_part, psum_part, st);
        if (e != hipSuccess) return check_hip(e, "unipool_route: fused router");
        return check_hip(launch_route_finalize(*shape, cnt_part, psum_part, counts, psum, st),
                         "unipool_route: statistics");
    }
    if (mfma_router_supported(*shape) && !force_naive())
        e = mfma_logits(*shape, x, w_router, z, (int32_t*)(base + w.tile_meta), st);
    else
        e = naive_logits(*shape, x, w_router, z, st);
    if (e != hipSuccess) return check_hip(e, "unipool_route: logits");
    e = launch_route_score_topk(*shape, z, topk_idx, topk_gate, counts, psum,
                                (int32_t*)(base + w.dsigma_part), (float*)(base + w.psum_part), st);
    return check_hip(e, "unipool_route: score/top-k");
}

int unipool_route_bwd(const unipool_shape* shape, const void* x, const void* w_router,
                      const float* logits, const int32_t* topk_idx, const float* dgate,
                      const float* aux_coef, float* d_w_router, float* d_sigma, void* dx,
                      int dx_accumulate, void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(x); REQUIRE_PTR(w_router); REQUIRE_PTR(logits); REQUIRE_PTR(topk_idx);
    REQUIRE_PTR(dgate); REQUIRE_PTR(d_w_router); REQUIRE_PTR(d_sigma); REQUIRE_PTR(dx);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    char* base = (char*)ws;
    hipStream_t st = (hipStream_t)stream;
    void* dz = base + w.dz;
    hipError_t e = launch_route_bwd_dz(*shape, logits, topk_idx, dgate, aux_coef, dz,
                                       (float*)(base + w.dsigma_part), d_sigma, st);
    if (e != hipSuccess) return check_hip(e, "unipool_route_bwd: dz");
    if (mfma_router_supported(*shape) && !force_naive()) {
        e = mfma_route_bwd_mm(*shape, x, w_router, dz, d_w_router, dx, dx_accumulate,
                              (int32_t*)(base + w.tile_meta), (float*)(base + w.wpart),
                              base + w.zeros, st);
    } else {
        e = naive_route_bwd_mm(*shape, x, w_router, dz, d_w_router, dx, dx_accumulate, st);
    }
    return check_hip(e, "unipool_route_bwd: contractions");
}

int unipool_permute(const unipool_shape* shape, const void* x, const int32_t* topk_idx,
                    const int32_t* counts, void* x_perm, int32_t* expert_offsets,
                    int32_t* row_of_slot, int32_t* slot_of_row, void* ws, size_t ws_bytes,
                    void* stream) {
    PROLOGUE();
    REQUIRE_PTR(topk_idx); REQUIRE_PTR(counts);
    REQUIRE_PTR(expert_offsets); REQUIRE_PTR(row_of_slot); REQUIRE_PTR(slot_of_row);
    if (x_perm) REQUIRE_PTR(x);                       // x_perm == NULL: index maps only
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    hipError_t e = launch_permute(*shape, x, topk_idx, counts, x_perm, expert_offsets, row_of_slot,
                                  slot_of_row, (int32_t*)((char*)ws + w.chunk_hist),
                                  (hipStream_t)stream);
    return check_hip(e, "unipool_permute");
}

int unipool_expert_ffn_fwd(const unipool_shape* shape, const void* x_perm,
                           const int32_t* expert_offsets, const void* w_gate_up, const void* w_down,
                           void* act_a, void* act_b, void* act_h, void* y_perm, void* ws,
                           size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(x_perm); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(w_gate_up); REQUIRE_PTR(w_down);
    REQUIRE_PTR(act_a); REQUIRE_PTR(act_b); REQUIRE_PTR(act_h); REQUIRE_PTR(y_perm);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (mfma_ffn_supported(*shape) && !force_naive())
        e = mfma_ffn_fwd(*shape, x_perm, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h,
                         y_perm, (int32_t*)((char*)ws + w.tile_meta), st);
    else
        e = naive_ffn_fwd(*shape, x_perm, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h,
                          y_perm, st);
    return check_hip(e, "unipool_expert_ffn_fwd");
}

int unipool_expert_ffn_fwd_gather(const unipool_shape* shape, const void* x, const int32_t* slot_of_row,
                                  const int32_t* expert_offsets, const void* w_gate_up, const void* w_down,
                                  void* act_a, void* act_b, void* act_h, void* y_perm, void* ws,
                                  size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(x); REQUIRE_PTR(slot_of_row); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(w_gate_up);
    REQUIRE_PTR(w_down); REQUIRE_PTR(act_a); REQUIRE_PTR(act_b); REQUIRE_PTR(act_h); REQUIRE_PTR(y_perm);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (mfma_ffn_supported(*shape) && !force_naive())
        e = mfma_ffn_fwd(*shape, x, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h, y_perm,
                         (int32_t*)((char*)ws + w.tile_meta), st, slot_of_row);
    else
        e = naive_ffn_fwd(*shape, x, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h, y_perm, st,
                          slot_of_row);
    return check_hip(e, "unipool_expert_ffn_fwd_gather");
}

int unipool_expert_ffn_recompute(const unipool_shape* shape, const void* x_perm,
                                 const int32_t* expert_offsets, const void* w_gate_up,
                                 void* act_a, void* act_b, void* act_h, void* ws, size_t ws_bytes,
                                 void* stream) {
    PROLOGUE();
    REQUIRE_PTR(x_perm); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(w_gate_up);
    REQUIRE_PTR(act_a); REQUIRE_PTR(act_b); REQUIRE_PTR(act_h);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (mfma_ffn_supported(*shape) && !force_naive())
        e = mfma_ffn_gate_up(*shape, x_perm, expert_offsets, w_gate_up, act_a, act_b, act_h,
                             (int32_t*)((char*)ws + w.tile_meta), st);
    else
        e = naive_ffn_gate_up(*shape, x_perm, expert_offsets, w_gate_up, act_a, act_b, act_h, st);
    return check_hip(e, "unipool_expert_ffn_recompute");
}

int unipool_expert_ffn_bwd(const unipool_shape* shape, const void* dy_perm, const void* x_perm,
                           const void* act_a, const void* act_b, const void* act_h,
                           const int32_t* expert_offsets, const void* w_gate_up, const void* w_down,
                           void* dx_perm, void* d_act, float* d_w_gate_up, float* d_w_down,
                           void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(dy_perm); REQUIRE_PTR(x_perm); REQUIRE_PTR(act_a); REQUIRE_PTR(act_b);
    REQUIRE_PTR(expert_offsets); REQUIRE_PTR(w_gate_up); REQUIRE_PTR(w_down); REQUIRE_PTR(dx_perm);
    REQUIRE_PTR(d_act);
    if ((d_w_gate_up == nullptr) != (d_w_down == nullptr))
        return set_error(UNIPOOL_EINVAL, "%s: d_w_gate_up and d_w_down must both be given or both be NULL", __func__);
    if (d_w_gate_up) REQUIRE_PTR(act_h);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    char* base = (char*)ws;
    hipStream_t st = (hipStream_t)stream;
    const bool mfma = mfma_ffn_supported(*shape) && !force_naive();
    hipError_t e;
    if (mfma)
        e = mfma_ffn_dgrad(*shape, dy_perm, act_a, act_b, expert_offsets, w_gate_up, w_down, dx_perm,
                           d_act, (int32_t*)(base + w.tile_meta), st);
    else
        e = naive_ffn_dgrad(*shape, dy_perm, act_a, act_b, expert_offsets, w_gate_up, w_down, dx_perm,
                            d_act, st);
    if (e != hipSuccess) return check_hip(e, "unipool_expert_ffn_bwd: dgrad");
    if (!d_w_gate_up) return UNIPOOL_OK;
    void** tab = (void**)(base + w.ptr_tab);
    e = launch_set_ptrs(tab, x_perm, d_act, act_h, dy_perm, expert_offsets, st);
    if (e != hipSuccess) return check_hip(e, "unipool_expert_ffn_bwd: pointer table");
    if (mfma) {
        e = launch_fill_zero(base + w.zeros, 256, st);
        if (e != hipSuccess) return check_hip(e, "unipool_expert_ffn_bwd: zero page");
        e = mfma_ffn_wgrad(*shape, 1, tab + 0, tab + 1, tab + 2, tab + 3,
                           (const int32_t* const*)(tab + 4), d_w_gate_up, d_w_down, 1,
                           base + w.zeros, st);
    } else {
        e = naive_ffn_wgrad(*shape, 1, tab + 0, tab + 1, tab + 2, tab + 3,
                            (const int32_t* const*)(tab + 4), d_w_gate_up, d_w_down, 1, st);
    }
    return check_hip(e, "unipool_expert_ffn_bwd: wgrad");
}

int unipool_expert_wgrad(const unipool_shape* shape, int n_layers, const void* const* x_perm_l,
                         const void* const* d_act_l, const void* const* act_h_l,
                         const void* const* dy_perm_l, const int32_t* const* expert_offsets_l,
                         float* d_w_gate_up, float* d_w_down, int accumulate, void* ws,
                         size_t ws_bytes, void* stream) {
    PROLOGUE();
    if (n_layers < 1 || n_layers > 256)
        return set_error(UNIPOOL_EINVAL, "%s: n_layers=%d outside [1, 256]", __func__, n_layers);
    REQUIRE_PTR(x_perm_l); REQUIRE_PTR(d_act_l); REQUIRE_PTR(act_h_l); REQUIRE_PTR(dy_perm_l);
    REQUIRE_PTR(expert_offsets_l); REQUIRE_PTR(d_w_gate_up); REQUIRE_PTR(d_w_down);
    NEED_WS();
    const WsLayout w = ws_layout(*shape);
    char* base = (char*)ws;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (mfma_ffn_supported(*shape) && !force_naive()) {
        e = launch_fill_zero(base + w.zeros, 256, st);
        if (e != hipSuccess) return check_hip(e, "unipool_expert_wgrad: zero page");
        e = mfma_ffn_wgrad(*shape, n_layers, x_perm_l, d_act_l, act_h_l, dy_perm_l, expert_offsets_l,
                           d_w_gate_up, d_w_down, accumulate, base + w.zeros, st);
    } else {
        e = naive_ffn_wgrad(*shape, n_layers, x_perm_l, d_act_l, act_h_l, dy_perm_l, expert_offsets_l,
                            d_w_gate_up, d_w_down, accumulate, st);
    }
    return check_hip(e, "unipool_expert_wgrad");
}

int unipool_combine(const unipool_shape* shape, const void* y_perm, const int32_t* row_of_slot,
                    const float* gate, void* out, void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(y_perm); REQUIRE_PTR(row_of_slot); REQUIRE_PTR(out);
    (void)ws; (void)ws_bytes;
    return check_hip(launch_combine(*shape, y_perm, row_of_slot, gate, out, (hipStream_t)stream),
                     "unipool_combine");
}

int unipool_combine_bwd(const unipool_shape* shape, const void* dout, const void* y_perm,
                        const int32_t* row_of_slot, const float* gate, void* dy_perm, float* dgate,
                        void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    REQUIRE_PTR(dout); REQUIRE_PTR(y_perm); REQUIRE_PTR(row_of_slot); REQUIRE_PTR(gate);
    REQUIRE_PTR(dy_perm); REQUIRE_PTR(dgate);
    (void)ws; (void)ws_bytes;
    return check_hip(launch_combine_bwd(*shape, dout, y_perm, row_of_slot, gate, dy_perm, dgate,
                                        (hipStream_t)stream),
                     "unipool_combine_bwd");
}

int unipool_pool_aux_loss(const unipool_shape* shape, const int32_t* counts, const float* psum,
                          const float* fbar_in, int32_t* pool_counts, float* fbar_out, float* loss,
                          float* aux_coef, void* ws, size_t ws_bytes, void* stream) {
    PROLOGUE();
    if (shape->L < 1) return set_error(UNIPOOL_EINVAL, "%s: L=%d must be positive", __func__, shape->L);
    REQUIRE_PTR(counts); REQUIRE_PTR(psum); REQUIRE_PTR(pool_counts); REQUIRE_PTR(fbar_out);
    REQUIRE_PTR(loss); REQUIRE_PTR(aux_coef);
    (void)ws; (void)ws_bytes;
    return check_hip(launch_pool_aux_loss(*shape, counts, psum, fbar_in, pool_counts, fbar_out, loss,
                                          aux_coef, (hipStream_t)stream),
                     "unipool_pool_aux_loss");
}

int unipool_estimate_c(int E, int k, const float* samples, int n_samples, float* c_out,
                       int32_t* samples_used, void* ws, size_t ws_bytes, void* stream) {
    if (E < 1 || E > unipool::kMaxE)
        return unipool::set_error(UNIPOOL_EINVAL, "%s: E=%d outside [1, %d]", __func__, E, unipool::kMaxE);
    if (k < 1 || k > unipool::kMaxK || k > E)
        return unipool::set_error(UNIPOOL_EINVAL, "%s: k=%d outside [1, min(%d, E=%d)]", __func__, k,
                                  unipool::kMaxK, E);
    if (n_samples < 1) return unipool::set_error(UNIPOOL_EINVAL, "%s: n_samples=%d must be positive", __func__, n_samples);
    REQUIRE_PTR(samples); REQUIRE_PTR(c_out); REQUIRE_PTR(samples_used);
    const size_t nb = (size_t)unipool::c_blocks(n_samples);
    const size_t need = 2 * unipool::align_up_256(nb * 4);
    if (!ws) return unipool::set_error(UNIPOOL_EWORKSPACE, "%s: workspace is NULL", __func__);
    if (((uintptr_t)ws & 255) != 0)
        return unipool::set_error(UNIPOOL_EWORKSPACE, "%s: workspace is not 256-byte aligned", __func__);
    if (ws_bytes < need)
        return unipool::set_error(UNIPOOL_EWORKSPACE, "%s: workspace has %zu bytes, %zu needed", __func__, ws_bytes, need);
    float* part_sum = (float*)ws;
    int32_t* part_used = (int32_t*)((char*)ws + unipool::align_up_256(nb * 4));
    return unipool::check_hip(unipool::launch_estimate_c(E, k, samples, n_samples, part_sum, part_used, c_out,
                                                         samples_used, (hipStream_t)stream),
                              "unipool_estimate_c");
}

int unipool_distinct_experts(const unipool_shape* shape, int n_layers, const void* const* topk_idx_l,
                             int32_t* distinct, float* mean_distinct, void* ws, size_t ws_bytes,
                             void* stream) {
    PROLOGUE();
    if (n_layers < 1) return set_error(UNIPOOL_EINVAL, "%s: n_layers=%d must be positive", __func__, n_layers);
    REQUIRE_PTR(topk_idx_l); REQUIRE_PTR(distinct); REQUIRE_PTR(mean_distinct);
    NEED_WS();
    // the block sums (T / 256 words) live in the router's partial-sum area
    const WsLayout w = ws_layout(*shape);
    return check_hip(launch_distinct_experts((const int32_t* const*)topk_idx_l, n_layers, shape->T, shape->k,
                                             distinct, (int32_t*)((char*)ws + w.psum_part), mean_distinct,
                                             (hipStream_t)stream),
                     "unipool_distinct_experts");
}

}  // extern "C"
