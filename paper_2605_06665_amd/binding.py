"""ctypes binding of libunipool.so.  Argument marshalling only: every function forwards torch
tensors (device memory) as raw pointers to the C entry point of the same name and raises on a
non-zero status.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

F32 = 0
BF16 = 1
ROUTER_NORM = 0
ROUTER_SOFTMAX = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class UniPoolError(RuntimeError):
    pass


class Shape(ctypes.Structure):
    """Mirror of `unipool_shape` (include/unipool.h)."""
    _fields_ = [("T", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("L", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("sigma", ctypes.c_float), ("c", ctypes.c_float),
                ("eps", ctypes.c_float), ("alpha_pool", ctypes.c_float), ("router", ctypes.c_int32)]


ENTRY_POINTS = ("unipool_workspace_bytes", "unipool_last_error", "unipool_version", "unipool_fast_path", "unipool_route",
                "unipool_route_bwd", "unipool_permute", "unipool_permute_static", "unipool_expert_ffn_fwd", "unipool_expert_ffn_fwd_gather",
                "unipool_expert_ffn_recompute", "unipool_expert_ffn_bwd", "unipool_expert_wgrad", "unipool_combine",
                "unipool_combine_bwd", "unipool_pool_aux_loss", "unipool_estimate_c",
                "unipool_distinct_experts")


def lib_path() -> str:
    """Path of the shared library; UNIPOOL_LIB overrides the in-tree build."""
    return os.environ.get("UNIPOOL_LIB") or os.path.join(_PKG, "libunipool.so")


def load_library():
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise UniPoolError(
                "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')" % path)
        lib = ctypes.CDLL(path)
        P, I, Z = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        SP = ctypes.POINTER(Shape)
        lib.unipool_workspace_bytes.restype = Z
        lib.unipool_workspace_bytes.argtypes = [SP]
        lib.unipool_last_error.restype = ctypes.c_char_p
        lib.unipool_last_error.argtypes = []
        lib.unipool_version.restype = I
        lib.unipool_version.argtypes = []
        lib.unipool_fast_path.restype = I
        lib.unipool_fast_path.argtypes = [SP]
        sigs = {
            "unipool_route": [SP] + [P] * 7 + [P, Z, P],
            "unipool_route_bwd": [SP] + [P] * 9 + [I, P, Z, P],
            "unipool_permute": [SP] + [P] * 7 + [P, Z, P],
            "unipool_permute_static": [SP] + [P] * 7 + [P],
            "unipool_expert_ffn_fwd": [SP] + [P] * 8 + [P, Z, P],
            "unipool_expert_ffn_fwd_gather": [SP] + [P] * 9 + [P, Z, P],
            "unipool_expert_ffn_recompute": [SP] + [P] * 6 + [P, Z, P],
            "unipool_expert_ffn_bwd": [SP] + [P] * 12 + [P, Z, P],
            "unipool_expert_wgrad": [SP, I] + [P] * 7 + [I, P, Z, P],
            "unipool_combine": [SP] + [P] * 4 + [P, Z, P],
            "unipool_combine_bwd": [SP] + [P] * 6 + [P, Z, P],
            "unipool_pool_aux_loss": [SP] + [P] * 7 + [P, Z, P],
            "unipool_estimate_c": [I, I, P, I, P, P, P, Z, P],
            "unipool_distinct_experts": [SP, I, P, P, P, P, Z, P],
        }
        for name, argtypes in sigs.items():
            fn = getattr(lib, name)
            fn.restype = I
            fn.argtypes = argtypes
        _LIB = lib
    return _LIB


def last_error() -> str:
    return load_library().unipool_last_error().decode()


def version() -> int:
    return load_library().unipool_version()


def fast_path(shape: Shape) -> int:
    """Bit mask of the kernel families the shape gets (bit 0 expert GEMMs on MFMA, bit 1 router contractions on
    MFMA, bit 2 fused router kernel)."""
    rc = load_library().unipool_fast_path(ctypes.byref(shape))
    _check(rc if rc < 0 else 0, "unipool_fast_path")
    return rc


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise UniPoolError("tensor arguments must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(rc: int, name: str):
    if rc != 0:
        raise UniPoolError("%s failed (%d): %s" % (name, rc, last_error()))


def workspace_bytes(shape: Shape) -> int:
    n = load_library().unipool_workspace_bytes(ctypes.byref(shape))
    if n == 0:
        raise UniPoolError("unipool_workspace_bytes: %s" % last_error())
    return n


def route(shape, x, w_router, topk_idx, topk_gate, logits, counts, psum, ws, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_route(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(topk_idx),
                                        _ptr(topk_gate), _ptr(logits), _ptr(counts), _ptr(psum), p, n,
                                        _stream(stream)), "unipool_route")


def route_bwd(shape, x, w_router, logits, topk_idx, dgate, aux_coef, d_w_router, d_sigma, dx,
              dx_accumulate, ws, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_route_bwd(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(logits),
                                            _ptr(topk_idx), _ptr(dgate), _ptr(aux_coef),
                                            _ptr(d_w_router), _ptr(d_sigma), _ptr(dx),
                                            int(bool(dx_accumulate)), p, n, _stream(stream)),
           "unipool_route_bwd")


def permute(shape, x, topk_idx, counts, x_perm, expert_offsets, row_of_slot, slot_of_row, ws,
            stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_permute(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(counts),
                                          _ptr(x_perm), _ptr(expert_offsets), _ptr(row_of_slot),
                                          _ptr(slot_of_row), p, n, _stream(stream)), "unipool_permute")


def permute_static(shape, x, topk_idx, counts, x_perm, expert_offsets, row_of_slot, slot_of_row, stream=None):
    _check(load_library().unipool_permute_static(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(counts),
                                                 _ptr(x_perm), _ptr(expert_offsets), _ptr(row_of_slot),
                                                 _ptr(slot_of_row), _stream(stream)), "unipool_permute_static")


def expert_ffn_fwd(shape, x_perm, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h, y_perm, ws,
                   stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_expert_ffn_fwd(ctypes.byref(shape), _ptr(x_perm), _ptr(expert_offsets),
                                                 _ptr(w_gate_up), _ptr(w_down), _ptr(act_a),
                                                 _ptr(act_b), _ptr(act_h), _ptr(y_perm), p, n,
                                                 _stream(stream)), "unipool_expert_ffn_fwd")


def expert_ffn_fwd_gather(shape, x, slot_of_row, expert_offsets, w_gate_up, w_down, act_a, act_b, act_h, y_perm, ws,
                          stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_expert_ffn_fwd_gather(ctypes.byref(shape), _ptr(x), _ptr(slot_of_row),
                                                        _ptr(expert_offsets), _ptr(w_gate_up), _ptr(w_down),
                                                        _ptr(act_a), _ptr(act_b), _ptr(act_h), _ptr(y_perm), p, n,
                                                        _stream(stream)), "unipool_expert_ffn_fwd_gather")


def expert_ffn_recompute(shape, x_perm, expert_offsets, w_gate_up, act_a, act_b, act_h, ws, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_expert_ffn_recompute(ctypes.byref(shape), _ptr(x_perm),
                                                       _ptr(expert_offsets), _ptr(w_gate_up), _ptr(act_a),
                                                       _ptr(act_b), _ptr(act_h), p, n, _stream(stream)),
           "unipool_expert_ffn_recompute")


def expert_ffn_bwd(shape, dy_perm, x_perm, act_a, act_b, act_h, expert_offsets, w_gate_up, w_down,
                   dx_perm, d_act, d_w_gate_up, d_w_down, ws, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_expert_ffn_bwd(ctypes.byref(shape), _ptr(dy_perm), _ptr(x_perm),
                                                 _ptr(act_a), _ptr(act_b), _ptr(act_h),
                                                 _ptr(expert_offsets), _ptr(w_gate_up), _ptr(w_down),
                                                 _ptr(dx_perm), _ptr(d_act), _ptr(d_w_gate_up),
                                                 _ptr(d_w_down), p, n, _stream(stream)),
           "unipool_expert_ffn_bwd")


def expert_wgrad(shape, n_layers, x_perm_tab, d_act_tab, act_h_tab, dy_perm_tab, offsets_tab,
                 d_w_gate_up, d_w_down, accumulate, ws, stream=None):
    """The *_tab arguments are int64 device tensors holding n_layers device addresses each."""
    p, n = _ws(ws)
    _check(load_library().unipool_expert_wgrad(ctypes.byref(shape), int(n_layers), _ptr(x_perm_tab),
                                               _ptr(d_act_tab), _ptr(act_h_tab), _ptr(dy_perm_tab),
                                               _ptr(offsets_tab), _ptr(d_w_gate_up), _ptr(d_w_down),
                                               int(bool(accumulate)), p, n, _stream(stream)),
           "unipool_expert_wgrad")


def combine(shape, y_perm, row_of_slot, gate, out, ws=None, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_combine(ctypes.byref(shape), _ptr(y_perm), _ptr(row_of_slot),
                                          _ptr(gate), _ptr(out), p, n, _stream(stream)),
           "unipool_combine")


def combine_bwd(shape, dout, y_perm, row_of_slot, gate, dy_perm, dgate, ws=None, stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_combine_bwd(ctypes.byref(shape), _ptr(dout), _ptr(y_perm),
                                              _ptr(row_of_slot), _ptr(gate), _ptr(dy_perm),
                                              _ptr(dgate), p, n, _stream(stream)), "unipool_combine_bwd")


def pool_aux_loss(shape, counts, psum, fbar_in, pool_counts, fbar_out, loss, aux_coef, ws=None,
                  stream=None):
    p, n = _ws(ws)
    _check(load_library().unipool_pool_aux_loss(ctypes.byref(shape), _ptr(counts), _ptr(psum),
                                                _ptr(fbar_in), _ptr(pool_counts), _ptr(fbar_out),
                                                _ptr(loss), _ptr(aux_coef), p, n, _stream(stream)),
           "unipool_pool_aux_loss")


def estimate_c(E, k, samples, c_out, samples_used, ws, stream=None):
    """samples: [n, E] float32 device tensor of N(0, 1) draws; c_out [1] float32; samples_used [1] int32."""
    p, n = _ws(ws)
    _check(load_library().unipool_estimate_c(int(E), int(k), _ptr(samples), int(samples.shape[0]), _ptr(c_out),
                                             _ptr(samples_used), p, n, _stream(stream)), "unipool_estimate_c")


def distinct_experts(shape, n_layers, topk_idx_tab, distinct, mean_distinct, ws, stream=None):
    """topk_idx_tab: int64 device tensor holding n_layers device addresses of [T, k] int32 tensors."""
    p, n = _ws(ws)
    _check(load_library().unipool_distinct_experts(ctypes.byref(shape), int(n_layers), _ptr(topk_idx_tab),
                                                   _ptr(distinct), _ptr(mean_distinct), p, n, _stream(stream)),
           "unipool_distinct_experts")
