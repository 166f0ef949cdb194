"""ctypes binding of libmoe_mi355x.so (declared in include/moe_mi355x.h).

Same names as the C entry points.  Tensors are torch CUDA(ROCm) tensors used as plain device
buffers; the functions pass their data pointers and the current HIP stream.  Nothing is computed
in Python.
"""
from __future__ import annotations

import ctypes as C
import os

ACT_RELU, ACT_GELU_TANH, ACT_SWIGLU, ACT_GELU_ERF = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
SAVED = {n: i for i, n in enumerate(
    ["logits", "probs", "topk_idx", "topk_w", "pos", "row_of", "count", "offsets", "src_of_row", "xe", "a1", "a3",
     "hh", "q"])}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ENTRY_POINTS = ["moe_capacity", "moe_workspace_bytes", "moe_route", "moe_dispatch", "moe_dispatch_bwd",
                "moe_expert_ffn_fwd", "moe_expert_ffn_bwd", "moe_combine", "moe_combine_bwd", "moe_route_bwd",
                "moe_layer_fwd", "moe_layer_bwd", "moe_layer_fwd_chunked", "moe_layer_bwd_chunked", "moe_saved_offset",
                "moe_pipeline_time", "moe_find_pipeline_degree", "moe_route_noisy", "moe_route_noisy_bwd", "moe_route_xmoe_workspace_bytes",
                "moe_route_xmoe", "moe_route_xmoe_bwd", "moe_layer_fwd_routed", "moe_layer_bwd_routed", "moe_route_static", "moe_last_error"]
MAX_CHUNKS = 16  # MOE_MAX_CHUNKS


class MoeError(RuntimeError):
    pass


class MoeConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_tokens", "d_model", "n_experts", "d_hidden", "top_k", "capacity", "dtype",
                                         "act", "renormalize", "add_residual", "accumulate_wgrad")]

    @classmethod
    def make(cls, N, M, E, H, k, capacity, dtype, act, renormalize=0, add_residual=0, accumulate_wgrad=0):
        return cls(N, M, E, H, k, capacity, dtype, act, renormalize, add_residual, accumulate_wgrad)


def lib_path() -> str:
    return os.path.join(_HERE, "libmoe_mi355x.so")


def load():
    """Load the HIP library (built by `python -m paper_2501_10714_amd.build`).  No fallback."""
    global _LIB
    if _LIB is None:
        p = lib_path()
        if not os.path.exists(p):
            raise MoeError(f"{p} is missing: build it first with `python -m paper_2501_10714_amd.build`")
        lib = C.CDLL(p)
        lib.moe_capacity.restype = C.c_int32
        lib.moe_capacity.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_double]
        lib.moe_last_error.restype = C.c_char_p
        for name in ENTRY_POINTS:
            if name not in ("moe_capacity", "moe_last_error", "moe_pipeline_time"):
                getattr(lib, name).restype = C.c_int32
        _LIB = lib
    return _LIB


def moe_last_error() -> str:
    return load().moe_last_error().decode()


def _check(st):
    if st != 0:
        raise MoeError(f"status {st}: {moe_last_error()}")


def _p(t):
    """Device pointer of a tensor (or NULL)."""
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _sz(t):
    return C.c_size_t(0 if t is None else t.numel() * t.element_size())


def moe_capacity(n_tokens, n_experts, top_k, f) -> int:
    return int(load().moe_capacity(n_tokens, n_experts, top_k, float(f)))


def moe_workspace_bytes(cfg):
    ws, sv = C.c_size_t(0), C.c_size_t(0)
    _check(load().moe_workspace_bytes(C.byref(cfg), C.byref(ws), C.byref(sv)))
    return int(ws.value), int(sv.value)


def moe_saved_offset(cfg, which):
    off, n = C.c_size_t(0), C.c_size_t(0)
    _check(load().moe_saved_offset(C.byref(cfg), C.c_int32(SAVED[which] if isinstance(which, str) else which),
                                   C.byref(off), C.byref(n)))
    return int(off.value), int(n.value)


def saved_view(cfg, saved, which, dtype):
    """A typed view of one tensor inside the layer's saved blob (a uint8 device tensor)."""
    off, n = moe_saved_offset(cfg, which)
    return saved[off:off + n].view(dtype)


def moe_route(cfg, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets, src_of_row, ws):
    _check(load().moe_route(C.byref(cfg), _p(x), _p(w_gate), _p(b_gate), _p(logits), _p(probs), _p(topk_idx),
                            _p(topk_w), _p(pos), _p(row_of), _p(count), _p(offsets), _p(src_of_row), _p(ws), _sz(ws),
                            _stream()))


def moe_route_static(cfg, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets, src_of_row):
    """moe_route on the library's built-in scratch array: no workspace argument, nothing allocated."""
    _check(load().moe_route_static(C.byref(cfg), _p(x), _p(w_gate), _p(b_gate), _p(logits), _p(probs), _p(topk_idx),
                                   _p(topk_w), _p(pos), _p(row_of), _p(count), _p(offsets), _p(src_of_row), _stream()))


def moe_dispatch(cfg, x, row_of, xe):
    _check(load().moe_dispatch(C.byref(cfg), _p(x), _p(row_of), _p(xe), _stream()))


def moe_dispatch_bwd(cfg, dxe, row_of, dy, dx):
    _check(load().moe_dispatch_bwd(C.byref(cfg), _p(dxe), _p(row_of), _p(dy), _p(dx), _stream()))


def moe_expert_ffn_fwd(cfg, xe, offsets, w1, w3, w2, q, a1, a3, hh, ws=None):
    _check(load().moe_expert_ffn_fwd(C.byref(cfg), _p(xe), _p(offsets), _p(w1), _p(w3), _p(w2), _p(q), _p(a1), _p(a3),
                                     _p(hh), _p(ws), _sz(ws), _stream()))


def moe_expert_ffn_bwd(cfg, dq, xe, offsets, w1, w3, w2, a1, a3, hh, dxe, dw1, dw3, dw2, ws):
    _check(load().moe_expert_ffn_bwd(C.byref(cfg), _p(dq), _p(xe), _p(offsets), _p(w1), _p(w3), _p(w2), _p(a1), _p(a3),
                                     _p(hh), _p(dxe), _p(dw1), _p(dw3), _p(dw2), _p(ws), _sz(ws), _stream()))


def moe_combine(cfg, q, topk_w, row_of, x, y):
    _check(load().moe_combine(C.byref(cfg), _p(q), _p(topk_w), _p(row_of), _p(x), _p(y), _stream()))


def moe_combine_bwd(cfg, dy, q, topk_w, row_of, dq, dtopk_w):
    _check(load().moe_combine_bwd(C.byref(cfg), _p(dy), _p(q), _p(topk_w), _p(row_of), _p(dq), _p(dtopk_w), _stream()))


def moe_route_bwd(cfg, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws):
    _check(load().moe_route_bwd(C.byref(cfg), _p(x), _p(w_gate), _p(probs), _p(topk_idx), _p(pos), _p(dtopk_w),
                                _p(dw_gate), _p(db_gate), _p(dx), _p(ws), _sz(ws), _stream()))


def moe_layer_fwd(cfg, x, w_gate, b_gate, w1, w3, w2, y, saved, ws):
    _check(load().moe_layer_fwd(C.byref(cfg), _p(x), _p(w_gate), _p(b_gate), _p(w1), _p(w3), _p(w2), _p(y), _p(saved),
                                _sz(saved), _p(ws), _sz(ws), _stream()))


def moe_layer_bwd(cfg, dy, x, w_gate, w1, w3, w2, saved, dx, dw_gate, db_gate, dw1, dw3, dw2, ws):
    _check(load().moe_layer_bwd(C.byref(cfg), _p(dy), _p(x), _p(w_gate), _p(w1), _p(w3), _p(w2), _p(saved), _sz(saved),
                                _p(dx), _p(dw_gate), _p(db_gate), _p(dw1), _p(dw3), _p(dw2), _p(ws), _sz(ws),
                                _stream()))


def moe_layer_fwd_chunked(cfg, x, w_gate, b_gate, w1, w3, w2, y, saved, ws, n_chunks, aux_stream=None):
    """aux_stream: a torch.cuda.Stream (or None) for the dispatch of the next chunk."""
    aux = C.c_void_p(None if aux_stream is None else aux_stream.cuda_stream)
    _check(load().moe_layer_fwd_chunked(C.byref(cfg), _p(x), _p(w_gate), _p(b_gate), _p(w1), _p(w3), _p(w2), _p(y),
                                        _p(saved), _sz(saved), _p(ws), _sz(ws), C.c_int32(n_chunks), _stream(), aux))


def moe_layer_bwd_chunked(cfg, dy, x, w_gate, w1, w3, w2, saved, dx, dw_gate, db_gate, dw1, dw3, dw2, ws, n_chunks):
    _check(load().moe_layer_bwd_chunked(C.byref(cfg), _p(dy), _p(x), _p(w_gate), _p(w1), _p(w3), _p(w2), _p(saved),
                                        _sz(saved), _p(dx), _p(dw_gate), _p(db_gate), _p(dw1), _p(dw3), _p(dw2), _p(ws),
                                        _sz(ws), C.c_int32(n_chunks), _stream()))


class PipelineModel(C.Structure):
    """moe_pipeline_model_t: the linear performance models of FSMoE Sec. 4.1 and the Gradient-AllReduce time."""
    _fields_ = [(n, C.c_double) for n in ("alpha_a2a", "beta_a2a", "n_a2a", "alpha_ag", "beta_ag", "n_ag", "alpha_rs",
                                          "beta_rs", "n_rs", "alpha_exp", "beta_exp", "n_exp", "t_gar")]


def moe_pipeline_time(model, r):
    """(t_moe, case) at pipeline degree r; host function."""
    lib = load()
    lib.moe_pipeline_time.restype = C.c_double
    which = C.c_int32(0)
    t = lib.moe_pipeline_time(C.byref(model), C.c_double(r), C.byref(which))
    return float(t), int(which.value)


def moe_find_pipeline_degree(model, r_max):
    """(r, t_moe, case) of Algorithm 1 over the degrees 1..r_max; host function."""
    r, which, t = C.c_int32(0), C.c_int32(0), C.c_double(0.0)
    _check(load().moe_find_pipeline_degree(C.byref(model), C.c_int32(r_max), C.byref(r), C.byref(t), C.byref(which)))
    return int(r.value), float(t.value), int(which.value)



def moe_route_noisy(cfg, x, w_gate, b_gate, w_noise, noise, logits, noise_logits, probs, topk_idx, topk_w, pos, row_of,
                    count, offsets, src_of_row, ws):
    _check(load().moe_route_noisy(C.byref(cfg), _p(x), _p(w_gate), _p(b_gate), _p(w_noise), _p(noise), _p(logits),
                                  _p(noise_logits), _p(probs), _p(topk_idx), _p(topk_w), _p(pos), _p(row_of), _p(count),
                                  _p(offsets), _p(src_of_row), _p(ws), _sz(ws), _stream()))


def moe_route_noisy_bwd(cfg, x, w_gate, w_noise, noise, noise_logits, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate,
                        dw_noise, dx, ws):
    _check(load().moe_route_noisy_bwd(C.byref(cfg), _p(x), _p(w_gate), _p(w_noise), _p(noise), _p(noise_logits),
                                      _p(probs), _p(topk_idx), _p(pos), _p(dtopk_w), _p(dw_gate), _p(db_gate),
                                      _p(dw_noise), _p(dx), _p(ws), _sz(ws), _stream()))


def moe_route_xmoe_workspace_bytes(cfg, d_proj) -> int:
    ws = C.c_size_t(0)
    _check(load().moe_route_xmoe_workspace_bytes(C.byref(cfg), C.c_int32(d_proj), C.byref(ws)))
    return int(ws.value)


def moe_route_xmoe(cfg, x, w_proj, w_gate, d_proj, proj, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets,
                   src_of_row, ws):
    _check(load().moe_route_xmoe(C.byref(cfg), _p(x), _p(w_proj), _p(w_gate), C.c_int32(d_proj), _p(proj), _p(logits),
                                 _p(probs), _p(topk_idx), _p(topk_w), _p(pos), _p(row_of), _p(count), _p(offsets),
                                 _p(src_of_row), _p(ws), _sz(ws), _stream()))


def moe_route_xmoe_bwd(cfg, x, w_proj, w_gate, d_proj, proj, probs, topk_idx, pos, dtopk_w, dw_proj, dw_gate, dx, ws):
    _check(load().moe_route_xmoe_bwd(C.byref(cfg), _p(x), _p(w_proj), _p(w_gate), C.c_int32(d_proj), _p(proj), _p(probs),
                                     _p(topk_idx), _p(pos), _p(dtopk_w), _p(dw_proj), _p(dw_gate), _p(dx), _p(ws),
                                     _sz(ws), _stream()))


def moe_layer_fwd_routed(cfg, x, w1, w3, w2, y, saved, ws, n_chunks=1, aux_stream=None):
    """The layer after the gate; the routing tensors of `saved` were filled by a moe_route* call (see saved_view)."""
    aux = C.c_void_p(None if aux_stream is None else aux_stream.cuda_stream)
    _check(load().moe_layer_fwd_routed(C.byref(cfg), _p(x), _p(w1), _p(w3), _p(w2), _p(y), _p(saved), _sz(saved), _p(ws),
                                       _sz(ws), C.c_int32(n_chunks), _stream(), aux))


def moe_layer_bwd_routed(cfg, dy, w1, w3, w2, saved, dx, dw1, dw3, dw2, dtopk_w, ws, n_chunks=1):
    _check(load().moe_layer_bwd_routed(C.byref(cfg), _p(dy), _p(w1), _p(w3), _p(w2), _p(saved), _sz(saved), _p(dx),
                                       _p(dw1), _p(dw3), _p(dw2), _p(dtopk_w), _p(ws), _sz(ws), C.c_int32(n_chunks),
                                       _stream()))
