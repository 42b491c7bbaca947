"""Thin ctypes binding of libdfk.so: same names as the C ABI (include/dfk.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch appears here solely as the owner of device memory and
streams.  There is no CPU fallback: if the library is missing the import of
a function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdfk.so")

DFK_OK = 0
DFK_ERR_INVALID_ARG = -1
DFK_ERR_UNSUPPORTED_SHAPE = -2
DFK_ERR_ALIGNMENT = -3
DFK_ERR_ALIAS = -4
DFK_ERR_WORKSPACE = -5
DFK_ERR_HIP = -6
DFK_ERR_IO = -7
DFK_ERR_NOT_FOUND = -8

DFK_BF16, DFK_FP32, DFK_FP16 = 0, 1, 2
DFK_VARIANT_AUTO, DFK_VARIANT_FUSED, DFK_VARIANT_TWO_KERNEL = 0, 1, 2
DFK_PATH_VALU, DFK_PATH_MFMA = 0, 1
DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC = 0, 1
DFK_MAX_M = 256


class dfk_config_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in (
        "variant", "path", "splits", "waves", "depth", "reduce",
        "k2_splits", "k2_col_blocks", "a2_dtype", "k2_rows_by_wave", "kmajor")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}

    def __repr__(self):
        return "dfk_config_t(" + ", ".join(f"{k}={v}" for k, v in self.as_dict().items()) + ")"


class DfkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().dfk_status_string(status).decode()
        if status == DFK_ERR_HIP:
            msg += f" (hipError {lib().dfk_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


_lib = None

# every symbol include/dfk.h declares: (name, restype, argtypes)
_vp, _ci, _sz, _cfgp = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(dfk_config_t)
SIGNATURES = [
    ("dfk_swiglu_mlp", _ci, [_vp] * 5 + [_ci] * 3 + [_vp]),
    ("dfk_swiglu_mlp_fused", _ci, [_vp] * 5 + [_ci] * 3 + [_vp]),
    ("dfk_swiglu_mlp_unfused", _ci, [_vp] * 5 + [_ci] * 3 + [_vp]),
    ("dfk_swiglu_mlp_ex", _ci, [_vp] * 5 + [_ci] * 4 + [_cfgp, _vp, _sz, _vp]),
    ("dfk_swiglu_mlp_wdt", _ci, [_vp] * 5 + [_ci] * 4 + [_cfgp, _vp, _sz, _vp]),
    ("dfk_transpose_w_down", _ci, [_vp, _vp, _ci, _ci, _ci, _vp]),
    ("dfk_num_candidates_wdt", _ci, [_ci] * 4),
    ("dfk_get_candidate_wdt", _ci, [_ci] * 5 + [_cfgp]),
    ("dfk_get_choice_wdt", _ci, [_ci] * 4 + [_cfgp, ctypes.POINTER(_ci)]),
    ("dfk_swiglu_mlp_static", _ci, [_vp] * 5 + [_ci] * 4 + [_cfgp, _vp]),
    ("dfk_mlp_block", _ci, [_vp, _vp, ctypes.c_float] + [_vp] * 4 + [_ci] * 4 + [_cfgp, _vp, _sz, _vp]),
    ("dfk_mlp_block_wdt", _ci, [_vp, _vp, ctypes.c_float] + [_vp] * 4 + [_ci] * 4 + [_cfgp, _vp, _sz, _vp]),
    ("dfk_check_args", _ci, [_vp] * 5 + [_ci] * 4 + [_cfgp, _vp, _sz]),
    ("dfk_workspace_bytes", _sz, [_ci] * 3),
    ("dfk_workspace_init", _ci, [_vp, _sz, _vp]),
    ("dfk_set_workspace", _ci, [_vp, _sz]),
    ("dfk_num_candidates", _ci, [_ci] * 4),
    ("dfk_get_candidate", _ci, [_ci] * 5 + [_cfgp]),
    ("dfk_config_valid", _ci, [_cfgp] + [_ci] * 4),
    ("dfk_tune_scratch_bytes", _sz, [_ci] * 5),
    ("dfk_tune", _ci, [ctypes.POINTER(_ci), _ci, _ci, _ci, _ci, _vp, _sz, _ci, _ci, _vp]),
    ("dfk_tune_skipped", _ci, [ctypes.POINTER(_ci)]),
    ("dfk_time_config", _ci, [_cfgp] + [_ci] * 4 + [_vp, _sz, _ci, _ci, _vp, ctypes.POINTER(ctypes.c_double)]),
    ("dfk_time_kernels", _ci, [_cfgp] + [_ci] * 4 + [_vp, _sz, _ci, _ci, _vp, ctypes.POINTER(ctypes.c_double)]),
    ("dfk_get_choice", _ci, [_ci] * 4 + [_cfgp, ctypes.POINTER(_ci)]),
    ("dfk_set_choice", _ci, [_ci] * 4 + [_cfgp, ctypes.c_double]),
    ("dfk_clear_tuning", None, []),
    ("dfk_save_tuning", _ci, [ctypes.c_char_p]),
    ("dfk_load_tuning", _ci, [ctypes.c_char_p]),
    ("dfk_stream_read", _ci, [_vp, _sz, _vp, _vp]),
    ("dfk_read_gateup_pattern", _ci, [_vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp]),
    ("dfk_fill_synthetic", _ci, [_vp, _sz, _ci, ctypes.c_float, ctypes.c_uint, _vp]),
    ("dfk_rms_normalize", _ci, [_vp, _vp, _ci, _ci, _vp]),
    ("dfk_set_trace_buffer", _ci, [_vp, _sz]),
    ("dfk_status_string", ctypes.c_char_p, [_ci]),
    ("dfk_last_hip_error", _ci, []),
    ("dfk_version", ctypes.c_char_p, []),
]


def lib():
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2602_11808_amd.build` "
                "(there is no fallback path)")
        l = ctypes.CDLL(LIB_PATH)
        for name, res, args in SIGNATURES:
            fn = getattr(l, name)          # AttributeError if a declared symbol is not exported
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def _check(status: int, where: str):
    if status != DFK_OK:
        raise DfkError(status, where)


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream(stream) -> int:
    """torch stream (or None = torch's current stream) -> hipStream_t value."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return DFK_BF16
    if t.dtype == torch.float32:
        return DFK_FP32
    if t.dtype == torch.float16:
        return DFK_FP16
    raise TypeError(f"dfk takes bfloat16, float16 or float32 tensors, got {t.dtype}")


def _shapes(X, W_gate, W_up, W_down, Y, wd_t=False):
    for t in (X, W_gate, W_up, W_down, Y):
        if not t.is_cuda:
            raise ValueError("dfk tensors must live in device memory")
        if not t.is_contiguous():
            raise ValueError("dfk tensors must be dense row-major")
        if t.dtype != X.dtype:
            raise TypeError("all dfk tensors must share one element type")
    M, d_model = X.shape
    d_ff = W_gate.shape[0]
    if tuple(W_gate.shape) != (d_ff, d_model) or tuple(W_up.shape) != (d_ff, d_model) \
            or tuple(W_down.shape) != ((d_model, d_ff) if wd_t else (d_ff, d_model)) or tuple(Y.shape) != (M, d_model):
        raise ValueError("expected X,Y [M,d_model], W_gate,W_up [d_ff,d_model] and W_down [d_ff,d_model] "
                         "(W_down_t [d_model,d_ff] for the _wdt entry point)")
    return M, d_model, d_ff


# ------------------------------------------------------------------ the block

def dfk_swiglu_mlp(X, W_gate, W_up, W_down, Y, stream=None):
    M, d, ff = _shapes(X, W_gate, W_up, W_down, Y)
    _check(lib().dfk_swiglu_mlp(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(Y), M, d, ff,
                                _stream(stream)), "dfk_swiglu_mlp")


def dfk_swiglu_mlp_fused(X, W_gate, W_up, W_down, Y, stream=None):
    M, d, ff = _shapes(X, W_gate, W_up, W_down, Y)
    _check(lib().dfk_swiglu_mlp_fused(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(Y), M, d, ff,
                                      _stream(stream)), "dfk_swiglu_mlp_fused")


def dfk_swiglu_mlp_unfused(X, W_gate, W_up, W_down, Y, stream=None):
    M, d, ff = _shapes(X, W_gate, W_up, W_down, Y)
    _check(lib().dfk_swiglu_mlp_unfused(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(Y), M, d, ff,
                                        _stream(stream)), "dfk_swiglu_mlp_unfused")


def dfk_swiglu_mlp_ex(X, W_gate, W_up, W_down, Y, cfg: Optional[dfk_config_t], workspace, stream=None):
    M, d, ff = _shapes(X, W_gate, W_up, W_down, Y)
    nbytes = workspace.numel() * workspace.element_size()
    _check(lib().dfk_swiglu_mlp_ex(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(Y), M, d, ff,
                                   _dtype_code(X), ctypes.byref(cfg) if cfg is not None else None,
                                   _ptr(workspace), nbytes, _stream(stream)), "dfk_swiglu_mlp_ex")


def dfk_swiglu_mlp_wdt(X, W_gate, W_up, W_down_t, Y, cfg: Optional[dfk_config_t], workspace, stream=None):
    """The block with the down projection's weights as W_down_t [d_model, d_ff] (a linear layer's own layout)."""
    M, d, ff = _shapes(X, W_gate, W_up, W_down_t, Y, wd_t=True)
    nbytes = workspace.numel() * workspace.element_size()
    _check(lib().dfk_swiglu_mlp_wdt(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down_t), _ptr(Y), M, d, ff,
                                    _dtype_code(X), ctypes.byref(cfg) if cfg is not None else None,
                                    _ptr(workspace), nbytes, _stream(stream)), "dfk_swiglu_mlp_wdt")


def dfk_transpose_w_down(W_down, W_down_t, stream=None):
    """W_down_t [d_model, d_ff] = transpose of W_down [d_ff, d_model], on the device."""
    ff, d = W_down.shape
    if tuple(W_down_t.shape) != (d, ff) or W_down_t.dtype != W_down.dtype or not W_down.is_cuda or not W_down_t.is_cuda \
            or not W_down.is_contiguous() or not W_down_t.is_contiguous():
        raise ValueError("expected dense device tensors W_down [d_ff,d_model] and W_down_t [d_model,d_ff] of one type")
    _check(lib().dfk_transpose_w_down(_ptr(W_down), _ptr(W_down_t), d, ff, _dtype_code(W_down), _stream(stream)),
           "dfk_transpose_w_down")


def dfk_swiglu_mlp_static(X, W_gate, W_up, W_down, Y, cfg: Optional[dfk_config_t] = None, stream=None):
    """The block on the library's own scratch array: no workspace argument, nothing allocated."""
    M, d, ff = _shapes(X, W_gate, W_up, W_down, Y)
    _check(lib().dfk_swiglu_mlp_static(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(Y), M, d, ff,
                                       _dtype_code(X), ctypes.byref(cfg) if cfg is not None else None,
                                       _stream(stream)), "dfk_swiglu_mlp_static")


def dfk_mlp_block(H, norm_weight, eps: float, W_gate, W_up, W_down, H_out, cfg: Optional[dfk_config_t], workspace,
                  stream=None):
    """H_out = H + SwiGLU_MLP(RMSNorm(H; norm_weight, eps)); H_out may be H itself."""
    M, d, ff = _shapes(H, W_gate, W_up, W_down, H_out)
    if not norm_weight.is_cuda or not norm_weight.is_contiguous() or norm_weight.dtype != H.dtype \
            or tuple(norm_weight.shape) != (d,):
        raise ValueError("norm_weight must be a dense device vector [d_model] of the inputs' type")
    nbytes = workspace.numel() * workspace.element_size()
    _check(lib().dfk_mlp_block(_ptr(H), _ptr(norm_weight), float(eps), _ptr(W_gate), _ptr(W_up), _ptr(W_down),
                               _ptr(H_out), M, d, ff, _dtype_code(H),
                               ctypes.byref(cfg) if cfg is not None else None,
                               _ptr(workspace), nbytes, _stream(stream)), "dfk_mlp_block")


def dfk_mlp_block_wdt(H, norm_weight, eps: float, W_gate, W_up, W_down_t, H_out, cfg: Optional[dfk_config_t], workspace,
                      stream=None):
    """dfk_mlp_block with the down projection's weights as W_down_t [d_model, d_ff]."""
    M, d, ff = _shapes(H, W_gate, W_up, W_down_t, H_out, wd_t=True)
    if not norm_weight.is_cuda or not norm_weight.is_contiguous() or norm_weight.dtype != H.dtype \
            or tuple(norm_weight.shape) != (d,):
        raise ValueError("norm_weight must be a dense device vector [d_model] of the inputs' type")
    nbytes = workspace.numel() * workspace.element_size()
    _check(lib().dfk_mlp_block_wdt(_ptr(H), _ptr(norm_weight), float(eps), _ptr(W_gate), _ptr(W_up), _ptr(W_down_t),
                                   _ptr(H_out), M, d, ff, _dtype_code(H),
                                   ctypes.byref(cfg) if cfg is not None else None,
                                   _ptr(workspace), nbytes, _stream(stream)), "dfk_mlp_block_wdt")


def dfk_check_args(X, W_gate, W_up, W_down, Y, M, d_model, d_ff, dtype=DFK_BF16, cfg=None,
                   workspace=0, workspace_bytes=0) -> int:
    """Raw host-only validation on integer addresses; returns the status code."""
    return lib().dfk_check_args(X, W_gate, W_up, W_down, Y, M, d_model, d_ff, dtype,
                                ctypes.byref(cfg) if cfg is not None else None,
                                workspace, workspace_bytes)


# ------------------------------------------------------------------ workspace

def dfk_workspace_bytes(M_max: int, d_model: int, d_ff: int) -> int:
    return int(lib().dfk_workspace_bytes(M_max, d_model, d_ff))


def dfk_workspace_init(workspace, stream=None):
    _check(lib().dfk_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)), "dfk_workspace_init")


def dfk_set_workspace(workspace):
    if workspace is None:
        _check(lib().dfk_set_workspace(None, 0), "dfk_set_workspace")
    else:
        _check(lib().dfk_set_workspace(_ptr(workspace), workspace.numel() * workspace.element_size()),
               "dfk_set_workspace")


def new_workspace(M_max: int, d_model: int, d_ff: int, device="cuda", stream=None):
    """Allocate (with torch) and initialise a workspace tensor for calls up to M_max."""
    import torch
    n = dfk_workspace_bytes(M_max, d_model, d_ff)
    if n == 0:
        raise ValueError("invalid shape for a workspace")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    dfk_workspace_init(ws, stream)
    return ws


# ------------------------------------------------------------------ scheduler

def dfk_num_candidates(M, d_model, d_ff, dtype=DFK_BF16) -> int:
    return int(lib().dfk_num_candidates(M, d_model, d_ff, dtype))


def dfk_get_candidate(M, d_model, d_ff, dtype, i) -> dfk_config_t:
    c = dfk_config_t()
    _check(lib().dfk_get_candidate(M, d_model, d_ff, dtype, i, ctypes.byref(c)), "dfk_get_candidate")
    return c


def dfk_num_candidates_wdt(M, d_model, d_ff, dtype=DFK_BF16) -> int:
    return int(lib().dfk_num_candidates_wdt(M, d_model, d_ff, dtype))


def dfk_get_candidate_wdt(M, d_model, d_ff, dtype, i) -> dfk_config_t:
    c = dfk_config_t()
    _check(lib().dfk_get_candidate_wdt(M, d_model, d_ff, dtype, i, ctypes.byref(c)), "dfk_get_candidate_wdt")
    return c


def dfk_get_choice_wdt(M, d_model, d_ff, dtype=DFK_BF16):
    c = dfk_config_t()
    tuned = ctypes.c_int(0)
    _check(lib().dfk_get_choice_wdt(M, d_model, d_ff, dtype, ctypes.byref(c), ctypes.byref(tuned)),
           "dfk_get_choice_wdt")
    return c, bool(tuned.value)


def dfk_config_valid(cfg, M, d_model, d_ff, dtype=DFK_BF16) -> bool:
    return bool(lib().dfk_config_valid(ctypes.byref(cfg), M, d_model, d_ff, dtype))


def dfk_tune_scratch_bytes(M_max, d_model, d_ff, dtype=DFK_BF16, sets=4) -> int:
    return int(lib().dfk_tune_scratch_bytes(M_max, d_model, d_ff, dtype, sets))


def dfk_tune(M_list: Sequence[int], d_model, d_ff, dtype, scratch, sets=4, iters=20, stream=None):
    arr = (ctypes.c_int * len(M_list))(*M_list)
    _check(lib().dfk_tune(arr, len(M_list), d_model, d_ff, dtype, _ptr(scratch),
                          scratch.numel() * scratch.element_size(), sets, iters, _stream(stream)),
           "dfk_tune")


def dfk_tune_skipped():
    """(count, status of the last one) of the candidates the last dfk_tune on this thread left out."""
    st = ctypes.c_int(0)
    n = int(lib().dfk_tune_skipped(ctypes.byref(st)))
    return n, int(st.value)


def dfk_time_config(cfg, M, d_model, d_ff, dtype, scratch, sets=4, iters=20, stream=None) -> float:
    us = ctypes.c_double(0.0)
    _check(lib().dfk_time_config(ctypes.byref(cfg), M, d_model, d_ff, dtype, _ptr(scratch),
                                 scratch.numel() * scratch.element_size(), sets, iters,
                                 _stream(stream), ctypes.byref(us)), "dfk_time_config")
    return us.value


def dfk_time_kernels(cfg, M, d_model, d_ff, dtype, scratch, sets=4, iters=20, stream=None):
    """Mean microseconds of the first and of the second launch of a call, (us1, us2)."""
    us = (ctypes.c_double * 2)(0.0, 0.0)
    _check(lib().dfk_time_kernels(ctypes.byref(cfg), M, d_model, d_ff, dtype, _ptr(scratch),
                                  scratch.numel() * scratch.element_size(), sets, iters,
                                  _stream(stream), us), "dfk_time_kernels")
    return us[0], us[1]


def dfk_get_choice(M, d_model, d_ff, dtype=DFK_BF16):
    c = dfk_config_t()
    tuned = ctypes.c_int(0)
    _check(lib().dfk_get_choice(M, d_model, d_ff, dtype, ctypes.byref(c), ctypes.byref(tuned)),
           "dfk_get_choice")
    return c, bool(tuned.value)


def dfk_set_choice(M, d_model, d_ff, dtype, cfg, usec=0.0):
    _check(lib().dfk_set_choice(M, d_model, d_ff, dtype, ctypes.byref(cfg), usec), "dfk_set_choice")


def dfk_clear_tuning():
    lib().dfk_clear_tuning()


def dfk_save_tuning(path: str):
    _check(lib().dfk_save_tuning(os.fsencode(path)), "dfk_save_tuning")


def dfk_load_tuning(path: str):
    _check(lib().dfk_load_tuning(os.fsencode(path)), "dfk_load_tuning")


# ------------------------------------------------------------------ measurement

def dfk_stream_read(src, sink, stream=None):
    _check(lib().dfk_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                 _stream(stream)), "dfk_stream_read")


def dfk_read_gateup_pattern(W_gate, W_up, splits: int, waves: int, sink, stream=None):
    """Reads W_gate and W_up [d_ff, d_model] in the gate/up kernel's access pattern, and nothing else."""
    if W_gate.shape != W_up.shape or W_gate.dim() != 2 or W_gate.element_size() != 2 \
            or not W_gate.is_contiguous() or not W_up.is_contiguous():
        raise ValueError("W_gate and W_up must be dense [d_ff, d_model] tensors of a 16-bit type")
    d_ff, d_model = W_gate.shape
    _check(lib().dfk_read_gateup_pattern(_ptr(W_gate), _ptr(W_up), d_model, d_ff, splits, waves, _ptr(sink),
                                         _stream(stream)), "dfk_read_gateup_pattern")


def dfk_fill_synthetic(dst, scale: float, seed: int, stream=None):
    _check(lib().dfk_fill_synthetic(_ptr(dst), dst.numel(), _dtype_code(dst), scale, seed,
                                    _stream(stream)), "dfk_fill_synthetic")


def dfk_rms_normalize(src, dst, stream=None):
    M, d = src.shape
    _check(lib().dfk_rms_normalize(_ptr(src), _ptr(dst), M, d, _stream(stream)), "dfk_rms_normalize")


def dfk_set_trace_buffer(buf):
    if buf is None:
        _check(lib().dfk_set_trace_buffer(None, 0), "dfk_set_trace_buffer")
    else:
        _check(lib().dfk_set_trace_buffer(_ptr(buf), buf.numel() * buf.element_size()), "dfk_set_trace_buffer")


def dfk_status_string(status: int) -> str:
    return lib().dfk_status_string(status).decode()


def dfk_last_hip_error() -> int:
    return int(lib().dfk_last_hip_error())


def dfk_version() -> str:
    return lib().dfk_version().decode()
