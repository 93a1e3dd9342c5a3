"""Python binding of the C-ABI SSD library (``include/ssd.h``): argument marshalling only.

Every step of prefill and decode runs in the HIP kernels of ``libssd_hip.so``; this module
turns torch tensors into device pointers, fills the ``ssd_shape`` struct, passes the current
HIP stream and raises on a non-zero status.  There is no fallback: if the library has not
been built (``python -m paper_2603_09555_amd.build``) importing this module fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssd_hip.so")

SSD_F32, SSD_BF16 = 0, 1
SSD_OK = 0

EXPORTS = ["ssd_prefill_workspace_bytes", "ssd_prefill", "ssd_prefill_static", "ssd_decode_step", "ssd_decode_step_layers",
           "ssd_decode_steps_layers", "ssd_prefill_varlen_workspace_bytes", "ssd_prefill_varlen",
           "ssd_conv1d_prefill", "ssd_conv1d_step", "ssd_prefill_dt", "ssd_prefill_varlen_dt",
           "ssd_decode_step_layers_dt", "ssd_decode_steps_layers_dt",
           "ssd_prefill_path", "ssd_status_string", "ssd_version",
           "ssd_testing_set_knob", "ssd_testing_reset_knobs", "ssd_testing_prefill_plan"]


class ssd_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "seqlen", "nheads", "headdim", "dstate", "ngroups", "chunk", "io_dtype")]


class SSDError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


if not os.path.exists(LIB_PATH):
    raise ImportError("libssd_hip.so is missing: build it with `python -m paper_2603_09555_amd.build` "
                      "(there is no CPU or PyTorch fallback)")

_lib = ctypes.CDLL(LIB_PATH)
_vp, _sz = ctypes.c_void_p, ctypes.c_size_t
_sp = ctypes.POINTER(ssd_shape)
_lib.ssd_prefill_workspace_bytes.restype = _sz
_lib.ssd_prefill_workspace_bytes.argtypes = [_sp]
_lib.ssd_prefill.restype = ctypes.c_int
_lib.ssd_prefill.argtypes = [_sp] + [_vp] * 10 + [_sz, _vp]
_lib.ssd_prefill_static.restype = ctypes.c_int
_lib.ssd_prefill_static.argtypes = [_sp] + [_vp] * 10
STATIC_SCRATCH_BYTES = 32 << 20   # SSD_STATIC_SCRATCH_BYTES of include/ssd.h
class ssd_dt_transform(ctypes.Structure):
    _fields_ = [("dt_bias", ctypes.c_void_p), ("dt_softplus", ctypes.c_int32), ("dt_min", ctypes.c_float),
                ("dt_max", ctypes.c_float)]


_lib.ssd_prefill_dt.restype = ctypes.c_int
_lib.ssd_prefill_dt.argtypes = [_sp, ctypes.POINTER(ssd_dt_transform)] + [_vp] * 10 + [_sz, _vp]
_lib.ssd_testing_set_knob.restype = ctypes.c_int
_lib.ssd_testing_set_knob.argtypes = [ctypes.c_int32, ctypes.c_int32]
_lib.ssd_testing_reset_knobs.restype = None
_lib.ssd_testing_reset_knobs.argtypes = []
_lib.ssd_testing_prefill_plan.restype = ctypes.c_int
_lib.ssd_testing_prefill_plan.argtypes = [ctypes.POINTER(ssd_shape), ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
_lib.ssd_decode_step.restype = ctypes.c_int
_lib.ssd_decode_step.argtypes = [_sp] + [_vp] * 9
_lib.ssd_decode_step_layers.restype = ctypes.c_int
_lib.ssd_decode_step_layers.argtypes = [ctypes.c_int32, _sp] + [_vp] * 9
_lib.ssd_prefill_varlen_workspace_bytes.restype = _sz
_lib.ssd_prefill_varlen_workspace_bytes.argtypes = [_sp]
_lib.ssd_prefill_varlen.restype = ctypes.c_int
_lib.ssd_prefill_varlen.argtypes = [_sp] + [_vp] * 11 + [_sz, _vp]
_i32 = ctypes.c_int32
_lib.ssd_conv1d_prefill.restype = ctypes.c_int
_lib.ssd_conv1d_prefill.argtypes = [_i32, _i32, _i32, _i32, ctypes.POINTER(_i32)] + [_vp] * 8 + [_i32, _vp]
_lib.ssd_conv1d_step.restype = ctypes.c_int
_lib.ssd_conv1d_step.argtypes = [_i32, _i32, _i32, ctypes.POINTER(_i32)] + [_vp] * 7 + [_i32, _vp]
_lib.ssd_decode_steps_layers.restype = ctypes.c_int
_lib.ssd_decode_steps_layers.argtypes = [ctypes.c_int32, ctypes.c_int32, _sp] + [_vp] * 9
_lib.ssd_prefill_varlen_dt.restype = ctypes.c_int
_lib.ssd_prefill_varlen_dt.argtypes = [_sp, ctypes.POINTER(ssd_dt_transform)] + [_vp] * 11 + [_sz, _vp]
_lib.ssd_decode_step_layers_dt.restype = ctypes.c_int
_lib.ssd_decode_step_layers_dt.argtypes = [ctypes.c_int32, _sp, ctypes.POINTER(ssd_dt_transform)] + [_vp] * 9
_lib.ssd_decode_steps_layers_dt.restype = ctypes.c_int
_lib.ssd_decode_steps_layers_dt.argtypes = [ctypes.c_int32, ctypes.c_int32, _sp, ctypes.POINTER(ssd_dt_transform)] + [_vp] * 9
_lib.ssd_prefill_path.restype = ctypes.c_char_p
_lib.ssd_prefill_path.argtypes = [_sp]
_lib.ssd_status_string.restype = ctypes.c_char_p
_lib.ssd_status_string.argtypes = [ctypes.c_int]
_lib.ssd_version.restype = ctypes.c_int


def raw():
    """The ctypes handle, for callers that want to pass raw pointers (tests of error paths)."""
    return _lib


def status_string(status: int) -> str:
    return _lib.ssd_status_string(int(status)).decode()


def version() -> int:
    return int(_lib.ssd_version())


def make_shape(batch, seqlen, nheads, headdim, dstate, ngroups, chunk, io_dtype) -> ssd_shape:
    if isinstance(io_dtype, torch.dtype):
        io_dtype = {torch.float32: SSD_F32, torch.bfloat16: SSD_BF16}.get(io_dtype, -1)
    return ssd_shape(batch, seqlen, nheads, headdim, dstate, ngroups, chunk, io_dtype)


def prefill_workspace_bytes(shape: ssd_shape) -> int:
    return int(_lib.ssd_prefill_workspace_bytes(ctypes.byref(shape)))


def prefill_path(shape: ssd_shape) -> str:
    return _lib.ssd_prefill_path(ctypes.byref(shape)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check_dev(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _stream_ptr():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt_transform(dt_bias, dt_softplus, dt_limit, bias_shape):
    """The ``ssd_dt_transform`` of a call, or None when dt is to be used as given."""
    if dt_bias is None and not dt_softplus and dt_limit is None:
        return None
    if dt_bias is not None and (dt_bias.dtype != torch.float32 or tuple(dt_bias.shape) != tuple(bias_shape)):
        raise ValueError("dt_bias must be fp32 of shape %s" % (tuple(bias_shape),))
    _check_dev(dt_bias)
    lo, hi = dt_limit if dt_limit is not None else (0.0, 0.0)
    return ssd_dt_transform(None if dt_bias is None else dt_bias.data_ptr(), int(bool(dt_softplus)), lo, hi)


def ssd_prefill(x, dt, A, B, C, D, chunk, h0=None, y=None, final_state=None, workspace=None,
                dt_bias=None, dt_softplus=False, dt_limit=None):
    """``ssd_prefill`` of the C ABI on torch device tensors.  Returns ``(y, final_state)``.

    ``x (Bt,T,H,P)``, ``B, C (Bt,T,G,N)`` in fp32 or bf16; ``dt (Bt,T,H)``, ``A, D (H)``,
    ``h0 (Bt,H,P,N)`` fp32.  Output and workspace tensors are allocated with torch unless given.
    With ``dt_bias (H)``, ``dt_softplus`` or ``dt_limit=(lo, hi)`` the call goes through
    ``ssd_prefill_dt``: ``dt`` is then the raw value and the kernels apply
    ``clamp(softplus(dt + dt_bias), lo, hi)`` as they read it.
    """
    Bt, T, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    shape = make_shape(Bt, T, H, P, N, G, chunk, x.dtype)
    if B.dtype != x.dtype or C.dtype != x.dtype:
        raise ValueError("x, B and C must share one dtype")
    for t in (dt, A, D, h0):
        if t is not None and t.dtype != torch.float32:
            raise ValueError("dt, A, D and h0 must be fp32")
    if tuple(dt.shape) != (Bt, T, H) or tuple(A.shape) != (H,) or tuple(D.shape) != (H,) \
            or tuple(C.shape) != tuple(B.shape) or tuple(B.shape[:2]) != (Bt, T) \
            or (h0 is not None and tuple(h0.shape) != (Bt, H, P, N)):
        raise ValueError("inconsistent tensor shapes")
    if y is None:
        y = torch.empty_like(x)
    if final_state is None:
        final_state = torch.empty((Bt, H, P, N), dtype=torch.float32, device=x.device)
    need = prefill_workspace_bytes(shape)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    _check_dev(x, dt, A, B, C, D, h0, y, final_state, workspace)
    args = (ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(h0), _ptr(y),
            _ptr(final_state), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_ptr())
    xf = _dt_transform(dt_bias, dt_softplus, dt_limit, (H,))
    if xf is not None:
        st = _lib.ssd_prefill_dt(args[0], ctypes.byref(xf), *args[1:])
    else:
        st = _lib.ssd_prefill(*args)
    if st != SSD_OK:
        raise SSDError(st, "ssd_prefill")
    return y, final_state


def ssd_prefill_static(x, dt, A, B, C, D, chunk, y, final_state, h0=None):
    """``ssd_prefill_static`` of the C ABI: the prefill on the library's own scratch buffer.  The C call
    allocates nothing; neither does this wrapper -- ``y`` and ``final_state`` must be given."""
    Bt, T, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    shape = make_shape(Bt, T, H, P, N, G, chunk, x.dtype)
    if B.dtype != x.dtype or C.dtype != x.dtype or y.dtype != x.dtype:
        raise ValueError("x, B, C and y must share one dtype")
    for t in (dt, A, D, h0, final_state):
        if t is not None and t.dtype != torch.float32:
            raise ValueError("dt, A, D, h0 and final_state must be fp32")
    if tuple(dt.shape) != (Bt, T, H) or tuple(A.shape) != (H,) or tuple(D.shape) != (H,) \
            or tuple(C.shape) != tuple(B.shape) or tuple(B.shape[:2]) != (Bt, T) or tuple(y.shape) != tuple(x.shape) \
            or tuple(final_state.shape) != (Bt, H, P, N) or (h0 is not None and tuple(h0.shape) != (Bt, H, P, N)):
        raise ValueError("inconsistent tensor shapes")
    _check_dev(x, dt, A, B, C, D, h0, y, final_state)
    st = _lib.ssd_prefill_static(ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(h0),
                                 _ptr(y), _ptr(final_state), _stream_ptr())
    if st != SSD_OK:
        raise SSDError(st, "ssd_prefill_static")
    return y, final_state


def ssd_decode_step(state, x, dt, A, B, C, D, y=None):
    """``ssd_decode_step``: updates ``state (Bt,H,P,N)`` in place, returns ``y (Bt,H,P)``."""
    Bt, H, P, N = state.shape
    G = B.shape[1]
    shape = make_shape(Bt, 1, H, P, N, G, 1, x.dtype)
    if y is None:
        y = torch.empty_like(x)
    if state.dtype != torch.float32 or tuple(x.shape) != (Bt, H, P) or tuple(dt.shape) != (Bt, H) \
            or tuple(B.shape) != (Bt, G, N) or tuple(C.shape) != (Bt, G, N):
        raise ValueError("inconsistent tensor shapes")
    _check_dev(state, x, dt, A, B, C, D, y)
    st = _lib.ssd_decode_step(ctypes.byref(shape), _ptr(state), _ptr(x), _ptr(dt), _ptr(A), _ptr(B),
                              _ptr(C), _ptr(D), _ptr(y), _stream_ptr())
    if st != SSD_OK:
        raise SSDError(st, "ssd_decode_step")
    return y


def ssd_decode_step_layers(state, x, dt, A, B, C, D, y=None, dt_bias=None, dt_softplus=False, dt_limit=None):
    """``ssd_decode_step_layers``: every tensor has a leading layer axis; one launch.  With ``dt_bias
    (Ly,H)``, ``dt_softplus`` or ``dt_limit=(lo, hi)`` the call goes through ``ssd_decode_step_layers_dt``
    and ``dt`` is the raw value."""
    Ly, Bt, H, P, N = state.shape
    G = B.shape[2]
    shape = make_shape(Bt, 1, H, P, N, G, 1, x.dtype)
    if y is None:
        y = torch.empty_like(x)
    if state.dtype != torch.float32 or tuple(x.shape) != (Ly, Bt, H, P) or tuple(dt.shape) != (Ly, Bt, H) \
            or tuple(A.shape) != (Ly, H) or tuple(D.shape) != (Ly, H) \
            or tuple(B.shape) != (Ly, Bt, G, N) or tuple(C.shape) != (Ly, Bt, G, N):
        raise ValueError("inconsistent tensor shapes")
    _check_dev(state, x, dt, A, B, C, D, y)
    xf = _dt_transform(dt_bias, dt_softplus, dt_limit, (Ly, H))
    tail = (_ptr(state), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(y), _stream_ptr())
    if xf is not None:
        st = _lib.ssd_decode_step_layers_dt(Ly, ctypes.byref(shape), ctypes.byref(xf), *tail)
    else:
        st = _lib.ssd_decode_step_layers(Ly, ctypes.byref(shape), *tail)
    if st != SSD_OK:
        raise SSDError(st, "ssd_decode_step_layers")
    return y


def ssd_decode_steps_layers(state, x, dt, A, B, C, D, y=None, dt_bias=None, dt_softplus=False, dt_limit=None):
    """``ssd_decode_steps_layers``: ``x (steps,Ly,Bt,H,P)``, ``dt (steps,Ly,Bt,H)``,
    ``B, C (steps,Ly,Bt,G,N)``, ``A, D (Ly,H)``; ``state (Ly,Bt,H,P,N)`` updated in place to the
    state after the last step.  Returns ``y (steps,Ly,Bt,H,P)``.  One launch.  ``dt_bias (Ly,H)``,
    ``dt_softplus``, ``dt_limit``: as for ``ssd_decode_step_layers`` (``ssd_decode_steps_layers_dt``)."""
    Ly, Bt, H, P, N = state.shape
    S, G = x.shape[0], B.shape[3]
    shape = make_shape(Bt, 1, H, P, N, G, 1, x.dtype)
    if y is None:
        y = torch.empty_like(x)
    if state.dtype != torch.float32 or tuple(x.shape) != (S, Ly, Bt, H, P) or tuple(dt.shape) != (S, Ly, Bt, H) \
            or tuple(A.shape) != (Ly, H) or tuple(D.shape) != (Ly, H) \
            or tuple(B.shape) != (S, Ly, Bt, G, N) or tuple(C.shape) != (S, Ly, Bt, G, N):
        raise ValueError("inconsistent tensor shapes")
    _check_dev(state, x, dt, A, B, C, D, y)
    xf = _dt_transform(dt_bias, dt_softplus, dt_limit, (Ly, H))
    tail = (_ptr(state), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(y), _stream_ptr())
    if xf is not None:
        st = _lib.ssd_decode_steps_layers_dt(S, Ly, ctypes.byref(shape), ctypes.byref(xf), *tail)
    else:
        st = _lib.ssd_decode_steps_layers(S, Ly, ctypes.byref(shape), *tail)
    if st != SSD_OK:
        raise SSDError(st, "ssd_decode_steps_layers")
    return y


def ssd_prefill_varlen(x, dt, A, B, C, D, cu_seqlens, chunk, h0=None, y=None, final_state=None, workspace=None,
                       dt_bias=None, dt_softplus=False, dt_limit=None):
    """``ssd_prefill_varlen``: packed batch ``x (tokens,H,P)``, ``dt (tokens,H)``, ``B, C (tokens,G,N)``,
    ``cu_seqlens (nseq+1)`` int32 on the device, ``h0 (nseq,H,P,N)`` optional.
    Returns ``(y (tokens,H,P), final_state (nseq,H,P,N))``.  ``dt_bias (H)``, ``dt_softplus``, ``dt_limit``: as
    for ``ssd_prefill`` (``ssd_prefill_varlen_dt``)."""
    T, H, P = x.shape
    G, N = B.shape[1], B.shape[2]
    nseq = cu_seqlens.numel() - 1
    if cu_seqlens.dtype != torch.int32 or nseq < 1:
        raise ValueError("cu_seqlens must hold nseq + 1 int32 values")
    shape = make_shape(nseq, T, H, P, N, G, chunk, x.dtype)
    if B.dtype != x.dtype or C.dtype != x.dtype:
        raise ValueError("x, B and C must share one dtype")
    if tuple(dt.shape) != (T, H) or tuple(A.shape) != (H,) or tuple(D.shape) != (H,) or tuple(B.shape) != (T, G, N) \
            or tuple(C.shape) != (T, G, N) or (h0 is not None and tuple(h0.shape) != (nseq, H, P, N)):
        raise ValueError("inconsistent tensor shapes")
    if y is None:
        y = torch.empty_like(x)
    if final_state is None:
        final_state = torch.empty((nseq, H, P, N), dtype=torch.float32, device=x.device)
    need = int(_lib.ssd_prefill_varlen_workspace_bytes(ctypes.byref(shape)))
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    _check_dev(x, dt, A, B, C, D, h0, y, final_state, workspace, cu_seqlens)
    xf = _dt_transform(dt_bias, dt_softplus, dt_limit, (H,))
    tail = (_ptr(cu_seqlens), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(h0), _ptr(y),
            _ptr(final_state), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_ptr())
    if xf is not None:
        st = _lib.ssd_prefill_varlen_dt(ctypes.byref(shape), ctypes.byref(xf), *tail)
    else:
        st = _lib.ssd_prefill_varlen(ctypes.byref(shape), *tail)
    if st != SSD_OK:
        raise SSDError(st, "ssd_prefill_varlen")
    return y, final_state


def _conv_split(channels, split):
    split = list(split) if split is not None else [channels]
    split += [0] * (3 - len(split))
    if len(split) != 3 or sum(split) != channels or split[0] < 1 or min(split) < 0:
        raise ValueError("split must be up to three non-negative widths summing to the channel count")
    return split


def ssd_conv1d_prefill(u, weight, bias=None, conv_state=None, split=None, activation="silu"):
    """``ssd_conv1d_prefill``: ``u (Bt,T,C)`` channels-last, ``weight (C,k)`` fp32, ``bias (C)`` fp32 or None,
    ``conv_state (Bt,C,k-1)`` or None.  Returns ``(outputs, new_conv_state)`` where outputs is a list of
    dense tensors ``(Bt,T,split[i])`` (one tensor ``(Bt,T,C)`` without ``split``)."""
    Bt, T, C = u.shape
    k = weight.shape[1]
    split = _conv_split(C, split)
    io = {torch.float32: SSD_F32, torch.bfloat16: SSD_BF16}.get(u.dtype, -1)
    if weight.dtype != torch.float32 or tuple(weight.shape) != (C, k) or (bias is not None and (
            bias.dtype != torch.float32 or tuple(bias.shape) != (C,))) or (conv_state is not None and (
            conv_state.dtype != u.dtype or tuple(conv_state.shape) != (Bt, C, k - 1))):
        raise ValueError("inconsistent tensor shapes or dtypes")
    outs = [torch.empty((Bt, T, w), dtype=u.dtype, device=u.device) if w > 0 else None for w in split]
    new_state = torch.empty((Bt, C, k - 1), dtype=u.dtype, device=u.device)
    _check_dev(u, weight, bias, conv_state, new_state, *outs)
    st = _lib.ssd_conv1d_prefill(Bt, T, k, io, (_i32 * 3)(*split), _ptr(u), _ptr(weight), _ptr(bias), _ptr(conv_state),
                                 _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]), _ptr(new_state),
                                 {"none": 0, "silu": 1}[activation], _stream_ptr())
    if st != SSD_OK:
        raise SSDError(st, "ssd_conv1d_prefill")
    return [o for o in outs if o is not None], new_state


def ssd_conv1d_step(conv_state, u, weight, bias=None, split=None, activation="silu"):
    """``ssd_conv1d_step``: ``u (Bt,C)``, ``conv_state (Bt,C,k-1)`` updated in place.  Returns the list of
    outputs ``(Bt,split[i])``."""
    Bt, C = u.shape
    k = weight.shape[1]
    split = _conv_split(C, split)
    io = {torch.float32: SSD_F32, torch.bfloat16: SSD_BF16}.get(u.dtype, -1)
    if weight.dtype != torch.float32 or tuple(weight.shape) != (C, k) or conv_state.dtype != u.dtype \
            or tuple(conv_state.shape) != (Bt, C, k - 1) or (bias is not None and tuple(bias.shape) != (C,)):
        raise ValueError("inconsistent tensor shapes or dtypes")
    outs = [torch.empty((Bt, w), dtype=u.dtype, device=u.device) if w > 0 else None for w in split]
    _check_dev(u, weight, bias, conv_state, *outs)
    st = _lib.ssd_conv1d_step(Bt, k, io, (_i32 * 3)(*split), _ptr(conv_state), _ptr(u), _ptr(weight), _ptr(bias),
                              _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]), {"none": 0, "silu": 1}[activation],
                              _stream_ptr())
    if st != SSD_OK:
        raise SSDError(st, "ssd_conv1d_step")
    return [o for o in outs if o is not None]


KNOBS = {"force_generic": 0, "seg_chunks": 1, "seg_blocks": 2, "seg_parts": 3, "y_stream": 4, "decode_stream": 5,
         "force_mfma_f32": 6, "f32_segments": 7, "fold_max_slots": 8}


def set_knob(name: str, value: int) -> None:
    """``ssd_testing_set_knob`` (include/ssd_testing.h): force a choice the library otherwise makes itself.
    Process-wide; for tests and tuning runs only."""
    st = _lib.ssd_testing_set_knob(KNOBS[name], int(value))
    if st != SSD_OK:
        raise SSDError(st, "ssd_testing_set_knob")


def reset_knobs() -> None:
    _lib.ssd_testing_reset_knobs()


def prefill_plan(shape, h0_aliases_final_state: bool = False) -> dict:
    """``ssd_testing_prefill_plan`` (include/ssd_testing.h): how ``ssd_prefill`` would run ``shape`` under the
    current knobs, as a dict.  Host arithmetic only."""
    out = (ctypes.c_int32 * 8)()
    st = _lib.ssd_testing_prefill_plan(ctypes.byref(shape), int(bool(h0_aliases_final_state)), out)
    if st != SSD_OK:
        raise SSDError(st, "ssd_testing_prefill_plan")
    return dict(path=("generic_f32", "mfma_bf16", "mfma_f32")[out[0]], seg_blocks=out[1], segments=out[2], parts=out[3],
                fold=bool(out[4]), f32_segments=out[5])
