"""ctypes binding of the measurement library ``libssd_measure.so`` (include/ssd_measure.h): per-kernel
timing of a prefill call and the machine-peak probes.  Used by ``bench.py`` and the tests of the probes;
the product path never loads it.  Both calls wait for the device."""
from __future__ import annotations

import ctypes
import os

import torch

from . import ssd as _ssd

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libssd_measure.so")
EXPORTS = ["ssd_prefill_profile", "ssd_peak_probe"]

if not os.path.exists(LIB_PATH):
    raise ImportError("libssd_measure.so is missing: build it with `python -m paper_2603_09555_amd.build`")

_lib = ctypes.CDLL(LIB_PATH)
_vp, _sz = ctypes.c_void_p, ctypes.c_size_t
_lib.ssd_peak_probe.restype = ctypes.c_int
_lib.ssd_peak_probe.argtypes = [ctypes.c_int32] * 3 + [_vp, _vp, _sz, ctypes.POINTER(ctypes.c_float),
                                ctypes.POINTER(ctypes.c_double), _vp]
_lib.ssd_prefill_profile.restype = ctypes.c_int
_lib.ssd_prefill_profile.argtypes = [ctypes.POINTER(_ssd.ssd_shape)] + [_vp] * 10 + \
    [_sz, _vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_char_p),
     ctypes.POINTER(ctypes.c_int32)]
_lib.ssd_prefill_workspace_bytes.restype = _sz
_lib.ssd_prefill_workspace_bytes.argtypes = [ctypes.POINTER(_ssd.ssd_shape)]


def raw():
    return _lib


def prefill_profile(x, dt, A, B, C, D, chunk, y, final_state, workspace, h0=None):
    """``ssd_prefill_profile``: one prefill with an event after every kernel.  Returns a list of
    ``(kernel name, milliseconds)``; ``y`` and ``final_state`` receive the results of ``ssd_prefill``."""
    Bt, T, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    shape = _ssd.make_shape(Bt, T, H, P, N, G, chunk, x.dtype)
    need = int(_lib.ssd_prefill_workspace_bytes(ctypes.byref(shape)))
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    ms = (ctypes.c_float * 8)()
    names = (ctypes.c_char_p * 8)()
    n = ctypes.c_int32(0)
    p = _ssd._ptr
    st = _lib.ssd_prefill_profile(ctypes.byref(shape), p(x), p(dt), p(A), p(B), p(C), p(D), p(h0), p(y),
                                  p(final_state), p(workspace), workspace.numel() * workspace.element_size(),
                                  _ssd._stream_ptr(), 8, ms, names, ctypes.byref(n))
    if st != _ssd.SSD_OK:
        raise _ssd.SSDError(st, "ssd_prefill_profile")
    return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def peak_probe(kind, a, b=None, iters=0, reps=1):
    """``ssd_peak_probe``: returns ``(work per second, milliseconds per launch)`` -- flop/s for
    ``kind="mfma"`` (bf16) and ``"mfma_f32"``, ``"mfma_f32_16x16x4"`` (the fp32 matrix instructions), bytes/s for ``"copy"``, ``"read"``, ``"write"`` and their non-temporal forms
    ``"copy_nt"``, ``"read_nt"``, ``"write_nt"``.  ``a``, ``b``: device tensors."""
    k = {"mfma": 0, "copy": 1, "read": 2, "write": 3, "copy_nt": 4, "read_nt": 5, "write_nt": 6,
         "mfma_f32": 7, "mfma_f32_16x16x4": 8}[kind]
    ms, work = ctypes.c_float(0), ctypes.c_double(0)
    nbytes = a.numel() * a.element_size() if k in (0, 1, 2, 4, 5, 7, 8) else b.numel() * b.element_size()
    _ssd._check_dev(a, b)
    st = _lib.ssd_peak_probe(k, iters, reps, _ssd._ptr(a), _ssd._ptr(b), nbytes, ctypes.byref(ms),
                             ctypes.byref(work), _ssd._stream_ptr())
    if st != _ssd.SSD_OK:
        raise _ssd.SSDError(st, "ssd_peak_probe")
    per = ms.value / reps
    return work.value / (per * 1e-3), per
