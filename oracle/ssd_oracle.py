"""ctypes front end of the fp64 CPU oracle (``ssd_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module; the product path (``paper_2603_09555_amd``) never does, and this
module imports nothing from it.

What lives here besides argument marshalling is the *layout* reading of the paper:

* tensors follow the axis order of the einsum signatures in the appendix "Exact SSD
  Einsum Signatures": ``x, y: (batch, T, H, P)``, ``B, C: (batch, T, G, N)``,
  ``dt: (batch, T, H)``, state ``(batch, H, P, N)`` (section "The O(1) state cache");
* the appendix labels B and C with a head axis; Mamba-2 shares them across the
  ``H / G`` heads of a group, so head ``h`` reads group ``h // (H // G)``.

All values are converted to float64 before the C code sees them (fp32 -> fp64 and
bf16 -> fp32 -> fp64 are exact), and all results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssd_oracle.c")
_LIB = os.path.join(_HERE, "libssd_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile ``ssd_oracle.c`` with gcc into ``libssd_oracle.so`` next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        cmd = ["gcc", "-O2", "-march=native", "-fopenmp", "-shared", "-fPIC", "-std=c11",
               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            ip = ctypes.POINTER(ctypes.c_int32)
            lib.ssd_oracle_scan.restype = ctypes.c_int
            lib.ssd_oracle_scan.argtypes = [ctypes.c_int] * 5 + [dp, dp, dp, ip, dp, dp, dp, dp, dp, dp,
                                                                ctypes.c_int]
            lib.ssd_oracle_step.restype = ctypes.c_int
            lib.ssd_oracle_step.argtypes = [ctypes.c_int] * 4 + [dp, dp, dp, dp, ip, dp, dp, dp, dp,
                                                                ctypes.c_int]
            lib.ssd_oracle_max_threads.restype = ctypes.c_int
            _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().ssd_oracle_max_threads())


def _f64(a):
    """float64, C-contiguous numpy copy/view of an array-like (torch tensors included)."""
    if hasattr(a, "detach"):  # torch tensor; bf16 has no numpy dtype, go through fp32 (exact)
        a = a.detach().cpu()
        if str(a.dtype) == "torch.bfloat16":
            a = a.float()
        a = a.numpy()
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _dptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def scan_pairs(x, dt, A, bc_index, B, C, D, h0=None, nthreads: int = 0):
    """Raw per-pair scan: ``x (n,T,P)``, ``dt (n,T)``, ``A, D (n)``, ``bc_index (n)``,
    ``B, C (nbc,T,N)``, ``h0 (n,P,N)`` or None.  Returns ``y (n,T,P)``, ``state (n,P,N)``."""
    x, dt, A, B, C, D = (_f64(v) for v in (x, dt, A, B, C, D))
    bc_index = np.ascontiguousarray(bc_index, dtype=np.int32)
    n, T, P = x.shape
    nbc, TB, N = B.shape
    assert dt.shape == (n, T) and A.shape == (n,) and D.shape == (n,) and bc_index.shape == (n,)
    assert C.shape == B.shape and TB == T
    if h0 is not None:
        h0 = _f64(h0)
        assert h0.shape == (n, P, N)
    y = np.empty((n, T, P), dtype=np.float64)
    state = np.empty((n, P, N), dtype=np.float64)
    rc = _load().ssd_oracle_scan(n, T, P, N, nbc, _dptr(x), _dptr(dt), _dptr(A), _iptr(bc_index),
                                 _dptr(B), _dptr(C), _dptr(D), _dptr(h0), _dptr(y), _dptr(state),
                                 int(nthreads))
    if rc != 0:
        raise ValueError("ssd_oracle_scan rejected its arguments (rc=%d)" % rc)
    return y, state


def gather_pairs(x, dt, A, B, C, D, h0, pairs):
    """Pull the listed ``(b, h)`` sequences out of the tensor layouts (see module docstring).
    Returns the argument tuple of :func:`scan_pairs`."""
    Bt, T, H, P = x.shape
    G = B.shape[2]
    if H % G != 0:
        raise ValueError("nheads must be a multiple of ngroups")
    hpg = H // G
    pairs = np.asarray(pairs, dtype=np.int64).reshape(-1, 2)
    bs, hs = pairs[:, 0], pairs[:, 1]
    tonp = lambda a: a.detach().cpu().float().numpy() if hasattr(a, "detach") else np.asarray(a)
    xn, dtn, Bn, Cn = tonp(x), tonp(dt), tonp(B), tonp(C)
    xp = np.stack([xn[b, :, h, :] for b, h in zip(bs, hs)]) if len(bs) else np.zeros((0, T, P))
    dtp = np.stack([dtn[b, :, h] for b, h in zip(bs, hs)]) if len(bs) else np.zeros((0, T))
    # one B/C row per distinct (b, g) that the pairs touch
    keys = {}
    bc_index = np.empty(len(bs), dtype=np.int32)
    for i, (b, h) in enumerate(zip(bs, hs)):
        bc_index[i] = keys.setdefault((int(b), int(h) // hpg), len(keys))
    N = Bn.shape[3]
    Bp = np.zeros((max(len(keys), 1), T, N))
    Cp = np.zeros_like(Bp)
    for (b, g), j in keys.items():
        Bp[j] = Bn[b, :, g, :]
        Cp[j] = Cn[b, :, g, :]
    An, Dn = _f64(A), _f64(D)
    h0p = None
    if h0 is not None:
        h0n = tonp(h0)
        h0p = np.stack([h0n[b, h] for b, h in zip(bs, hs)]) if len(bs) else np.zeros((0, P, N))
    return xp, dtp, An[hs], bc_index, Bp, Cp, Dn[hs], h0p


def prefill(x, dt, A, B, C, D, h0=None, pairs=None, nthreads: int = 0):
    """Sequential-recurrence result for a whole prompt.

    ``x (Bt,T,H,P)``, ``dt (Bt,T,H)``, ``A, D (H)``, ``B, C (Bt,T,G,N)``, ``h0 (Bt,H,P,N)``.
    With ``pairs=None`` returns ``y (Bt,T,H,P)`` and ``state (Bt,H,P,N)``; with a list of
    ``(b, h)`` pairs returns only those sequences, ``y (n,T,P)`` and ``state (n,P,N)``.
    There is no chunk argument: the recurrence has none (the result of the chunked method
    does not depend on the chunk length).
    """
    Bt, T, H, P = x.shape
    full = pairs is None
    if full:
        pairs = [(b, h) for b in range(Bt) for h in range(H)]
    args = gather_pairs(x, dt, A, B, C, D, h0, pairs)
    y, state = scan_pairs(*args, nthreads=nthreads)
    if full:
        N = state.shape[-1]
        y = np.ascontiguousarray(y.reshape(Bt, H, T, P).transpose(0, 2, 1, 3))
        state = state.reshape(Bt, H, P, N)
    return y, state


def decode_step(state, x, dt, A, B, C, D, nthreads: int = 0):
    """One cached decode step (one iteration of the prefill loop).

    ``state (Bt,H,P,N)``, ``x (Bt,H,P)``, ``dt (Bt,H)``, ``A, D (H)``, ``B, C (Bt,G,N)``.
    Returns ``(y (Bt,H,P), new_state (Bt,H,P,N))`` as float64; the input is not modified.
    """
    st = _f64(state).copy()
    x, dt, A, B, C, D = (_f64(v) for v in (x, dt, A, B, C, D))
    Bt, H, P, N = st.shape
    G = B.shape[1]
    if H % G != 0:
        raise ValueError("nheads must be a multiple of ngroups")
    hpg = H // G
    n = Bt * H
    bc_index = np.ascontiguousarray(
        (np.arange(Bt)[:, None] * G + (np.arange(H)[None, :] // hpg)).reshape(-1), dtype=np.int32)
    Ap = np.ascontiguousarray(np.broadcast_to(A[None, :], (Bt, H)).reshape(-1))
    Dp = np.ascontiguousarray(np.broadcast_to(D[None, :], (Bt, H)).reshape(-1))
    y = np.empty((n, P), dtype=np.float64)
    rc = _load().ssd_oracle_step(n, P, N, Bt * G, _dptr(st), _dptr(x.reshape(n, P)), _dptr(dt.reshape(n)),
                                 _dptr(Ap), _iptr(bc_index), _dptr(B.reshape(Bt * G, N)),
                                 _dptr(C.reshape(Bt * G, N)), _dptr(Dp), _dptr(y), int(nthreads))
    if rc != 0:
        raise ValueError("ssd_oracle_step rejected its arguments (rc=%d)" % rc)
    return y.reshape(Bt, H, P), st


def decode_step_layers(state, x, dt, A, B, C, D, nthreads: int = 0):
    """``nlayers`` independent layers, every array with a leading layer axis
    (``A, D (Ly,H)``): the layer axis is just more independent sequences."""
    st = _f64(state)
    Ly = st.shape[0]
    ys, sts = [], []
    for l in range(Ly):
        y, s = decode_step(st[l], _f64(x)[l], _f64(dt)[l], _f64(A)[l], _f64(B)[l], _f64(C)[l], _f64(D)[l],
                           nthreads=nthreads)
        ys.append(y)
        sts.append(s)
    return np.stack(ys), np.stack(sts)


def decode_steps_layers(state, x, dt, A, B, C, D, nthreads: int = 0):
    """``nsteps`` consecutive decode steps (Alg. 2 applied once per leading index of the
    per-step arrays): ``x (S,Ly,Bt,H,P)``, ``dt (S,Ly,Bt,H)``, ``B, C (S,Ly,Bt,G,N)``,
    ``A, D (Ly,H)``, ``state (Ly,Bt,H,P,N)``.  Returns ``(y (S,Ly,Bt,H,P), state after the last step)``."""
    st = _f64(state)
    xs, dts, Bs, Cs = _f64(x), _f64(dt), _f64(B), _f64(C)
    ys = []
    for s in range(xs.shape[0]):
        y, st = decode_step_layers(st, xs[s], dts[s], A, Bs[s], Cs[s], D, nthreads=nthreads)
        ys.append(y)
    return np.stack(ys), st


def prefill_varlen(x, dt, A, B, C, D, cu_seqlens, h0=None, nthreads: int = 0):
    """Packed variable-length batch: sequence q owns tokens ``[cu[q], cu[q+1])`` of
    ``x (tokens,H,P)``, ``dt (tokens,H)``, ``B, C (tokens,G,N)`` and is scanned on its own from
    ``h0[q]`` (or zero): the recurrence of Eq. 2 restarted at every boundary.
    Returns ``y (tokens,H,P)`` (zeros outside every sequence) and ``state (nseq,H,P,N)``."""
    tonp = lambda a: a.detach().cpu().float().numpy() if hasattr(a, "detach") else np.asarray(a)
    xn, dtn, Bn, Cn = tonp(x), tonp(dt), tonp(B), tonp(C)
    cu = [int(v) for v in np.asarray(tonp(cu_seqlens)).reshape(-1)]
    T, H, P = xn.shape
    N = Bn.shape[2]
    nseq = len(cu) - 1
    y = np.zeros((T, H, P), dtype=np.float64)
    state = np.zeros((nseq, H, P, N), dtype=np.float64)
    h0n = None if h0 is None else _f64(h0)
    for q in range(nseq):
        a, b = cu[q], cu[q + 1]
        if b == a:  # no token: the state is untouched
            if h0n is not None:
                state[q] = h0n[q]
            continue
        yq, sq = prefill(xn[None, a:b], dtn[None, a:b], A, Bn[None, a:b], Cn[None, a:b], D,
                         h0=None if h0n is None else h0n[q:q + 1], nthreads=nthreads)
        y[a:b] = yq[0]
        state[q] = sq[0]
    return y, state


def conv1d_prefill(u, weight, bias=None, conv_state=None, activation="silu"):
    """Depthwise causal convolution with a rolling cache (Alg. 2, "Update conv state" and
    "DepthwiseConv"): ``u (Bt,T,C)``, ``weight (C,k)``, ``bias (C)``, ``conv_state (Bt,C,k-1)`` = the
    k-1 inputs before the prompt (zeros if None).  ``z[t,c] = act(bias[c] + sum_j weight[c,j] *
    window_t[j,c])`` with ``window_t`` the k inputs ending at token t.  Returns ``(z, new cache)``,
    float64.  Plain loops over tokens and taps."""
    u, weight = _f64(u), _f64(weight)
    Bt, T, C = u.shape
    k = weight.shape[1]
    prev = np.zeros((Bt, C, k - 1)) if conv_state is None else _f64(conv_state)
    ext = np.concatenate([prev.transpose(0, 2, 1), u], axis=1)      # (Bt, k-1+T, C)
    z = np.zeros((Bt, T, C))
    for t in range(T):
        for j in range(k):
            z[:, t, :] += weight[None, :, j] * ext[:, t + j, :]
    if bias is not None:
        z += _f64(bias)[None, None, :]
    if activation == "silu":
        z = z / (1.0 + np.exp(-z))
    elif activation != "none":
        raise ValueError("activation must be 'none' or 'silu'")
    new_state = np.ascontiguousarray(ext[:, T:, :].transpose(0, 2, 1))  # the last k-1 inputs
    return z, new_state


def conv1d_step(conv_state, u, weight, bias=None, activation="silu"):
    """One token of :func:`conv1d_prefill`: ``u (Bt,C)``.  Returns ``(z (Bt,C), new cache)``."""
    z, st = conv1d_prefill(_f64(u)[:, None, :], weight, bias, conv_state, activation)
    return z[:, 0, :], st


def dt_transform(raw, bias=None, softplus=False, limit=None):
    """Step size from the raw projection output (Alg. 1, "Discretise"; softplus and clip are the
    elementwise neighbours named in section "Mapping SSD onto JAX primitives"):
    ``clamp(softplus(raw + bias[h]), lo, hi)``, each part optional.  ``raw (..., H)``, float64 out."""
    v = _f64(raw).copy()
    if bias is not None:
        v = v + _f64(bias)
    if softplus:
        v = np.logaddexp(0.0, v)          # log(1 + exp(v)) without overflow
    if limit is not None:
        v = np.clip(v, limit[0], limit[1])
    return v
