"""CPU model of the arithmetic of the bf16 MFMA prefill path.  TEST INFRASTRUCTURE ONLY.

The chunked identities of Alg. 1 / Eq. 3 evaluated on 64-token blocks in fp64, in the form the
MFMA kernels use -- the decay mask of a diagonal block factorised around the prefix sum at token
31, ``exp(cs_l - cs_s) = exp(cs_l - c31) * exp(c31 - cs_s)`` -- with the places where those kernels
round an MFMA operand to bf16 switchable one by one:

  ``state``  the copy of the carried state fed to the state -> output product ``C_l . H``
  ``xm``     the scaled input ``dt_s exp(c31 - cs_s) x_s``
  ``g``      the masked scores ``tril(C B^T)``
  ``y``      the output itself (the io dtype)

With every switch off the model equals the oracle to rounding (pinned in test_blocked_model.py), so
whatever error a switch adds is the error of that rounding alone.  It shares no code with the HIP
sources or the oracle; it exists to attribute errors the GPU parity tests see to a named rounding,
and to work out, on the CPU, for which step sizes the mid-block factorisation stays inside the fp32
exponent range (``block_half_spans``).

A block whose decay across either half exceeds ``steep_at`` (log2 units) is "steep": the two factors
would leave the fp32 exponent range there.  For such a block the model -- like the kernels -- keeps
the mask un-factorised: ``exp(cs_l - cs_s)``, whose exponent is never positive, multiplies the
scores of the head (``gh``, rounded like ``g``), the state -> output term is scaled by ``exp(cs_l)``
and the state update takes weights relative to the END of the block, ``dt_s exp(c63 - cs_s)``.
"""
from __future__ import annotations

import numpy as np
import torch

BLK = 64
LOG2E = 1.4426950408889634


def bf16(a):
    """Round to bf16 (nearest even) and return as float64."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.bfloat16().float().numpy().astype(np.float64)


def _np(t):
    if hasattr(t, "detach"):
        t = t.detach().float().cpu().numpy()
    return np.asarray(t, dtype=np.float64)


def block_half_spans(dt, A):
    """log2 of the decay across each half of every 64-token block: ``(Bt, H, nblocks, 2)``, values >= 0.
    The two mask factors of a block evaluate exponents up to these."""
    dt, A = _np(dt), _np(A)
    Bt, T, H = dt.shape
    nb = (T + BLK - 1) // BLK
    a = np.zeros((Bt, nb * BLK, H))
    a[:, :T] = -dt * A[None, None, :] * LOG2E
    a = a.reshape(Bt, nb, BLK, H)
    lo = a[:, :, 1:32].sum(axis=2)      # cs_0 - c31
    hi = a[:, :, 32:].sum(axis=2)       # c31 - c63
    return np.stack([lo, hi], axis=-1).transpose(0, 2, 1, 3)


def prefill(inp, h0=None, state=True, xm=True, g=True, y=True, clamp=None, steep_at=None):
    """``inp``: dict of x (Bt,T,H,P), dt (Bt,T,H), A (H), B, C (Bt,T,G,N), D (H).  ``clamp``: limit on the
    magnitude of the exponent of either mask factor (None: none).  ``steep_at``: half-block decay (log2)
    beyond which a block of a head takes the un-factorised form (None: never).
    Returns ``y, final_state`` (float64)."""
    x, dt, A, B, C, D = (_np(inp[k]) for k in ("x", "dt", "A", "B", "C", "D"))
    Bt, T, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    hpg = H // G
    out = np.zeros_like(x)
    S = np.zeros((Bt, H, P, N)) if h0 is None else _np(h0).copy()
    rnd = lambda on, v: bf16(v) if on else v
    for t0 in range(0, T, BLK):
        n = min(BLK, T - t0)
        pad = lambda v: np.concatenate([v, np.zeros((Bt, BLK - n) + v.shape[2:])], axis=1)
        dtb, xb = pad(dt[:, t0:t0 + n]), pad(x[:, t0:t0 + n])           # (Bt,64,H), (Bt,64,H,P)
        Bb, Cb = pad(B[:, t0:t0 + n]), pad(C[:, t0:t0 + n])             # (Bt,64,G,N)
        cs = np.cumsum(dtb * A[None, None, :] * LOG2E, axis=1)          # (Bt,64,H)
        c31, c63 = cs[:, 31:32], cs[:, 63:64]
        e_row, e_in = cs - c31, c31 - cs
        if clamp is not None:
            e_row, e_in = np.clip(e_row, -clamp, clamp), np.clip(e_in, -clamp, clamp)
        rowf = np.exp2(e_row)
        f = dtb * np.exp2(e_in)
        Gm = rnd(g, np.tril(np.einsum("blgn,bsgn->bgls", Cb, Bb)))      # (Bt,G,64,64)
        Xm = rnd(xm, f[..., None] * xb)                                   # (Bt,64,H,P)
        Ht = np.exp2(c31[:, 0])[:, :, None, None] * S                    # state at the middle of the block
        Hop = rnd(state, Ht)
        Gh, Ch, Bh = (np.repeat(v, hpg, axis=a) for v, a in ((Gm, 1), (Cb, 2), (Bb, 2)))
        Y = np.einsum("blhn,bhpn->blhp", Ch, Hop) + np.einsum("bhls,bshp->blhp", Gh, Xm)
        yb = rowf[..., None] * Y + D[None, None, :, None] * xb
        S_next = np.exp2(c63[:, 0] - c31[:, 0])[:, :, None, None] * (Ht + np.einsum("bshn,bshp->bhpn", Bh, Xm))
        if steep_at is not None:
            steep = np.maximum(cs[:, 0] - c31[:, 0], c31[:, 0] - c63[:, 0]) > steep_at          # (Bt,H)
            if steep.any():
                mask = np.exp2(np.minimum(cs[:, :, None, :] - cs[:, None, :, :], 0.0))             # (Bt,l,s,H)
                Gs = rnd(g, np.einsum("bhls,blsh,bsh->bhls", Gh, mask, dtb))                       # tril is in Gh
                Sop = rnd(state, S)
                Ys = (np.exp2(cs)[..., None] * np.einsum("blhn,bhpn->blhp", Ch, Sop) +
                      np.einsum("bhls,bshp->blhp", Gs, xb))
                ys = Ys + D[None, None, :, None] * xb
                Xe = rnd(xm, (dtb * np.exp2(c63 - cs))[..., None] * xb)
                Ss = np.exp2(c63[:, 0])[:, :, None, None] * S + np.einsum("bshn,bshp->bhpn", Bh, Xe)
                yb = np.where(steep[:, None, :, None], ys, yb)
                S_next = np.where(steep[:, :, None, None], Ss, S_next)
        yb = rnd(y, yb)
        out[:, t0:t0 + n] = yb[:, :n]
        S = S_next
    return out, S
