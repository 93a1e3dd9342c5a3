"""Pins for an implementation of the SSD layer core.

Every ``check_*`` function takes ``prefill(x, dt, A, B, C, D, h0=None) -> (y, state)`` and
``step(state, x, dt, A, B, C, D) -> (y, new_state)`` in the tensor layouts
``x (Bt,T,H,P)``, ``dt (Bt,T,H)``, ``A, D (H)``, ``B, C (Bt,T,G,N)``, state ``(Bt,H,P,N)``
(numpy float64 in, numpy float64 out) and raises ``AssertionError`` when the implementation
disagrees with what the paper and the mathematics fix independently of it.  None of them
re-types the token recurrence: they use a hand-worked example, closed forms, reductions to
library routines (``numpy.tril`` + matmul, ``scipy.signal.lfilter``), the O(T^2) kernel form
of Eq. 3 written out with explicit sums, and invariants.

The same checks are run (a) on the oracle, which must pass them all, and (b) on deliberately
broken re-implementations ("mutants"), each of which must be caught by at least one check.
"""
from __future__ import annotations

import json
import os

import numpy as np
from scipy.signal import lfilter

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def random_problem(seed, Bt=2, T=7, H=4, P=3, N=5, G=2, with_h0=False):
    r = _rng(seed)
    p = dict(
        x=r.standard_normal((Bt, T, H, P)),
        dt=r.uniform(0.01, 0.6, (Bt, T, H)),
        A=-np.exp(r.uniform(0.0, np.log(16.0), H)),
        B=r.standard_normal((Bt, T, G, N)),
        C=r.standard_normal((Bt, T, G, N)),
        D=r.standard_normal(H),
    )
    if with_h0:
        p["h0"] = r.standard_normal((Bt, H, P, N))
    return p


def _close(a, b, rtol=1e-12, atol=1e-12, what=""):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, "%s: shape %s vs %s" % (what, a.shape, b.shape)
    err = np.abs(a - b)
    tol = atol + rtol * np.abs(b)
    assert np.all(err <= tol), "%s: max err %.3e (tol %.1e/%.1e)" % (what, float(err.max()), rtol, atol)


# 1. the hand-worked example ---------------------------------------------------------------
def load_hand_example():
    with open(os.path.join(GOLDEN, "hand_example.json")) as f:
        g = json.load(f)
    T, P, N = 4, 2, 2
    x = np.array(g["x"], dtype=np.float64).reshape(1, T, 1, P)
    dt = np.array(g["dt"], dtype=np.float64).reshape(1, T, 1)
    B = np.array(g["B"], dtype=np.float64).reshape(1, T, 1, N)
    C = np.array(g["C"], dtype=np.float64).reshape(1, T, 1, N)
    A = np.array([-np.log(2.0)])
    D = np.array(g["D"], dtype=np.float64)
    y = np.array(g["y"], dtype=np.float64).reshape(1, T, 1, P)
    states = np.array(g["state_after"], dtype=np.float64)  # (T, P, N)
    return dict(x=x, dt=dt, A=A, B=B, C=C, D=D), y, states


def check_hand_example(prefill, step):
    p, y_ref, states = load_hand_example()
    y, st = prefill(**p)
    _close(y, y_ref, rtol=4e-16, atol=0, what="hand example y")
    _close(st[0, 0], states[-1], rtol=4e-16, atol=0, what="hand example final state")
    # every prefix: the state after t tokens is the printed one
    for t in range(1, 5):
        q = {k: (v[:, :t] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
        yt, stt = prefill(**q)
        _close(stt[0, 0], states[t - 1], rtol=4e-16, atol=0, what="hand example state after %d" % t)
        _close(yt, y_ref[:, :t], rtol=4e-16, atol=0, what="hand example y prefix %d" % t)
    # three tokens of prefill, then the fourth as a decode step
    q = {k: (v[:, :3] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
    _, st3 = prefill(**q)
    y4, st4 = step(st3, p["x"][:, 3], p["dt"][:, 3], p["A"], p["B"][:, 3], p["C"][:, 3], p["D"])
    _close(y4, y_ref[:, 3], rtol=4e-16, atol=0, what="hand example decode y")
    _close(st4[0, 0], states[3], rtol=4e-16, atol=0, what="hand example decode state")


# 2. closed form for constant dt, A, x, B, C ------------------------------------------------
def check_closed_form_constant(prefill, step):
    r = _rng(11)
    T, P, N = 40, 3, 4
    delta, alpha, Dh = 0.07, -3.5, 0.8
    xv, Bv, Cv = r.standard_normal(P), r.standard_normal(N), r.standard_normal(N)
    x = np.broadcast_to(xv, (1, T, 1, P)).copy()
    B = np.broadcast_to(Bv, (1, T, 1, N)).copy()
    C = np.broadcast_to(Cv, (1, T, 1, N)).copy()
    dt = np.full((1, T, 1), delta)
    y, st = prefill(x, dt, np.array([alpha]), B, C, np.array([Dh]))
    rho = np.exp(delta * alpha)
    t = np.arange(1, T + 1)
    geo = delta * (1.0 - rho ** t) / (1.0 - rho)  # sum_{k<t} rho^k * delta
    y_ref = (Cv @ Bv) * geo[:, None] * xv[None, :] + Dh * xv[None, :]
    _close(y[0, :, 0, :], y_ref, rtol=1e-12, atol=1e-13, what="closed form y")
    _close(st[0, 0], geo[-1] * np.outer(xv, Bv), rtol=1e-12, atol=1e-13, what="closed form state")


# 3. A = 0: causal linear attention, by numpy.tril and matmul --------------------------------
def check_A_zero_linear_attention(prefill, step):
    p = random_problem(3, Bt=2, T=9, H=4, P=3, N=5, G=2)
    p["A"] = np.zeros_like(p["A"])
    y, st = prefill(**p)
    Bt, T, H, P = p["x"].shape
    hpg = H // p["B"].shape[2]
    for b in range(Bt):
        for h in range(H):
            g = h // hpg
            Cm, Bm = p["C"][b, :, g, :], p["B"][b, :, g, :]
            X = p["dt"][b, :, h, None] * p["x"][b, :, h, :]
            y_ref = np.tril(Cm @ Bm.T) @ X + p["D"][h] * p["x"][b, :, h, :]
            _close(y[b, :, h, :], y_ref, rtol=1e-12, atol=1e-12, what="A=0 y")
            _close(st[b, h], X.T @ Bm, rtol=1e-12, atol=1e-12, what="A=0 state")


# 4. N = 1, B = C = 1: first-order IIR filter, by scipy.signal.lfilter ------------------------
def check_ema_lfilter(prefill, step):
    r = _rng(5)
    T, P = 50, 2
    delta, alpha, Dh = 0.2, -1.3, -0.4
    x = r.standard_normal((1, T, 1, P))
    ones = np.ones((1, T, 1, 1))
    y, st = prefill(x, np.full((1, T, 1), delta), np.array([alpha]), ones, ones, np.array([Dh]))
    rho = np.exp(delta * alpha)
    for p_ in range(P):
        hseq = lfilter([delta], [1.0, -rho], x[0, :, 0, p_])
        _close(y[0, :, 0, p_], hseq + Dh * x[0, :, 0, p_], rtol=1e-12, atol=1e-13, what="EMA y")
        _close(st[0, 0, p_, 0], hseq[-1], rtol=1e-12, atol=1e-13, what="EMA state")


# 5. brute force: the O(T^2) kernel form of Eq. 3 with one chunk = the whole sequence --------
def kernel_form(x, dt, A, B, C, D, h0=None):
    """y_t = sum_{s<=t} (C_t.B_s) exp(sum_{j=s+1..t} dt_j A) dt_s x_s + D x_t (+ the h0 term),
    written with explicit sums; state = sum_s exp(sum_{j>s} dt_j A) dt_s x_s (x) B_s."""
    Bt, T, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    hpg = H // G
    y = np.zeros((Bt, T, H, P))
    st = np.zeros((Bt, H, P, N))
    for b in range(Bt):
        for h in range(H):
            g = h // hpg
            a = dt[b, :, h] * A[h]
            for t in range(T):
                acc = np.zeros(P)
                for s in range(t + 1):
                    decay = np.exp(np.sum(a[s + 1:t + 1]))
                    acc += np.dot(C[b, t, g], B[b, s, g]) * decay * dt[b, s, h] * x[b, s, h]
                if h0 is not None:
                    acc += np.exp(np.sum(a[:t + 1])) * (h0[b, h] @ C[b, t, g])
                y[b, t, h] = acc + D[h] * x[b, t, h]
            for s in range(T):
                st[b, h] += np.exp(np.sum(a[s + 1:])) * dt[b, s, h] * np.outer(x[b, s, h], B[b, s, g])
            if h0 is not None:
                st[b, h] += np.exp(np.sum(a)) * h0[b, h]
    return y, st


def check_brute_force(prefill, step):
    for seed, kw in [(1, dict(Bt=2, T=7, H=4, P=3, N=5, G=2)), (2, dict(Bt=1, T=12, H=6, P=2, N=3, G=3)),
                     (4, dict(Bt=3, T=5, H=2, P=4, N=4, G=1))]:
        p = random_problem(seed, **kw)
        y, st = prefill(**p)
        y_ref, st_ref = kernel_form(**p)
        _close(y, y_ref, rtol=1e-11, atol=1e-12, what="brute force y seed %d" % seed)
        _close(st, st_ref, rtol=1e-11, atol=1e-12, what="brute force state seed %d" % seed)
    p = random_problem(6, Bt=2, T=6, H=4, P=3, N=5, G=2, with_h0=True)
    y, st = prefill(**p)
    y_ref, st_ref = kernel_form(**p)
    _close(y, y_ref, rtol=1e-11, atol=1e-12, what="brute force y with h0")
    _close(st, st_ref, rtol=1e-11, atol=1e-12, what="brute force state with h0")


# 6. T = 1 ------------------------------------------------------------------------------------
def check_single_token(prefill, step):
    p = random_problem(8, Bt=2, T=1, H=4, P=3, N=5, G=2)
    y, st = prefill(**p)
    hpg = 2
    for b in range(2):
        for h in range(4):
            g = h // hpg
            cb = p["C"][b, 0, g] @ p["B"][b, 0, g]
            _close(y[b, 0, h], cb * p["dt"][b, 0, h] * p["x"][b, 0, h] + p["D"][h] * p["x"][b, 0, h],
                   what="T=1 y")
            _close(st[b, h], p["dt"][b, 0, h] * np.outer(p["x"][b, 0, h], p["B"][b, 0, g]), what="T=1 state")


# 7. invariants -------------------------------------------------------------------------------
def check_prefill_plus_decode(prefill, step):
    """prefill(T+1) == prefill(T) followed by one decode step (cached decode reproduces the
    recompute-everything baseline)."""
    p = random_problem(9, Bt=2, T=9, H=4, P=3, N=5, G=2, with_h0=True)
    y_all, st_all = prefill(**p)
    q = {k: (v[:, :-1] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
    y_pre, st_pre = prefill(**q)
    y_last, st_last = step(st_pre, p["x"][:, -1], p["dt"][:, -1], p["A"], p["B"][:, -1], p["C"][:, -1], p["D"])
    _close(y_pre, y_all[:, :-1], what="T+1: prefix y")
    _close(y_last, y_all[:, -1], what="T+1: decode y")
    _close(st_last, st_all, what="T+1: state")


def check_split_with_h0(prefill, step):
    p = random_problem(10, Bt=2, T=11, H=4, P=3, N=5, G=2)
    y_all, st_all = prefill(**p)
    for cut in (0, 1, 4, 11):
        q1 = {k: (v[:, :cut] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
        q2 = {k: (v[:, cut:] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
        y1, st1 = prefill(**q1)
        y2, st2 = prefill(h0=st1, **q2)
        _close(np.concatenate([y1, y2], axis=1), y_all, what="split y cut %d" % cut)
        _close(st2, st_all, what="split state cut %d" % cut)


def check_linearity_and_decay(prefill, step):
    p = random_problem(12, Bt=1, T=8, H=2, P=3, N=4, G=1)
    p2 = dict(p)
    p2["x"] = random_problem(13, Bt=1, T=8, H=2, P=3, N=4, G=1)["x"]
    ya, sa = prefill(**p)
    yb, sb = prefill(**p2)
    p3 = dict(p)
    p3["x"] = 2.0 * p["x"] - 3.0 * p2["x"]
    yc, sc = prefill(**p3)
    _close(yc, 2.0 * ya - 3.0 * yb, rtol=1e-11, atol=1e-11, what="linearity y")
    _close(sc, 2.0 * sa - 3.0 * sb, rtol=1e-11, atol=1e-11, what="linearity state")
    # zero input: the state only decays, state_T = exp(A * sum dt) * h0, y_t = C_t . h_t
    h0 = _rng(14).standard_normal((1, 2, 3, 4))
    pz = dict(p)
    pz["x"] = np.zeros_like(p["x"])
    yz, sz = prefill(h0=h0, **pz)
    tot = np.exp(p["A"][None, :] * p["dt"].sum(axis=1))  # (Bt, H)
    _close(sz, tot[:, :, None, None] * h0, rtol=1e-12, atol=1e-13, what="pure decay state")
    cum = np.exp(p["A"][None, None, :] * np.cumsum(p["dt"], axis=1))  # (Bt, T, H)
    y_ref = np.einsum("bth,bhpn,btn->bthp", cum, h0, p["C"][:, :, 0, :])
    _close(yz, y_ref, rtol=1e-12, atol=1e-13, what="pure decay y")


def check_batch_head_independence(prefill, step):
    p = random_problem(15, Bt=3, T=6, H=4, P=3, N=5, G=2)
    y, st = prefill(**p)
    q = {k: (v[1:2] if k in ("x", "dt", "B", "C") else v) for k, v in p.items()}
    y1, st1 = prefill(**q)
    _close(y1, y[1:2], rtol=0, atol=0, what="batch row independence y")
    _close(st1, st[1:2], rtol=0, atol=0, what="batch row independence state")
    # changing head 3's input must not change heads 0..2
    p2 = {k: v.copy() for k, v in p.items()}
    p2["x"][:, :, 3, :] += 1.0
    y2, _ = prefill(**p2)
    _close(y2[:, :, :3], y[:, :, :3], rtol=0, atol=0, what="head independence")
    assert np.abs(y2[:, :, 3] - y[:, :, 3]).max() > 1e-3


ALL_CHECKS = [check_hand_example, check_closed_form_constant, check_A_zero_linear_attention,
              check_ema_lfilter, check_brute_force, check_single_token, check_prefill_plus_decode,
              check_split_with_h0, check_linearity_and_decay, check_batch_head_independence]
