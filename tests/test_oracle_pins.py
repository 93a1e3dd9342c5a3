"""The oracle against what the paper and the mathematics fix (CPU only), and proof that
those pins have teeth: each deliberately wrong variant of the recurrence is rejected."""
import numpy as np
import pytest

import pins
from oracle import ssd_oracle


def oracle_prefill(x, dt, A, B, C, D, h0=None):
    return ssd_oracle.prefill(x, dt, A, B, C, D, h0=h0)


def oracle_step(state, x, dt, A, B, C, D):
    return ssd_oracle.decode_step(state, x, dt, A, B, C, D)


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_oracle_passes_pin(check):
    check(oracle_prefill, oracle_step)


# ---- mutants: the token recurrence with one planted mistake each -----------------------------
MUTATIONS = [
    "y_reads_old_state",      # y_t = C h_{t-1} + D x_t
    "no_dt_on_B",             # Bbar = B
    "zoh_B",                  # Bbar = (exp(dt A) - 1)/A * B  (true zero-order hold, not what Alg. 2 uses)
    "decay_sign",             # Abar = exp(-dt A)
    "decay_no_dt",            # Abar = exp(A)
    "D_on_dt_x",              # y += D * dt * x
    "no_D",                   # y has no skip term
    "swap_B_C",               # update with C, read out with B
    "group_modulo",           # head h reads group h % G
    "decay_after_add",        # h = Abar * (h + Bbar x)
    "h0_ignored",             # prefill always starts from zero
    "state_transposed",       # state returned as (N, P) data in a (P, N) buffer
    "decode_skips_decay",     # the decode step forgets Abar
    "x_outer_transposed",     # h[p][n] += u[n % P] * B[p % N]
]


def make_mutant(kind):
    def scan(x, dt, A, B, C, D, h0, decode):
        Bt, T, H, P = x.shape
        G, N = B.shape[2], B.shape[3]
        hpg = H // G
        y = np.zeros((Bt, T, H, P))
        st = np.zeros((Bt, H, P, N))
        for b in range(Bt):
            for h in range(H):
                g = (h % G) if kind == "group_modulo" else h // hpg
                S = np.zeros((P, N))
                if h0 is not None and not (kind == "h0_ignored" and not decode):
                    S = np.array(h0[b, h], dtype=np.float64)
                for t in range(T):
                    d = dt[b, t, h]
                    dA = np.exp(d * A[h])
                    if kind == "decay_sign":
                        dA = np.exp(-d * A[h])
                    if kind == "decay_no_dt":
                        dA = np.exp(A[h])
                    if kind == "decode_skips_decay" and decode:
                        dA = 1.0
                    Bb = d * B[b, t, g]
                    if kind == "no_dt_on_B":
                        Bb = B[b, t, g]
                    if kind == "zoh_B":
                        Bb = (np.exp(d * A[h]) - 1.0) / A[h] * B[b, t, g] if A[h] != 0 else d * B[b, t, g]
                    Cr = C[b, t, g]
                    if kind == "swap_B_C":
                        Bb, Cr = d * C[b, t, g], B[b, t, g]
                    S_old = S
                    upd = np.outer(x[b, t, h], Bb)
                    if kind == "x_outer_transposed":
                        upd = np.array([[x[b, t, h, n % P] * Bb[p % N] for n in range(N)] for p in range(P)])
                    if kind == "decay_after_add":
                        S = dA * (S + upd)
                    else:
                        S = dA * S + upd
                    yy = (S_old if kind == "y_reads_old_state" else S) @ Cr
                    if kind == "D_on_dt_x":
                        yy = yy + D[h] * d * x[b, t, h]
                    elif kind != "no_D":
                        yy = yy + D[h] * x[b, t, h]
                    y[b, t, h] = yy
                st[b, h] = S.T.reshape(P, N) if kind == "state_transposed" else S
        return y, st

    def prefill(x, dt, A, B, C, D, h0=None):
        return scan(x, dt, A, B, C, D, h0, decode=False)

    def step(state, x, dt, A, B, C, D):
        y, st = scan(x[:, None], dt[:, None], A, B[:, None], C[:, None], D, state, decode=True)
        return y[:, 0], st

    return prefill, step


def test_unmutated_reimplementation_passes_every_pin():
    """Guards the mutant harness itself: with no mistake planted it must pass."""
    prefill, step = make_mutant("none")
    for check in pins.ALL_CHECKS:
        check(prefill, step)


@pytest.mark.parametrize("kind", MUTATIONS)
def test_pins_catch_mutant(kind):
    prefill, step = make_mutant(kind)
    caught = []
    for check in pins.ALL_CHECKS:
        try:
            check(prefill, step)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin notices the planted mistake %r" % kind


def test_oracle_matches_unmutated_reimplementation_bitwise_order():
    """Same summation order in C and in the Python loops above => agreement to a few ulp."""
    p = pins.random_problem(21, Bt=2, T=9, H=4, P=3, N=5, G=2, with_h0=True)
    y, st = oracle_prefill(**p)
    y2, st2 = make_mutant("none")[0](**p)
    np.testing.assert_allclose(y, y2, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(st, st2, rtol=1e-13, atol=1e-14)


def test_pairs_subset_equals_full():
    p = pins.random_problem(22, Bt=3, T=8, H=6, P=4, N=5, G=3, with_h0=True)
    y, st = oracle_prefill(**p)
    pairs = [(2, 5), (0, 0), (1, 3), (2, 2)]
    yp, sp = ssd_oracle.prefill(p["x"], p["dt"], p["A"], p["B"], p["C"], p["D"], h0=p["h0"], pairs=pairs)
    for i, (b, h) in enumerate(pairs):
        np.testing.assert_array_equal(yp[i], y[b, :, h, :])
        np.testing.assert_array_equal(sp[i], st[b, h])


def test_thread_count_does_not_change_results():
    p = pins.random_problem(23, Bt=2, T=16, H=8, P=4, N=8, G=2)
    y1, s1 = ssd_oracle.prefill(p["x"], p["dt"], p["A"], p["B"], p["C"], p["D"], nthreads=1)
    y4, s4 = ssd_oracle.prefill(p["x"], p["dt"], p["A"], p["B"], p["C"], p["D"], nthreads=4)
    np.testing.assert_array_equal(y1, y4)
    np.testing.assert_array_equal(s1, s4)


def test_decode_layers_equals_per_layer():
    r = np.random.default_rng(3)
    Ly, Bt, H, P, N, G = 3, 2, 4, 3, 5, 2
    st = r.standard_normal((Ly, Bt, H, P, N))
    x = r.standard_normal((Ly, Bt, H, P))
    dt = r.uniform(0.01, 0.1, (Ly, Bt, H))
    A = -r.uniform(1, 16, (Ly, H))
    D = r.standard_normal((Ly, H))
    B = r.standard_normal((Ly, Bt, G, N))
    C = r.standard_normal((Ly, Bt, G, N))
    y, s2 = ssd_oracle.decode_step_layers(st, x, dt, A, B, C, D)
    for l in range(Ly):
        yl, sl = ssd_oracle.decode_step(st[l], x[l], dt[l], A[l], B[l], C[l], D[l])
        np.testing.assert_array_equal(y[l], yl)
        np.testing.assert_array_equal(s2[l], sl)


def test_decode_steps_equal_the_scan_over_the_same_tokens():
    """Several decode steps (the step routine applied repeatedly) against the scan routine run
    over the same tokens from the same initial state: two separate C functions."""
    r = np.random.default_rng(5)
    S, Ly, Bt, H, P, N, G = 6, 2, 2, 4, 3, 5, 2
    st = r.standard_normal((Ly, Bt, H, P, N))
    x = r.standard_normal((S, Ly, Bt, H, P))
    dt = r.uniform(0.01, 0.1, (S, Ly, Bt, H))
    A = -r.uniform(1, 16, (Ly, H))
    D = r.standard_normal((Ly, H))
    B = r.standard_normal((S, Ly, Bt, G, N))
    C = r.standard_normal((S, Ly, Bt, G, N))
    y, s2 = ssd_oracle.decode_steps_layers(st, x, dt, A, B, C, D)
    assert y.shape == (S, Ly, Bt, H, P) and s2.shape == st.shape
    for l in range(Ly):
        yl, sl = ssd_oracle.prefill(x[:, l].transpose(1, 0, 2, 3), dt[:, l].transpose(1, 0, 2), A[l],
                                    B[:, l].transpose(1, 0, 2, 3), C[:, l].transpose(1, 0, 2, 3), D[l], h0=st[l])
        np.testing.assert_allclose(y[:, l].transpose(1, 0, 2, 3), yl, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(s2[l], sl, rtol=1e-12, atol=1e-12)


def packed_kernel_form(x, dt, A, B, C, D, cu, h0=None):
    """The O(T^2) form of Eq. 3 over the PACKED token axis with a block-diagonal mask:
    y_t = sum_{s<=t, seq(s)=seq(t)} (C_t.B_s) exp(sum_{j=s+1..t} dt_j A) dt_s x_s + D x_t
    (+ the h0 term decayed from the start of t's sequence).  No slicing per sequence."""
    T, H, P = x.shape
    G, N = B.shape[1], B.shape[2]
    hpg = H // G
    seq = np.full(T, -1)
    for q in range(len(cu) - 1):
        seq[cu[q]:cu[q + 1]] = q
    y = np.zeros((T, H, P))
    st = np.zeros((len(cu) - 1, H, P, N)) if h0 is None else np.array(h0, dtype=np.float64)
    for h in range(H):
        g = h // hpg
        a = dt[:, h] * A[h]
        ca = np.concatenate([[0.0], np.cumsum(a)])          # ca[t+1] = sum_{j<=t} a_j
        for t in range(T):
            if seq[t] < 0:
                continue
            acc = np.zeros(P)
            for s in range(t + 1):
                if seq[s] == seq[t]:
                    acc += np.dot(C[t, g], B[s, g]) * np.exp(ca[t + 1] - ca[s + 1]) * dt[s, h] * x[s, h]
            if h0 is not None:
                acc += np.exp(ca[t + 1] - ca[cu[seq[t]]]) * (h0[seq[t], h] @ C[t, g])
            y[t, h] = acc + D[h] * x[t, h]
        for q in range(len(cu) - 1):
            e = cu[q + 1]
            if e == cu[q]:
                continue
            acc = np.zeros((P, N))
            for s in range(cu[q], e):
                acc += np.exp(ca[e] - ca[s + 1]) * dt[s, h] * np.outer(x[s, h], B[s, g])
            if h0 is not None:
                acc += np.exp(ca[e] - ca[cu[q]]) * h0[q, h]
            st[q, h] = acc
    return y, st


def test_varlen_oracle_against_block_diagonal_kernel_form():
    r = np.random.default_rng(11)
    T, H, P, N, G = 23, 4, 3, 5, 2
    cu = [2, 2, 9, 10, 10, 21]      # leading gap, empty sequences, a single token, trailing gap
    x = r.standard_normal((T, H, P))
    dt = r.uniform(0.01, 0.3, (T, H))
    A = -r.uniform(0.5, 4, H)
    D = r.standard_normal(H)
    B = r.standard_normal((T, G, N))
    C = r.standard_normal((T, G, N))
    for h0 in (None, r.standard_normal((len(cu) - 1, H, P, N))):
        y, st = ssd_oracle.prefill_varlen(x, dt, A, B, C, D, np.array(cu, dtype=np.int32), h0=h0)
        y_ref, st_ref = packed_kernel_form(x, dt, A, B, C, D, cu, h0=h0)
        np.testing.assert_allclose(y, y_ref, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(st, st_ref, rtol=1e-11, atol=1e-12)
        assert not y[:2].any() and not y[21:].any()


def test_varlen_oracle_equal_lengths_is_the_batched_prefill():
    r = np.random.default_rng(12)
    Bt, T, H, P, N, G = 3, 6, 4, 2, 3, 1
    x = r.standard_normal((Bt, T, H, P))
    dt = r.uniform(0.01, 0.3, (Bt, T, H))
    A = -r.uniform(0.5, 4, H)
    D = r.standard_normal(H)
    B = r.standard_normal((Bt, T, G, N))
    C = r.standard_normal((Bt, T, G, N))
    h0 = r.standard_normal((Bt, H, P, N))
    y, st = ssd_oracle.prefill(x, dt, A, B, C, D, h0=h0)
    cu = np.arange(Bt + 1, dtype=np.int32) * T
    yv, stv = ssd_oracle.prefill_varlen(x.reshape(Bt * T, H, P), dt.reshape(Bt * T, H), A, B.reshape(Bt * T, G, N),
                                        C.reshape(Bt * T, G, N), D, cu, h0=h0)
    np.testing.assert_array_equal(yv.reshape(Bt, T, H, P), y)
    np.testing.assert_array_equal(stv, st)


# ---- the depthwise convolution in front of the core -------------------------------------------
def test_conv_hand_example_one_step():
    """k = 4, one channel: cache (oldest first) [1, 2, 3], input 4, weights [0.5, -1, 2, 0.25],
    bias 0.125: z = 0.5*1 - 1*2 + 2*3 + 0.25*4 + 0.125 = 5.625; the cache becomes [2, 3, 4]."""
    st = np.array([[[1.0, 2.0, 3.0]]])
    z, st2 = ssd_oracle.conv1d_step(st, np.array([[4.0]]), np.array([[0.5, -1.0, 2.0, 0.25]]), np.array([0.125]),
                                    activation="none")
    assert z.shape == (1, 1) and z[0, 0] == 5.625
    np.testing.assert_array_equal(st2, [[[2.0, 3.0, 4.0]]])
    zs, _ = ssd_oracle.conv1d_step(st, np.array([[4.0]]), np.array([[0.5, -1.0, 2.0, 0.25]]), np.array([0.125]))
    np.testing.assert_allclose(zs[0, 0], 5.625 / (1.0 + np.exp(-5.625)), rtol=1e-15)


def test_conv_prefill_is_an_fir_filter():
    """Zero cache, no activation: per channel the prompt is filtered by the FIR filter whose taps are
    the weights reversed (scipy.signal.lfilter), and equals the head of numpy's full convolution."""
    from scipy.signal import lfilter
    r = np.random.default_rng(21)
    Bt, T, C, k = 2, 19, 5, 4
    u = r.standard_normal((Bt, T, C))
    w = r.standard_normal((C, k))
    b = r.standard_normal(C)
    z, st = ssd_oracle.conv1d_prefill(u, w, b, None, activation="none")
    for bi in range(Bt):
        for c in range(C):
            np.testing.assert_allclose(z[bi, :, c], lfilter(w[c, ::-1], [1.0], u[bi, :, c]) + b[c], rtol=1e-12,
                                       atol=1e-12)
            np.testing.assert_allclose(z[bi, :, c], np.convolve(u[bi, :, c], w[c, ::-1])[:T] + b[c], rtol=1e-12,
                                       atol=1e-12)
    np.testing.assert_array_equal(st, u[:, T - (k - 1):, :].transpose(0, 2, 1))


def test_conv_split_prompt_and_steps_agree_with_one_prefill():
    r = np.random.default_rng(22)
    Bt, T, C, k = 2, 11, 3, 4
    u = r.standard_normal((Bt, T, C))
    w = r.standard_normal((C, k))
    b = r.standard_normal(C)
    st0 = r.standard_normal((Bt, C, k - 1))
    z, st = ssd_oracle.conv1d_prefill(u, w, b, st0)
    for cut in (1, 2, 5, 10):   # including pieces shorter than the cache
        z1, s1 = ssd_oracle.conv1d_prefill(u[:, :cut], w, b, st0)
        z2, s2 = ssd_oracle.conv1d_prefill(u[:, cut:], w, b, s1)
        np.testing.assert_allclose(np.concatenate([z1, z2], axis=1), z, rtol=1e-13, atol=1e-13)
        np.testing.assert_array_equal(s2, st)
    s = st0
    for t in range(T):
        zt, s = ssd_oracle.conv1d_step(s, u[:, t], w, b)
        np.testing.assert_allclose(zt, z[:, t], rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(s, st)
    # the cache is the k-1 inputs before the prompt: a prompt preceded by them, from a zero cache
    zz, _ = ssd_oracle.conv1d_prefill(np.concatenate([st0.transpose(0, 2, 1), u], axis=1), w, b, None)
    np.testing.assert_allclose(zz[:, k - 1:], z, rtol=1e-13, atol=1e-13)


def test_dt_transform_values():
    import torch
    z = np.array([[-30.0, -1.0, 0.0, 1.0, 30.0, 800.0]])
    out = ssd_oracle.dt_transform(z, softplus=True)
    assert out[0, 2] == np.log(2.0) and out[0, 5] == 800.0
    np.testing.assert_allclose(out[0, 0], np.exp(-30.0), rtol=1e-12)       # log1p(e^v) ~ e^v far below zero
    np.testing.assert_allclose(out, torch.nn.functional.softplus(torch.from_numpy(z)).numpy(), rtol=1e-12)
    b = np.array([0.5, -0.5, 0.0, 1.0, 2.0, 3.0])
    np.testing.assert_array_equal(ssd_oracle.dt_transform(z, bias=b), z + b)
    np.testing.assert_array_equal(ssd_oracle.dt_transform(z, limit=(-1.0, 2.0)), np.clip(z, -1.0, 2.0))
    full = ssd_oracle.dt_transform(z, bias=b, softplus=True, limit=(1e-3, 1e-1))
    assert full.min() >= 1e-3 and full.max() <= 1e-1


def test_bf16_decay_would_be_visible():
    """The paper's decay-precision ablation: rounding exp(dt*A) to bf16 shows up far above the
    fp32 tolerance (1e-4), so a parity test at that tolerance can tell the two apart."""
    import torch
    p = pins.random_problem(30, Bt=1, T=256, H=2, P=4, N=8, G=1)
    p["dt"] = np.random.default_rng(1).uniform(1e-3, 1e-1, p["dt"].shape)
    y, _ = oracle_prefill(**p)
    # emulate the ablation through the inputs: pick dt so that exp(dt*A) is a bf16 number
    dA = np.exp(p["dt"] * p["A"][None, None, :])
    dA16 = torch.from_numpy(dA).to(torch.bfloat16).double().numpy()
    q = dict(p)
    # keep the input term dt*x*B unchanged by rescaling x
    q["dt"] = np.log(dA16) / p["A"][None, None, :]
    q["x"] = p["x"] * (p["dt"] / q["dt"])[..., None]
    y16, _ = oracle_prefill(**q)
    d = y16 - (y + (q["x"] - p["x"]) * p["D"][None, None, :, None])
    rel = np.abs(d).max() / np.abs(y).max()
    assert rel > 1e-3, rel
