"""GPU parity at the full benchmark sizes, in the launch configuration ``bench.py`` times.

The oracle cannot evaluate every (batch row, head) sequence of these shapes in seconds, but
sequences are independent (one scalar A and one state per head), so it evaluates a seeded
sample of them completely -- every token, every channel, the final state -- and those are
compared element by element.  Properties that hold at any size cover the rest: every output
is finite, and a second run is bitwise identical.
"""
import numpy as np
import pytest
import torch

from oracle import ssd_oracle
from paper_2603_09555_amd import inputs
from parity import assert_close, to_np64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ssd():
    from paper_2603_09555_amd import ssd as binding
    return binding


def sample_pairs(cfg, n, seed):
    """n distinct (b, h) pairs: the first and the last sequence plus seeded random ones."""
    rng = np.random.default_rng(seed)
    total = cfg.batch * cfg.nheads
    picks = {0, total - 1}
    while len(picks) < min(n, total):
        picks.add(int(rng.integers(total)))
    return [(i // cfg.nheads, i % cfg.nheads) for i in sorted(picks)]


@pytest.mark.parametrize("name,npairs", [("c1_130m", 24), ("c2_780m_b8", 8), ("c3_2p7b_long", 6)])
def test_full_size_prefill_sampled_sequences(ssd, name, npairs):
    cfg = inputs.CONFIGS[name]
    print("full-size prefill", cfg, flush=True)
    inp = inputs.make_prefill_inputs(cfg, seed=0)
    dev = {k: v.cuda() for k, v in inp.items()}
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        cfg.torch_io_dtype)
    assert ssd.prefill_path(sh) == "mfma_bf16"
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    y2, st2 = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all() and torch.isfinite(st).all()
    assert torch.equal(y, y2) and torch.equal(st, st2)
    pairs = sample_pairs(cfg, npairs, seed=41)
    y_ref, st_ref = ssd_oracle.prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], pairs=pairs)
    bs = torch.tensor([b for b, _ in pairs], device="cuda")
    hs = torch.tensor([h for _, h in pairs], device="cuda")
    y_got = y[bs, :, hs, :]      # (n, T, P)
    st_got = st[bs, hs]          # (n, P, N)
    e = assert_close(y_got, y_ref, 2e-2, "%s y on sampled sequences" % name)
    assert_close(st_got, st_ref, 2e-2, "%s final state on sampled sequences" % name)
    print("errors", e, flush=True)


@pytest.mark.parametrize("name", ["c4_decode_b1", "c4_decode_b16"])
def test_full_size_stacked_decode_sampled_sequences(ssd, name):
    """All 64 layers in one launch per step, states seeded by a 2048-token prefill per layer; the
    oracle runs the token recurrence over prompt + generated steps for sampled (layer, row, head)."""
    cfg = inputs.CONFIGS[name]
    Ly, nsteps = cfg.nlayers, 24
    print("full-size decode", cfg, "steps", nsteps, flush=True)
    dev = "cuda"
    rng = np.random.default_rng(43)
    layers = sorted({0, Ly - 1, int(rng.integers(Ly))})
    state = torch.empty((Ly, cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
    A = torch.empty((Ly, cfg.nheads), dtype=torch.float32, device=dev)
    D = torch.empty_like(A)
    kept = {}
    ytmp = None
    for l in range(Ly):
        inp = inputs.make_prefill_inputs(cfg, seed=0, layer=l, device=dev)
        if ytmp is None:
            ytmp = torch.empty_like(inp["x"])
        ssd.ssd_prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], cfg.chunk, y=ytmp,
                        final_state=state[l])
        A[l], D[l] = inp["A"], inp["D"]
        if l in layers:
            kept[l] = {k: v.cpu() for k, v in inp.items()}
    del ytmp, inp
    steps = [inputs.make_decode_inputs(cfg, nsteps, seed=0, layer=l, device=dev) for l in range(Ly)]
    xs = torch.stack([s["x"] for s in steps], dim=1)      # (steps, Ly, Bt, H, P)
    dts = torch.stack([s["dt"] for s in steps], dim=1)
    Bs = torch.stack([s["B"] for s in steps], dim=1)
    Cs = torch.stack([s["C"] for s in steps], dim=1)
    del steps
    ys = torch.empty((nsteps, Ly, cfg.batch, cfg.nheads, cfg.headdim), dtype=xs.dtype, device=dev)
    for i in range(nsteps):
        ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=ys[i])
    torch.cuda.synchronize()
    assert torch.isfinite(ys.float()).all() and torch.isfinite(state).all()
    for l in layers:
        pairs = sample_pairs(cfg, 4, seed=47 + l)
        p = kept[l]
        full = {"x": torch.cat([p["x"], xs[:, l].transpose(0, 1).cpu()], dim=1),
                "dt": torch.cat([p["dt"], dts[:, l].transpose(0, 1).cpu()], dim=1),
                "B": torch.cat([p["B"], Bs[:, l].transpose(0, 1).cpu()], dim=1),
                "C": torch.cat([p["C"], Cs[:, l].transpose(0, 1).cpu()], dim=1)}
        y_ref, st_ref = ssd_oracle.prefill(full["x"], full["dt"], p["A"], full["B"], full["C"], p["D"], pairs=pairs)
        bs = torch.tensor([b for b, _ in pairs], device=dev)
        hs = torch.tensor([h for _, h in pairs], device=dev)
        y_got = ys[:, l][:, bs, hs, :].transpose(0, 1)    # (n, steps, P)
        assert_close(y_got, y_ref[:, cfg.seqlen:], 2e-2, "%s layer %d decode y" % (name, l))
        assert_close(state[l][bs, hs], st_ref, 2e-2, "%s layer %d state after %d steps" % (name, l, nsteps))


def test_full_size_multi_step_decode_equals_single_steps(ssd):
    """Config 4 at batch 16, all 64 layers: 8 steps in one launch against 8 stacked launches,
    from a random state (y up to summation order, the state bitwise)."""
    cfg = inputs.CONFIGS["c4_decode_b16"]
    Ly, S = cfg.nlayers, 8
    print("full-size multi-step decode", cfg, "steps", S, flush=True)
    g = torch.Generator(device="cuda")
    g.manual_seed(53)
    state = torch.randn((Ly, cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), generator=g, device="cuda")
    x = torch.randn((S, Ly, cfg.batch, cfg.nheads, cfg.headdim), generator=g, device="cuda").bfloat16()
    dt = torch.rand((S, Ly, cfg.batch, cfg.nheads), generator=g, device="cuda") * 0.1 + 1e-3
    A = -(torch.rand((Ly, cfg.nheads), generator=g, device="cuda") * 15 + 1)
    D = torch.randn((Ly, cfg.nheads), generator=g, device="cuda")
    B = (0.25 * torch.randn((S, Ly, cfg.batch, cfg.ngroups, cfg.dstate), generator=g, device="cuda")).bfloat16()
    C = (0.25 * torch.randn((S, Ly, cfg.batch, cfg.ngroups, cfg.dstate), generator=g, device="cuda")).bfloat16()
    s1 = state.clone()
    y = ssd.ssd_decode_steps_layers(state, x, dt, A, B, C, D)
    y1 = torch.stack([ssd.ssd_decode_step_layers(s1, x[i], dt[i], A, B[i], C[i], D) for i in range(S)])
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    assert_close(y, to_np64(y1), 2e-2, "multi-step y vs single steps")
    assert torch.equal(state, s1)  # the state update involves no sum: identical bits


def test_full_size_ragged_batch_sampled_sequences(ssd):
    """Config 3's token count and heads as a packed batch of 16 ragged sequences (lengths
    log-uniform over a 64x range), library-chosen segments: sampled (sequence, head) pairs
    against the oracle, every token of them."""
    cfg = inputs.CONFIGS["c3_2p7b_long"]
    T, H = cfg.seqlen, cfg.nheads
    r = np.random.default_rng(7)
    w = np.exp(r.uniform(0.0, np.log(64.0), 16))
    lens = np.maximum(1, np.floor(w / w.sum() * T).astype(np.int64))
    lens[np.argmax(lens)] += T - lens.sum()
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    print("full-size ragged batch", lens.tolist(), flush=True)
    inp = inputs.make_prefill_inputs(cfg, seed=0)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    dev = {k: v.cuda() for k, v in pk.items()}
    h0 = 0.5 * torch.randn((16, H, cfg.headdim, cfg.dstate), generator=torch.Generator().manual_seed(3))
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), cfg.chunk, h0=h0.cuda())
    y2, st2 = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                     torch.from_numpy(cu).cuda(), cfg.chunk, h0=h0.cuda())
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all() and torch.isfinite(st).all()
    assert torch.equal(y, y2) and torch.equal(st, st2)
    picks = sorted({(0, 0), (15, H - 1), (int(np.argmax(lens)), 17), (int(np.argmin(lens)), 40)} |
                   {(int(r.integers(16)), int(r.integers(H))) for _ in range(6)})
    for q, h in picks:
        a, b = int(cu[q]), int(cu[q + 1])
        y_ref, st_ref = ssd_oracle.prefill(pk["x"][None, a:b], pk["dt"][None, a:b], pk["A"], pk["B"][None, a:b],
                                           pk["C"][None, a:b], pk["D"], h0=h0[q:q + 1], pairs=[(0, h)])
        assert_close(y[a:b, h], y_ref[0], 2e-2, "ragged y seq %d head %d" % (q, h))
        assert_close(st[q, h], st_ref[0], 2e-2, "ragged state seq %d head %d" % (q, h))


def test_longest_addressable_sequence(ssd):
    """One sequence close to the largest the MFMA kernels address with 32-bit byte offsets (x of one
    batch row just under 4 GiB): 4,000,000 tokens x 8 heads.  With A = -16 and dt >= 0.05 the state
    forgets within a few hundred tokens (decay <= e^-0.8 per token), so the oracle can check windows
    anywhere in the sequence from a zero state after a 512-token run-in: the first tokens, the
    tokens around the 2 GiB and 3 GiB byte offsets of x, and the ragged end with the final state."""
    T, H, P, N, L = 4_000_000, 8, 64, 128, 256
    sh = ssd.make_shape(1, T, H, P, N, 1, L, torch.bfloat16)
    assert ssd.prefill_path(sh) == "mfma_bf16"
    print("longest sequence", T, "tokens;", T * H * P * 2 / 2 ** 30, "GiB of x", flush=True)
    g = torch.Generator(device="cuda")
    g.manual_seed(97)
    x = torch.empty((1, T, H, P), dtype=torch.bfloat16, device="cuda")
    B = torch.empty((1, T, 1, N), dtype=torch.bfloat16, device="cuda")
    C = torch.empty_like(B)
    step = 1 << 18
    for t0 in range(0, T, step):   # drawn in pieces to bound the fp32 temporaries
        n = min(step, T - t0)
        x[0, t0:t0 + n] = torch.randn((n, H, P), generator=g, device="cuda").bfloat16()
        B[0, t0:t0 + n] = (0.25 * torch.randn((n, 1, N), generator=g, device="cuda")).bfloat16()
        C[0, t0:t0 + n] = (0.25 * torch.randn((n, 1, N), generator=g, device="cuda")).bfloat16()
    dt = torch.rand((1, T, H), generator=g, device="cuda") * 0.05 + 0.05
    A = torch.full((H,), -16.0, device="cuda")
    D = torch.randn((H,), generator=g, device="cuda")
    y, st = ssd.ssd_prefill(x, dt, A, B, C, D, L)
    torch.cuda.synchronize()
    assert torch.isfinite(st).all()
    run_in, width = 512, 1024
    row_bytes = H * P * 2
    starts = [0, (2 << 30) // row_bytes - width // 2, (3 << 30) // row_bytes - width // 2, T - width]
    for s0 in starts:
        a = max(0, s0 - run_in)
        b = min(T, s0 + width)
        sl = slice(a, b)
        y_ref, st_ref = ssd_oracle.prefill(x[:, sl].cpu(), dt[:, sl].cpu(), A.cpu(), B[:, sl].cpu(), C[:, sl].cpu(),
                                           D.cpu(), pairs=[(0, 0), (0, 3), (0, H - 1)])
        got = y[0, s0:b][:, [0, 3, H - 1]].transpose(0, 1)        # (3, width, P)
        assert torch.isfinite(got.float()).all()
        assert_close(got, y_ref[:, s0 - a:], 2e-2, "y in the window at token %d" % s0)
        if b == T:
            assert_close(st[0, [0, 3, H - 1]], st_ref, 2e-2, "final state")
