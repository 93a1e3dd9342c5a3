"""GPU parity at the full benchmark sizes, in the launch configuration ``bench.py`` times.

Sequences are independent (one scalar A and one state per head) and the oracle scans a whole
benchmark configuration in seconds on the host cores, so the prefill configurations are compared
with it completely: every (batch row, head) sequence, every token, every channel, the final
state, under both gates of ``parity.assert_close``.  The decode configuration runs as the
benchmark words it -- a 2048-token prefill per layer, then 1024 single-token steps of all 64
layers -- and every step's output and the final state are compared: all layers at batch 1, and at
batch 16 all rows and heads of four layers (the oracle's cost for all 64 would be minutes).
A second run must be bitwise identical.
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


@pytest.mark.parametrize("name", ["c1_130m", "c2_780m_b8", "c3_2p7b_long"])
def test_full_size_prefill_every_sequence(ssd, name):
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
    y_ref, st_ref = ssd_oracle.prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"])
    print("oracle done", y_ref.shape, flush=True)
    e = assert_close(y, y_ref, 2e-2, "%s y, all %d sequences" % (name, cfg.batch * cfg.nheads))
    assert_close(st, st_ref, 2e-2, "%s final state, all sequences" % name)
    # per sequence as well: a sequence whose outputs are small must not hide behind the tensor-wide scale
    yg = to_np64(y)
    err = np.abs(yg - y_ref).max(axis=(1, 3))                       # (Bt, H)
    scale = np.abs(y_ref).max(axis=(1, 3))
    worst = float((err / scale).max())
    print("errors", e, "worst per-sequence normalised error %.3e" % worst, flush=True)
    assert worst <= 2e-2, "worst per-sequence normalised error %.3e" % worst


SWEEP_SHAPES = {
    # the head-shape / group / chunk-length variations of config 3 that the benchmark sweeps
    "chunk_64": dict(chunk=64),
    "chunk_1024": dict(chunk=1024),
    "ngroups_4": dict(ngroups=4),
    "ngroups_20": dict(ngroups=20),
    "headdim_128": dict(nheads=40, headdim=128),
    "dstate_64": dict(dstate=64),
    "dstate_256": dict(dstate=256),
}


@pytest.mark.parametrize("name", list(SWEEP_SHAPES))
def test_full_size_sweep_shapes_every_sequence(ssd, name):
    """The shapes of the benchmark's sweeps at their full size, every sequence against the oracle."""
    cfg = inputs.CONFIGS["c3_2p7b_long"].with_(name="c3_" + name, **SWEEP_SHAPES[name])
    print("full-size sweep shape", cfg, flush=True)
    inp = inputs.make_prefill_inputs(cfg, seed=1)
    dev = {k: v.cuda() for k, v in inp.items()}
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        cfg.torch_io_dtype)
    assert ssd.prefill_path(sh) == "mfma_bf16"
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"])
    e = assert_close(y, y_ref, 2e-2, "%s y" % name)
    assert_close(st, st_ref, 2e-2, "%s final state" % name)
    err = np.abs(to_np64(y) - y_ref).max(axis=(1, 3))
    worst = float((err / np.abs(y_ref).max(axis=(1, 3))).max())
    print("errors", e, "worst per-sequence normalised error %.3e" % worst, flush=True)
    assert worst <= 2e-2


def test_full_size_conv_prefill_every_element(ssd):
    """The convolution in front of the core at the long-prompt benchmark shape: 16384 tokens, the x | B | C
    channels of the 2.7B configuration (5120 + 128 + 128), k = 4, SiLU, with a cache going in and out.
    At this size a thread walks a long run of tokens, which the small cases never reach."""
    T, split, k = 16384, (5120, 128, 128), 4
    C = sum(split)
    g = torch.Generator().manual_seed(71)
    u = torch.randn((1, T, C), generator=g).bfloat16()
    w = torch.randn((C, k), generator=g) * 0.5
    b = torch.randn((C,), generator=g) * 0.1
    st = torch.randn((1, C, k - 1), generator=g).bfloat16()
    print("full-size conv", T, split, k, flush=True)
    outs, new_st = ssd.ssd_conv1d_prefill(u.cuda(), w.cuda(), b.cuda(), st.cuda(), split=split, activation="silu")
    torch.cuda.synchronize()
    z_ref, st_ref = ssd_oracle.conv1d_prefill(u, w, b, st, "silu")
    assert_close(torch.cat(outs, dim=2), z_ref, 2e-2, "conv z at 16384 x 5376")
    assert np.array_equal(to_np64(new_st), st_ref)


STEP_BLOCK = 128   # decode steps whose inputs are resident at a time


@pytest.mark.parametrize("name,nchecked", [("c4_decode_b1", 64), ("c4_decode_b16", 4)])
def test_full_size_decode_1024_steps(ssd, name, nchecked):
    """Config 4 as stated: states seeded by a 2048-token prefill per layer, then 1024 single-token steps,
    all 64 layers in one launch per step.  The oracle runs the token recurrence over prompt + generated
    steps for every (row, head) of the checked layers; y of every step and the final state are compared."""
    cfg = inputs.CONFIGS[name]
    Ly, nsteps = cfg.nlayers, cfg.decode_steps
    assert nsteps == 1024 and nsteps % STEP_BLOCK == 0
    print("full-size decode", cfg, "steps", nsteps, flush=True)
    dev = "cuda"
    rng = np.random.default_rng(43)
    layers = list(range(Ly)) if nchecked >= Ly else sorted(
        {0, Ly - 1} | {int(v) for v in rng.choice(np.arange(1, Ly - 1), nchecked - 2, replace=False)})
    state = torch.empty((Ly, cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
    A = torch.empty((Ly, cfg.nheads), dtype=torch.float32, device=dev)
    D = torch.empty_like(A)
    prompt = {}
    ytmp = None
    for l in range(Ly):
        inp = inputs.make_prefill_inputs(cfg, seed=0, layer=l, device=dev)
        if ytmp is None:
            ytmp = torch.empty_like(inp["x"])
        ssd.ssd_prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], cfg.chunk, y=ytmp,
                        final_state=state[l])
        A[l], D[l] = inp["A"], inp["D"]
        if l in layers:
            prompt[l] = {k: v.cpu() for k, v in inp.items()}
    del ytmp, inp
    torch.cuda.synchronize()
    print("prefilled", Ly, "layers", flush=True)
    # the steps, in blocks of STEP_BLOCK (the inputs of all 1024 steps of 64 layers at batch 16 are 22 GB)
    gen = {l: {k: [] for k in ("x", "dt", "B", "C")} for l in layers}    # CPU copies for the oracle
    got = {l: [] for l in layers}                                          # GPU outputs of the checked layers
    for blk in range(nsteps // STEP_BLOCK):
        per = [inputs.make_decode_inputs(cfg, STEP_BLOCK, seed=100 + blk, layer=l, device=dev) for l in range(Ly)]
        xs = torch.stack([s["x"] for s in per], dim=1)      # (steps, Ly, Bt, H, P)
        dts = torch.stack([s["dt"] for s in per], dim=1)
        Bs = torch.stack([s["B"] for s in per], dim=1)
        Cs = torch.stack([s["C"] for s in per], dim=1)
        del per
        ys = torch.empty_like(xs)
        for i in range(STEP_BLOCK):
            ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=ys[i])
        torch.cuda.synchronize()
        assert torch.isfinite(ys.float()).all()
        for l in layers:
            for k, t in (("x", xs), ("dt", dts), ("B", Bs), ("C", Cs)):
                gen[l][k].append(t[:, l].transpose(0, 1).cpu())            # (Bt, steps, ...)
            got[l].append(ys[:, l].transpose(0, 1).cpu())
        del xs, dts, Bs, Cs, ys
        print("steps", (blk + 1) * STEP_BLOCK, flush=True)
    assert torch.isfinite(state).all()
    worst = 0.0
    for l in layers:
        p = prompt[l]
        full = {k: torch.cat([p[k]] + gen[l][k], dim=1) for k in ("x", "dt", "B", "C")}
        y_ref, st_ref = ssd_oracle.prefill(full["x"], full["dt"], p["A"], full["B"], full["C"], p["D"])
        y_got = torch.cat(got[l], dim=1)                                   # (Bt, 1024, H, P)
        e = assert_close(y_got, y_ref[:, cfg.seqlen:], 2e-2, "%s layer %d decode y, 1024 steps" % (name, l))
        assert_close(state[l], st_ref, 2e-2, "%s layer %d state after 1024 steps" % (name, l))
        worst = max(worst, e["worst_allclose"])
        gen[l] = got[l] = prompt[l] = None
        if l % 8 == 0 or nchecked < Ly:
            print("layer", l, "ok", e, flush=True)
    print("checked layers", layers, "worst allclose ratio %.3e" % worst, flush=True)


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
