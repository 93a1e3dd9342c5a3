"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on the same seeded inputs.  Sizes here are ones the oracle finishes in seconds; they span
several tiles and ragged tails.  Full-size configurations are in test_gpu_full_size.py."""
import numpy as np
import pytest
import torch

from oracle import ssd_oracle
from paper_2603_09555_amd import inputs
import blocked_model
from parity import TOL, assert_close, errors, to_np64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ssd():
    from paper_2603_09555_amd import ssd as binding
    return binding


@pytest.fixture(autouse=True)
def _library_choices_restored(ssd):
    """Tests force segment lengths, kernel families and cache policies through the test-only knobs of the
    library; every test starts from, and leaves behind, the library's own choices."""
    ssd.reset_knobs()
    yield
    ssd.reset_knobs()


def cfg_of(Bt, T, H, P, N, G, L, io):
    return inputs.SSDConfig("t", Bt, T, H, P, N, G, L, io)


def run_prefill(ssd, cfg, seed=0, h0=None, chunk=None):
    inp = inputs.make_prefill_inputs(cfg, seed=seed)
    dev = {k: v.cuda() for k, v in inp.items()}
    h0d = None if h0 is None else h0.cuda()
    print("prefill case", cfg, "seed", seed, "h0" if h0 is not None else "", flush=True)
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                            chunk if chunk is not None else cfg.chunk, h0=h0d)
    torch.cuda.synchronize()
    return inp, y, st


def oracle_prefill(inp, h0=None, pairs=None):
    return ssd_oracle.prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], h0=h0, pairs=pairs)


PREFILL_CASES = [
    # Bt, T, H, P, N, G, L
    (1, 512, 4, 32, 16, 1, 64),     # configs[0]
    (2, 100, 4, 32, 16, 2, 32),     # ragged tail (100 = 3*32 + 4)
    (1, 1, 2, 8, 4, 1, 16),         # single token
    (1, 65, 2, 16, 8, 1, 64),       # one full chunk + one token
    (2, 37, 6, 24, 20, 3, 7),       # nothing is a multiple of any tile
    (1, 48, 2, 64, 128, 1, 256),    # chunk longer than the sequence
    (1, 300, 3, 72, 40, 1, 128),    # P and N beyond one 64-wide tile
    (3, 129, 8, 64, 128, 2, 64),    # Mamba-2 head shape, small T
]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("case", PREFILL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_prefill_matches_oracle(ssd, case, io):
    cfg = cfg_of(*case, io)
    inp, y, st = run_prefill(ssd, cfg, seed=1)
    y_ref, st_ref = oracle_prefill(inp)
    assert y.dtype == cfg.torch_io_dtype and st.dtype == torch.float32
    assert_close(y, y_ref, TOL[io], "y")
    assert_close(st, st_ref, TOL[io], "final state")


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_prefill_with_initial_state_and_aliasing(ssd, io):
    cfg = cfg_of(2, 90, 4, 32, 16, 2, 32, io)
    h0 = inputs.make_state(cfg, seed=3)
    inp, y, st = run_prefill(ssd, cfg, seed=2, h0=h0)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    assert_close(y, y_ref, TOL[io], "y with h0")
    assert_close(st, st_ref, TOL[io], "state with h0")
    # h0 may alias final_state
    dev = {k: v.cuda() for k, v in inp.items()}
    buf = h0.cuda().clone()
    y2, st2 = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk, h0=buf,
                              final_state=buf)
    torch.cuda.synchronize()
    assert st2.data_ptr() == buf.data_ptr()
    assert torch.equal(y2, y) and torch.equal(st2, st)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_chunk_size_independence(ssd, io):
    base = cfg_of(1, 200, 4, 32, 16, 1, 64, io)
    inp = inputs.make_prefill_inputs(base, seed=5)
    y_ref, st_ref = oracle_prefill(inp)
    for L in (1, 3, 16, 64, 100, 200, 256, 1000):
        _, y, st = run_prefill(ssd, base, seed=5, chunk=L)
        assert_close(y, y_ref, TOL[io], "y chunk %d" % L)
        assert_close(st, st_ref, TOL[io], "state chunk %d" % L)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_prefill_then_decode_equals_longer_prefill(ssd, io):
    cfg = cfg_of(2, 97, 4, 32, 16, 2, 32, io)
    inp = inputs.make_prefill_inputs(cfg, seed=7)
    dev = {k: v.cuda() for k, v in inp.items()}
    y_all, st_all = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    cut = {k: (v[:, :-1].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in dev.items()}
    y_pre, st_pre = ssd.ssd_prefill(cut["x"], cut["dt"], cut["A"], cut["B"], cut["C"], cut["D"], cfg.chunk)
    y_last = ssd.ssd_decode_step(st_pre, dev["x"][:, -1].contiguous(), dev["dt"][:, -1].contiguous(), dev["A"],
                                 dev["B"][:, -1].contiguous(), dev["C"][:, -1].contiguous(), dev["D"])
    torch.cuda.synchronize()
    y_ref, st_ref = oracle_prefill(inp)
    assert_close(y_pre, y_ref[:, :-1], TOL[io], "prefix y")
    assert_close(y_last, y_ref[:, -1], TOL[io], "decode y")
    assert_close(st_pre, st_ref, TOL[io], "state after prefill+decode")
    assert_close(st_pre, to_np64(st_all), TOL[io], "GPU prefill(T+1) vs GPU prefill(T)+decode")


def test_split_prompt_with_carried_state(ssd):
    cfg = cfg_of(1, 150, 4, 32, 16, 1, 64, "f32")
    inp = inputs.make_prefill_inputs(cfg, seed=9)
    dev = {k: v.cuda() for k, v in inp.items()}
    y_ref, st_ref = oracle_prefill(inp)
    for cut in (1, 64, 77):
        a = {k: (v[:, :cut].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in dev.items()}
        b = {k: (v[:, cut:].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in dev.items()}
        y1, s1 = ssd.ssd_prefill(a["x"], a["dt"], a["A"], a["B"], a["C"], a["D"], cfg.chunk)
        y2, s2 = ssd.ssd_prefill(b["x"], b["dt"], b["A"], b["B"], b["C"], b["D"], cfg.chunk, h0=s1)
        torch.cuda.synchronize()
        assert_close(torch.cat([y1, y2], dim=1), y_ref, 1e-4, "split y at %d" % cut)
        assert_close(s2, st_ref, 1e-4, "split state at %d" % cut)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_bitwise_determinism_and_batch_invariance(ssd, io):
    cfg = cfg_of(3, 130, 4, 32, 16, 2, 32, io)
    inp, y1, s1 = run_prefill(ssd, cfg, seed=11)
    _, y2, s2 = run_prefill(ssd, cfg, seed=11)
    assert torch.equal(y1, y2) and torch.equal(s1, s2)
    dev = {k: v.cuda() for k, v in inp.items()}
    row = {k: (v[1:2].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in dev.items()}
    yr, sr = ssd.ssd_prefill(row["x"], row["dt"], row["A"], row["B"], row["C"], row["D"], cfg.chunk)
    torch.cuda.synchronize()
    assert torch.equal(yr, y1[1:2]) and torch.equal(sr, s1[1:2])


def test_extreme_decay_stays_finite(ssd):
    """Largest step size times the most negative A over a whole chunk: exponents reach -400,
    masked entries must be exact zeros and nothing may overflow."""
    cfg = cfg_of(1, 512, 2, 32, 16, 1, 256, "f32")
    inp = inputs.make_prefill_inputs(cfg, seed=13)
    inp["dt"] = torch.full_like(inp["dt"], 0.1)
    inp["A"] = torch.tensor([-16.0, -1e-3])
    dev = {k: v.cuda() for k, v in inp.items()}
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    torch.cuda.synchronize()
    y_ref, st_ref = oracle_prefill(inp)
    assert_close(y, y_ref, 1e-4, "extreme decay y")
    assert_close(st, st_ref, 1e-4, "extreme decay state")


# ---- decode ---------------------------------------------------------------------------------
DECODE_CASES = [
    # Ly, Bt, H, P, N, G
    (1, 1, 4, 32, 16, 1),
    (1, 3, 6, 24, 20, 3),     # N not a multiple of 4
    (1, 2, 4, 16, 24, 2),     # N/4 = 6, not a power of two
    (2, 2, 8, 64, 128, 1),    # Mamba-2 head shape
    (3, 1, 5, 7, 4, 5),
    (2, 1, 2, 40, 256, 1),
    (1, 2, 3, 100, 64, 1),    # P beyond one unrolled pass
]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("case", DECODE_CASES, ids=lambda c: "x".join(map(str, c)))
def test_decode_matches_oracle(ssd, case, io):
    Ly, Bt, H, P, N, G = case
    iod = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator().manual_seed(17)
    state = torch.randn((Ly, Bt, H, P, N), generator=g)
    x = torch.randn((Ly, Bt, H, P), generator=g).to(iod)
    dt = torch.rand((Ly, Bt, H), generator=g) * 0.1 + 1e-3
    A = -(torch.rand((Ly, H), generator=g) * 15 + 1)
    D = torch.randn((Ly, H), generator=g)
    B = (0.25 * torch.randn((Ly, Bt, G, N), generator=g)).to(iod)
    C = (0.25 * torch.randn((Ly, Bt, G, N), generator=g)).to(iod)
    print("decode case", case, io, flush=True)
    sd = state.cuda().clone()
    y = ssd.ssd_decode_step_layers(sd, x.cuda(), dt.cuda(), A.cuda(), B.cuda(), C.cuda(), D.cuda())
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.decode_step_layers(state, x, dt, A, B, C, D)
    assert_close(y, y_ref, TOL[io], "decode y")
    assert_close(sd, st_ref, 1e-5, "decode state")  # the state is fp32 whatever the io dtype
    if Ly == 1:
        sd1 = state[0].cuda().clone()
        y1 = ssd.ssd_decode_step(sd1, x[0].cuda(), dt[0].cuda(), A[0].cuda(), B[0].cuda(), C[0].cuda(),
                                 D[0].cuda())
        torch.cuda.synchronize()
        assert torch.equal(y1, y[0]) and torch.equal(sd1, sd[0])


def test_many_decode_steps_track_the_oracle(ssd):
    """64 consecutive steps from a prefilled state (the generation loop of Alg. 2, SSM part)."""
    cfg = cfg_of(2, 64, 8, 64, 128, 1, 64, "bf16")
    inp = inputs.make_prefill_inputs(cfg, seed=19)
    steps = inputs.make_decode_inputs(cfg, 64, seed=19)
    dev = {k: v.cuda() for k, v in inp.items()}
    _, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    sdev = {k: v.cuda() for k, v in steps.items()}
    ys = [ssd.ssd_decode_step(st, sdev["x"][i], sdev["dt"][i], dev["A"], sdev["B"][i], sdev["C"][i], dev["D"])
          for i in range(64)]
    torch.cuda.synchronize()
    full = {"x": torch.cat([inp["x"], steps["x"].transpose(0, 1)], dim=1),
            "dt": torch.cat([inp["dt"], steps["dt"].transpose(0, 1)], dim=1),
            "B": torch.cat([inp["B"], steps["B"].transpose(0, 1)], dim=1),
            "C": torch.cat([inp["C"], steps["C"].transpose(0, 1)], dim=1), "A": inp["A"], "D": inp["D"]}
    y_ref, st_ref = oracle_prefill(full)
    assert_close(torch.stack(ys, dim=1), y_ref[:, 64:], 2e-2, "decode y over 64 steps")
    assert_close(st, st_ref, 2e-2, "state after 64 steps")


STEPS_CASES = [
    # steps, Ly, Bt, H, P, N, G
    (5, 2, 2, 8, 64, 128, 1),    # Mamba-2 head shape: state stays in registers
    (1, 1, 1, 4, 64, 128, 2),    # a single step
    (7, 1, 2, 4, 128, 128, 1),
    (4, 2, 1, 4, 64, 64, 2),
    (3, 1, 2, 4, 64, 16, 1),
    (6, 1, 2, 4, 64, 256, 1),
    (4, 2, 2, 6, 24, 20, 3),     # no register-resident variant: one launch per step
    (3, 1, 1, 3, 100, 64, 1),
]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("case", STEPS_CASES, ids=lambda c: "x".join(map(str, c)))
def test_multi_step_decode_matches_oracle_and_single_steps(ssd, case, io):
    S, Ly, Bt, H, P, N, G = case
    iod = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator().manual_seed(23)
    state = torch.randn((Ly, Bt, H, P, N), generator=g)
    x = torch.randn((S, Ly, Bt, H, P), generator=g).to(iod)
    dt = torch.rand((S, Ly, Bt, H), generator=g) * 0.1 + 1e-3
    A = -(torch.rand((Ly, H), generator=g) * 15 + 1)
    D = torch.randn((Ly, H), generator=g)
    B = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).to(iod)
    C = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).to(iod)
    print("multi-step decode case", case, io, flush=True)
    dev = [t.cuda() for t in (x, dt, A, B, C, D)]
    sd = state.cuda().clone()
    y = ssd.ssd_decode_steps_layers(sd, dev[0], dev[1], dev[2], dev[3], dev[4], dev[5])
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.decode_steps_layers(state, x, dt, A, B, C, D)
    assert_close(y, y_ref, TOL[io], "multi-step y")
    assert_close(sd, st_ref, 1e-5, "multi-step state")
    # the same steps one launch at a time: the same values up to the order of the sum over dstate
    s1 = state.cuda().clone()
    # (slices are copied: the single-step entry point wants 16-byte aligned pointers)
    y1 = torch.stack([ssd.ssd_decode_step_layers(s1, dev[0][i].clone(), dev[1][i].clone(), dev[2], dev[3][i].clone(),
                                                 dev[4][i].clone(), dev[5]) for i in range(S)])
    torch.cuda.synchronize()
    assert_close(y, to_np64(y1), TOL[io], "multi-step y vs single steps")
    assert torch.equal(s1, sd)  # the state update involves no sum: identical bits


def test_decode_steps_replayed_from_a_hip_graph(ssd):
    """Stacked decode launches captured into a HIP graph: every replay (with eager work and
    synchronisations in between) continues the recurrence exactly as eager launches do."""
    S, Ly, Bt, H, P, N, G = 4, 3, 2, 8, 64, 128, 1
    g = torch.Generator().manual_seed(29)
    state = torch.randn((Ly, Bt, H, P, N), generator=g).cuda()
    x = torch.randn((S, Ly, Bt, H, P), generator=g).bfloat16().cuda()
    dt = (torch.rand((S, Ly, Bt, H), generator=g) * 0.1 + 1e-3).cuda()
    A = (-(torch.rand((Ly, H), generator=g) * 15 + 1)).cuda()
    D = torch.randn((Ly, H), generator=g).cuda()
    B = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).bfloat16().cuda()
    C = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).bfloat16().cuda()
    sg, se = state.clone(), state.clone()
    yg = torch.empty_like(x)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    keep = sg.clone()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for i in range(S):
                ssd.ssd_decode_step_layers(sg, x[i], dt[i], A, B[i], C[i], D, y=yg[i])
    torch.cuda.current_stream().wait_stream(side)
    sg.copy_(keep)  # capture does not execute, but make the start state explicit
    for rep in range(3):
        graph.replay()
        torch.cuda.synchronize()
        ye = torch.stack([ssd.ssd_decode_step_layers(se, x[i], dt[i], A, B[i], C[i], D) for i in range(S)])
        torch.cuda.synchronize()
        assert torch.equal(yg, ye) and torch.equal(sg, se), "replay %d differs from eager" % rep


# ---- MFMA path (headdim 64, dstate 128, bf16) --------------------------------------------------
MFMA_CASES = [
    # Bt, T, H, P, N, G, L, forced chunks per segment (0 = library's choice)
    (1, 64, 4, 64, 128, 1, 64, 0),       # exactly one block
    (1, 1, 4, 64, 128, 1, 64, 0),        # single token
    (2, 300, 4, 64, 128, 1, 256, 0),     # ragged tail inside the second chunk
    (1, 1000, 4, 64, 128, 1, 128, 1),    # one chunk per segment: 8 segments, ragged last block
    (1, 1000, 12, 64, 128, 1, 128, 3),   # 3 chunks per segment
    (2, 513, 8, 64, 128, 2, 64, 2),      # two groups, T = 8 blocks + 1 token
    (1, 2048, 24, 64, 128, 1, 256, 0),   # configs[1]
    (1, 777, 4, 64, 128, 1, 1024, 0),    # chunk longer than the sequence
    (2, 300, 4, 128, 128, 2, 64, 1),     # headdim 128: two 64-column slices per head, two heads per group
    (1, 500, 4, 192, 128, 1, 128, 2),    # headdim 192
    (1, 700, 2, 256, 128, 2, 64, 0),     # headdim 256, one head per group
    (2, 300, 4, 64, 64, 1, 64, 1),       # dstate 64: one zero-padded state slice
    (1, 1000, 8, 64, 256, 2, 128, 2),    # dstate 256: two state slices, outputs added
    (1, 500, 4, 64, 32, 1, 256, 0),      # dstate 32
    (2, 300, 4, 128, 192, 1, 64, 1),     # dstate 192 (one and a half slices), headdim 128
    (1, 1000, 1, 64, 128, 1, 128, 2),    # a single head: three slots of its workgroup idle
    (2, 513, 6, 64, 128, 2, 64, 2),      # three heads per group
    (1, 700, 24, 64, 128, 8, 100, 0),    # 24 heads in 8 groups; a chunk length that is no multiple of 64
    (2, 300, 5, 128, 128, 1, 37, 1),     # ten 64-column slices in one group: 2 idle slots; chunk 37
    (1, 500, 7, 64, 64, 7, 200, 0),      # one head per group, dstate 64
    (1, 600, 3, 64, 256, 1, 256, 2),     # three heads, two state slices
]


@pytest.mark.parametrize("case", MFMA_CASES, ids=lambda c: "x".join(map(str, c)))
def test_mfma_prefill_matches_oracle(ssd, case):
    *dims, seg = case
    cfg = cfg_of(*dims, "bf16")
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        torch.bfloat16)
    assert ssd.prefill_path(sh) == "mfma_bf16"
    if seg:
        ssd.set_knob("seg_chunks", seg)
    else:
        ssd.set_knob("seg_chunks", 0)
    # T = 300: an initial state of realistic size (what a prefill of similar inputs leaves behind);
    # T = 1000: a large N(0,1) one, far bigger than anything the inputs build up, whose early outputs are
    # sums of large cancelling terms.  Both gates apply to every case.  For the large initial state the
    # limit of the allclose gate is what the documented bf16 rounding of the state operand of the
    # state -> output product costs on these very inputs, computed on the CPU by blocked_model.py (it is
    # 2.05e-2 from that rounding alone, see test_blocked_model.py), plus 5 %; and the componentwise bound
    # is gated in addition.
    h0, mag_y, mag_st, lim = None, None, None, None
    if cfg.seqlen == 300:
        warm = inputs.make_prefill_inputs(cfg, seed=77)
        h0 = torch.from_numpy(oracle_prefill(warm)[1]).float()
    if cfg.seqlen == 1000:
        h0 = inputs.make_state(cfg, seed=4)
    inp, y, st = run_prefill(ssd, cfg, seed=23, h0=h0)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    if cfg.seqlen == 1000:
        ab = {k: (v.abs() if k in ("x", "B", "C", "D") else v) for k, v in inp.items()}
        mag_y, mag_st = oracle_prefill(ab, h0=h0.abs())
        model_y, _ = blocked_model.prefill(inp, h0)
        lim = max(2e-2, 1.05 * errors(model_y, y_ref)["worst_allclose"])
        print("allclose limit from the CPU model of the bf16 roundings: %.4e" % lim, flush=True)
    e = assert_close(y, y_ref, 2e-2, "mfma y", mag=mag_y, allclose_tol=lim)
    assert_close(st, st_ref, 2e-2, "mfma final state", mag=mag_st)
    print("errors", e, flush=True)


@pytest.mark.parametrize("case", [(1, 1000, 4, 64, 128, 1, 128, 1), (1, 1000, 12, 64, 128, 1, 128, 3),
                                  (2, 1500, 8, 64, 128, 2, 64, 4)], ids=lambda c: "x".join(map(str, c)))
def test_mfma_prefill_continues_a_cached_prompt(ssd, case):
    """Several segments from the state a prefill of similar inputs leaves behind (section "The O(1) state
    cache": later calls continue from the cache), under the plain gates."""
    *dims, seg = case
    cfg = cfg_of(*dims, "bf16")
    ssd.set_knob("seg_chunks", seg)
    warm = inputs.make_prefill_inputs(cfg, seed=78)
    h0 = torch.from_numpy(oracle_prefill(warm)[1]).float()
    inp, y, st = run_prefill(ssd, cfg, seed=24, h0=h0)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    e = assert_close(y, y_ref, 2e-2, "continued y")
    assert_close(st, st_ref, 2e-2, "continued final state")
    print("errors", e, flush=True)


@pytest.mark.parametrize("with_h0", [False, True], ids=["zero", "h0"])
@pytest.mark.parametrize("parts", [1, 2, 4])
@pytest.mark.parametrize("case", [(2, 1024, 8, 64, 128, 1, 256, 8), (1, 1000, 4, 128, 256, 2, 128, 10),
                                  (3, 777, 12, 64, 64, 3, 64, 8), (2, 1300, 8, 64, 128, 1, 64, 4)],
                         ids=lambda c: "x".join(map(str, c)))
def test_mfma_prefill_segment_states_folded(ssd, case, parts, with_h0):
    """A prompt cut into few segments runs no pass over segment states: every later segment's workgroups sum
    the local end states of the pieces before them (and the decayed h0) as they load them.  Checked against
    the oracle with two segments (one, two and four pieces; a ragged last block; two state slices at dstate
    256; a carried state) and, with the limit raised, six segments of up to four pieces (a chain of 20
    slots); against the separate pass on the same inputs; and with h0 and final_state in the same memory,
    where the library must fall back to the separate pass."""
    *dims, seg_blocks = case
    cfg = cfg_of(*dims, "bf16")
    ssd.set_knob("seg_blocks", seg_blocks)
    ssd.set_knob("seg_parts", parts)
    ssd.set_knob("fold_max_slots", 64)
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        torch.bfloat16)
    plan = ssd.prefill_plan(sh)
    assert plan["fold"] and plan["seg_blocks"] == seg_blocks and plan["segments"] >= 2, plan
    assert not ssd.prefill_plan(sh, h0_aliases_final_state=True)["fold"]
    h0 = None
    if with_h0:  # an initial state of realistic size: what a prefill of similar inputs leaves behind
        h0 = torch.from_numpy(oracle_prefill(inputs.make_prefill_inputs(cfg, seed=79))[1]).float()
    inp, y, st = run_prefill(ssd, cfg, seed=52, h0=h0)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    e = assert_close(y, y_ref, 2e-2, "folded y")
    assert_close(st, st_ref, 2e-2, "folded final state")
    print("errors", e, flush=True)
    ssd.set_knob("fold_max_slots", 0)
    assert not ssd.prefill_plan(sh)["fold"]
    _, y2, st2 = run_prefill(ssd, cfg, seed=52, h0=h0)
    assert_close(y2, y_ref, 2e-2, "separate pass y")
    assert_close(st2, st_ref, 2e-2, "separate pass final state")
    ssd.set_knob("fold_max_slots", 64)
    if with_h0:
        dev = {k: v.cuda() for k, v in inp.items()}
        shared = h0.cuda().clone()
        y3, st3 = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk, h0=shared,
                                  final_state=shared)
        torch.cuda.synchronize()
        assert st3.data_ptr() == shared.data_ptr()
        assert torch.equal(y3, y2) and torch.equal(st3, st2)   # the separate pass ran: the same bits


# ---- fp32 io on fp32 MFMA (headdim % 32 == 0, dstate % 8 == 0 up to 128) -----------------------------------
F32_MFMA_CASES = [
    # Bt, T, H, P, N, G, L, with h0
    (1, 512, 4, 32, 16, 1, 64, False),      # configs[0]
    (1, 700, 4, 64, 128, 2, 256, True),     # Mamba-2 head shape, ragged last block, carried state
    (2, 2048, 8, 64, 128, 1, 256, False),   # 32 blocks per sequence
    (2, 130, 6, 96, 72, 3, 64, True),       # three column slices per head, dstate 72: a padded third state tile
    (1, 1, 2, 32, 8, 1, 16, True),          # a single token
    (3, 65, 4, 32, 40, 2, 100, False),      # one block and one token; chunk neither a divisor nor a multiple of 64
]


@pytest.mark.parametrize("case", F32_MFMA_CASES, ids=lambda c: "x".join(map(str, c)))
def test_f32_mfma_prefill_matches_oracle(ssd, case):
    *dims, with_h0 = case
    cfg = cfg_of(*dims, "f32")
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        torch.float32)
    if cfg.seqlen == 512:
        assert ssd.prefill_path(sh) == "mfma_f32"      # configs[0] takes it by the library's own choice
    ssd.set_knob("force_mfma_f32", 1)                  # (few heads and many blocks would go to the generic kernels)
    assert ssd.prefill_path(sh) == "mfma_f32"
    h0 = inputs.make_state(cfg, seed=6, scale=0.3) if with_h0 else None
    inp, y, st = run_prefill(ssd, cfg, seed=41, h0=h0)
    _, y2, st2 = run_prefill(ssd, cfg, seed=41, h0=h0)
    assert torch.equal(y, y2) and torch.equal(st, st2)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    e = assert_close(y, y_ref, 1e-4, "fp32 mfma y")
    assert_close(st, st_ref, 1e-4, "fp32 mfma final state")
    print("errors", e, flush=True)
    # the generic fp32 kernels on the same inputs: both families are held to the same tolerance
    ssd.set_knob("force_generic", 1)
    assert ssd.prefill_path(sh) == "generic_f32"
    _, yg, stg = run_prefill(ssd, cfg, seed=41, h0=h0)
    assert_close(yg, y_ref, 1e-4, "generic fp32 y")
    assert_close(stg, st_ref, 1e-4, "generic fp32 final state")


@pytest.mark.parametrize("nseg", [2, 3, 5, 64])
@pytest.mark.parametrize("case", [(1, 700, 4, 64, 128, 2, 256, True), (2, 130, 6, 96, 72, 3, 64, True),
                                  (1, 512, 4, 32, 16, 1, 64, False), (3, 65, 4, 32, 40, 2, 100, False)],
                         ids=lambda c: "x".join(map(str, c)))
def test_f32_mfma_time_segments(ssd, case, nseg):
    """The fp32 MFMA kernel with every sequence cut into time segments (one workgroup each, the state up to
    the segment recomputed -- by all four waves, in partial sums -- not handed over): the oracle's results
    within the fp32 tolerance, the same on a second run.  More segments than blocks (64 here) leave the
    surplus workgroups without work."""
    *dims, with_h0 = case
    cfg = cfg_of(*dims, "f32")
    ssd.set_knob("force_mfma_f32", 1)
    h0 = inputs.make_state(cfg, seed=6, scale=0.3) if with_h0 else None
    ssd.set_knob("f32_segments", nseg)
    inp, y, st = run_prefill(ssd, cfg, seed=47, h0=h0)
    _, y2, st2 = run_prefill(ssd, cfg, seed=47, h0=h0)
    assert torch.equal(y, y2) and torch.equal(st, st2)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    assert_close(y, y_ref, 1e-4, "fp32 mfma y, %d time segments" % nseg)
    assert_close(st, st_ref, 1e-4, "fp32 mfma final state, %d time segments" % nseg)


def test_f32_mfma_prefill_with_steep_decay_and_fused_dt(ssd):
    """fp32 MFMA path at dt*|A| of 0.5 ... 12 per token (the mask is evaluated un-factorised, exponent never
    positive, so no step size is special), and with the step-size activation applied as dt is read."""
    cfg = cfg_of(2, 300, 4, 64, 128, 1, 64, "f32")
    ssd.set_knob("force_mfma_f32", 1)
    assert ssd.prefill_path(ssd.make_shape(2, 300, 4, 64, 128, 1, 64, torch.float32)) == "mfma_f32"
    inp = _steep_inputs(cfg, "uniform", seed=43)
    dev = {k: v.cuda() for k, v in inp.items()}
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    torch.cuda.synchronize()
    y_ref, st_ref = oracle_prefill(inp)
    for h in range(cfg.nheads):
        assert_close(to_np64(y)[:, :, h], y_ref[:, :, h], 1e-4, "steep fp32 y, head %d" % h)
        assert_close(to_np64(st)[:, h], st_ref[:, h], 1e-4, "steep fp32 state, head %d" % h)
    raw = inputs.make_prefill_inputs(cfg, seed=44)
    g = torch.Generator().manual_seed(45)
    dt_raw = torch.randn(raw["dt"].shape, generator=g) * 1.5 - 3.0
    bias = torch.randn((cfg.nheads,), generator=g) * 0.5
    dev = {k: v.cuda() for k, v in raw.items()}
    y, st = ssd.ssd_prefill(dev["x"], dt_raw.cuda(), dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk,
                            dt_bias=bias.cuda(), dt_softplus=True, dt_limit=(1e-3, 0.5))
    torch.cuda.synchronize()
    raw["dt"] = torch.from_numpy(ssd_oracle.dt_transform(dt_raw, bias, True, (1e-3, 0.5))).float()
    y_ref, st_ref = oracle_prefill(raw)
    assert_close(y, y_ref, 1e-4, "fp32 mfma y with fused dt")
    assert_close(st, st_ref, 1e-4, "fp32 mfma state with fused dt")


# ---- steep decay: step sizes far beyond the benchmark's dt*|A| <= 1.6 ------------------------------------
def _steep_inputs(cfg, kind, seed):
    inp = inputs.make_prefill_inputs(cfg, seed=seed)
    H = cfg.nheads
    if kind == "uniform":
        # dt*|A| per token = 0.5, 3, 6, 12, repeated over the heads: the decay across half a 64-token block
        # is 2^23, 2^139, 2^277, 2^554
        inp["dt"] = torch.full_like(inp["dt"], 0.5)
        inp["A"] = torch.tensor([-1.0, -6.0, -12.0, -24.0] * (H // 4))
    elif kind == "spikes":
        # the benchmark's step sizes with one token in sixteen 300 times larger: blocks differ, heads differ
        g = torch.Generator().manual_seed(seed + 1)
        spike = torch.rand(inp["dt"].shape, generator=g) < 1.0 / 16.0
        inp["dt"] = torch.where(spike, inp["dt"] * 300.0, inp["dt"])
    elif kind == "scaled_A":
        # the benchmark's step sizes (median 0.01, up to 0.1) against |A| up to 1200: dt*|A| of 3 and 12 at
        # the median, blocks on either side of the threshold inside one head
        inp["A"] = torch.tensor([-16.0, -300.0, -1200.0, -1.0] * (H // 4))
    else:
        raise ValueError(kind)
    return inp


STEEP_CASES = [
    # Bt, T, H, P, N, G, L, forced chunks per segment, kind, with h0
    (1, 300, 4, 64, 128, 1, 64, 0, "uniform", False),
    (2, 1000, 8, 64, 128, 2, 128, 1, "uniform", True),     # several segments, two groups, carried state
    (1, 1000, 4, 64, 128, 1, 128, 2, "spikes", True),
    (1, 2048, 8, 64, 128, 1, 256, 0, "scaled_A", False),
    (1, 700, 4, 128, 128, 1, 64, 1, "scaled_A", True),     # headdim 128: two slices share a head's records
    (1, 500, 4, 64, 256, 1, 128, 2, "scaled_A", False),    # dstate 256: two state slices
]


@pytest.mark.parametrize("case", STEEP_CASES, ids=lambda c: "x".join(map(str, c)))
def test_mfma_prefill_with_steep_decay_matches_oracle(ssd, case):
    """Blocks whose decay across half a block leaves the range of the factorised mask take the
    un-factorised form inside the same kernels (Eq. 3 holds for any dt and A): the result matches the
    oracle like any other, nothing is clamped and nothing turns non-finite."""
    *dims, seg, kind, with_h0 = case
    cfg = cfg_of(*dims, "bf16")
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        torch.bfloat16)
    assert ssd.prefill_path(sh) == "mfma_bf16"
    if seg:
        ssd.set_knob("seg_chunks", seg)
    else:
        ssd.set_knob("seg_chunks", 0)
    inp = _steep_inputs(cfg, kind, seed=61)
    spans = blocked_model.block_half_spans(inp["dt"], inp["A"]).max(axis=-1)      # (Bt, H, blocks)
    steep = spans > 96.0
    print("steep case", case, "steep blocks per head", steep.sum(axis=(0, 2)).tolist(), "of", steep.shape[2],
          "largest half-block exponent %.0f" % spans.max(), flush=True)
    assert steep.any() and not steep.all()
    h0 = None
    if with_h0:
        warm = inputs.make_prefill_inputs(cfg, seed=79)
        h0 = torch.from_numpy(oracle_prefill(warm)[1]).float()
    dev = {k: v.cuda() for k, v in inp.items()}
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk,
                            h0=None if h0 is None else h0.cuda())
    y2, st2 = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk,
                              h0=None if h0 is None else h0.cuda())
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(st, st2)
    y_ref, st_ref = oracle_prefill(inp, h0=h0)
    e = assert_close(y, y_ref, 2e-2, "steep y")
    assert_close(st, st_ref, 2e-2, "steep final state")
    # head by head: a steep head's outputs must not hide behind the scale of a gentle one
    yg = to_np64(y)
    for h in range(cfg.nheads):
        assert_close(yg[:, :, h], y_ref[:, :, h], 2e-2, "steep y, head %d" % h)
        assert_close(to_np64(st)[:, h], st_ref[:, h], 2e-2, "steep state, head %d" % h)
    print("errors", e, flush=True)


def test_varlen_prefill_with_steep_decay_matches_oracle(ssd):
    ssd.set_knob("seg_chunks", 1)
    lens = [130, 0, 700, 64, 5, 301]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = cfg_of(1, int(cu[-1]), 8, 64, 128, 2, 64, "bf16")
    inp = _steep_inputs(cfg, "scaled_A", seed=67)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    dev = {k: v.cuda() for k, v in pk.items()}
    h0 = 0.1 * torch.randn((len(lens), 8, 64, 128), generator=torch.Generator().manual_seed(5))
    print("steep packed batch", lens, flush=True)
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), cfg.chunk, h0=h0.cuda())
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, h0=h0)
    for h in range(cfg.nheads):
        assert_close(to_np64(y)[:, h], y_ref[:, h], 2e-2, "steep packed y, head %d" % h)
        assert_close(to_np64(st)[:, h], st_ref[:, h], 2e-2, "steep packed state, head %d" % h)


def test_mfma_and_generic_paths_agree(ssd):
    cfg = cfg_of(2, 700, 8, 64, 128, 2, 128, "bf16")
    inp, y, st = run_prefill(ssd, cfg, seed=29)
    ssd.set_knob("force_generic", 1)
    _, yg, stg = run_prefill(ssd, cfg, seed=29)
    ssd.set_knob("force_generic", 0)
    assert_close(y, to_np64(yg), 2e-2, "mfma vs generic y")
    assert_close(st, to_np64(stg), 2e-2, "mfma vs generic state")


@pytest.mark.parametrize("case", [(2, 1000, 8, 64, 128, 2, 128, 2), (1, 700, 4, 128, 128, 1, 64, 1)],
                         ids=lambda c: "x".join(map(str, c)))
def test_cache_policy_of_the_y_stores_changes_no_bit(ssd, case):
    """The full kernel writes y with ordinary or with non-temporal stores, chosen from the size of x;
    either way the result matches the oracle and the two agree bit for bit (plain and packed batches)."""
    *dims, seg = case
    cfg = cfg_of(*dims, "bf16")
    ssd.set_knob("seg_chunks", seg)
    outs = {}
    for pol in ("0", "1"):
        ssd.set_knob("y_stream", int(pol))
        print("y store policy", pol, case, flush=True)
        inp, y, st = run_prefill(ssd, cfg, seed=31)
        dev = {k: v.cuda() for k, v in inp.items()}
        Bt, T = cfg.batch, cfg.seqlen
        cu = torch.arange(0, Bt * T + 1, T, dtype=torch.int32, device="cuda")
        flat = lambda t: t.reshape(Bt * T, *t.shape[2:]).contiguous()
        yp, stp = ssd.ssd_prefill_varlen(flat(dev["x"]), flat(dev["dt"]), dev["A"], flat(dev["B"]), flat(dev["C"]),
                                         dev["D"], cu, cfg.chunk)
        torch.cuda.synchronize()
        outs[pol] = (y.clone(), st.clone(), yp.clone(), stp.clone())
    ssd.set_knob("y_stream", -1)
    y_ref, st_ref = oracle_prefill(inp)
    assert_close(outs["1"][0], y_ref, 2e-2, "streamed y")
    assert_close(outs["1"][1], st_ref, 2e-2, "final state beside streamed y")
    for a, b in zip(outs["0"], outs["1"]):
        assert torch.equal(a, b)
    assert_close(outs["1"][2].reshape(outs["1"][0].shape), y_ref, 2e-2, "streamed y, packed batch")


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_cache_policy_of_the_decode_state_changes_no_bit(ssd, io):
    """The decode step streams the state past the caches when the states of the call exceed the memory-side
    cache; forced on and off on a small call, both match the oracle and agree bit for bit."""
    Ly, Bt, H, P, N, G = 3, 2, 8, 64, 128, 2
    iod = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator().manual_seed(19)
    state = torch.randn((Ly, Bt, H, P, N), generator=g)
    x = torch.randn((Ly, Bt, H, P), generator=g).to(iod)
    dt = torch.rand((Ly, Bt, H), generator=g) * 0.1 + 1e-3
    A = -(torch.rand((Ly, H), generator=g) * 15 + 1)
    D = torch.randn((Ly, H), generator=g)
    B = (0.25 * torch.randn((Ly, Bt, G, N), generator=g)).to(iod)
    C = (0.25 * torch.randn((Ly, Bt, G, N), generator=g)).to(iod)
    outs = {}
    for pol in ("0", "1"):
        ssd.set_knob("decode_stream", int(pol))
        print("decode state policy", pol, io, flush=True)
        sd = state.cuda().clone()
        y = ssd.ssd_decode_step_layers(sd, x.cuda(), dt.cuda(), A.cuda(), B.cuda(), C.cuda(), D.cuda())
        torch.cuda.synchronize()
        outs[pol] = (y, sd)
    ssd.set_knob("decode_stream", -1)
    y_ref, st_ref = ssd_oracle.decode_step_layers(state, x, dt, A, B, C, D)
    assert_close(outs["1"][0], y_ref, TOL[io], "decode y, streamed state")
    assert_close(outs["1"][1], st_ref, 1e-5, "decode state, streamed")
    assert torch.equal(outs["0"][0], outs["1"][0]) and torch.equal(outs["0"][1], outs["1"][1])


def test_mfma_extreme_decay_and_determinism(ssd):
    cfg = cfg_of(1, 640, 4, 64, 128, 1, 256, "bf16")
    inp = inputs.make_prefill_inputs(cfg, seed=31)
    inp["dt"] = torch.full_like(inp["dt"], 0.1)
    inp["A"] = torch.tensor([-16.0, -1e-3, -4.0, -16.0])
    dev = {k: v.cuda() for k, v in inp.items()}
    y, st = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    y2, st2 = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(st, st2)
    y_ref, st_ref = oracle_prefill(inp)
    assert_close(y, y_ref, 2e-2, "extreme decay y (mfma)")
    assert_close(st, st_ref, 2e-2, "extreme decay state (mfma)")


# ---- packed variable-length batches (MFMA kernel family) ----------------------------------------
VARLEN_CASES = [
    # lengths (a tuple marks a filler sequence), H, G, L, forced chunks per segment, with h0
    ([64], 4, 1, 64, 0, False),                                  # one sequence, one block
    ([1, 63, 64, 65, 0, 300, 129], 4, 1, 64, 0, False),          # ragged ends, an empty sequence
    ([1, 63, 64, 65, 0, 300, 129], 8, 2, 64, 1, True),           # two groups, one chunk per segment, h0
    ([700, 5, 0, 0, 1000, 64], 4, 1, 128, 1, True),              # several segments per sequence
    ([(3,), 200, (70,), 130, (1,)], 4, 1, 256, 0, True),         # short fillers between long sequences
    ([1000, 1048], 12, 1, 256, 2, False),
    ([17] * 40, 4, 1, 64, 0, True),                              # many short sequences
    ([130, 0, 700, 64], (2, 128), 1, 64, 2, True),               # headdim 128 (H given as (heads, headdim))
    ([130, 0, 700, 64], (4, 64, 64), 1, 64, 2, True),            # dstate 64 (heads, headdim, dstate)
    ([130, 0, 700, 64], (4, 64, 256), 1, 64, 2, False),          # dstate 256: two state slices, outputs added
    ([300, 5, 200], (4, 128, 192), 2, 128, 1, True),             # dstate 192, headdim 128, two groups
    ([130, 0, 700, 64, 1], 6, 2, 100, 1, True),                  # three heads per group, chunk no multiple of 64
    ([64, 65, 300], 1, 1, 50, 2, False),                         # a single head
]


@pytest.mark.parametrize("case", VARLEN_CASES, ids=lambda c: "-".join(str(v) for v in c[1:]) + "-n%d" % len(c[0]))
def test_varlen_prefill_matches_oracle(ssd, case):
    lengths, H, G, L, seg_chunks, with_h0 = case
    H, P, N = (tuple(H) + (128,))[:3] if isinstance(H, tuple) else (H, 64, 128)
    lens = [v[0] if isinstance(v, tuple) else v for v in lengths]   # gaps are simply more sequences
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, nseq = int(cu[-1]), len(lens)
    if seg_chunks:
        ssd.set_knob("seg_chunks", seg_chunks)
    cfg = cfg_of(1, T, H, P, N, G, L, "bf16")
    inp = inputs.make_prefill_inputs(cfg, seed=31)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    h0 = inputs.make_state(cfg_of(nseq, 1, H, P, N, G, L, "bf16"), seed=31) if with_h0 else None
    print("varlen case", lens, "H", H, "G", G, "L", L, "seg_chunks", seg_chunks, "h0", with_h0, flush=True)
    dev = {k: v.cuda() for k, v in pk.items()}
    y = torch.full_like(dev["x"], 7.0)
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), L, h0=None if h0 is None else h0.cuda(), y=y)
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, h0=h0)
    assert_close(y, y_ref, 2e-2, "varlen y")
    assert_close(st, st_ref, 2e-2, "varlen final states")
    # every sequence on its own through the plain entry point: same kernels, same values
    for q in range(nseq):
        a, b = int(cu[q]), int(cu[q + 1])
        if b == a:
            continue
        # (copies: a slice of a contiguous tensor is a view, and its pointer need not be 16-byte aligned)
        yq, sq = ssd.ssd_prefill(dev["x"][None, a:b].clone(), dev["dt"][None, a:b].clone(), dev["A"],
                                 dev["B"][None, a:b].clone(), dev["C"][None, a:b].clone(), dev["D"], L,
                                 h0=None if h0 is None else h0[q:q + 1].cuda())
        torch.cuda.synchronize()
        assert_close(y[a:b], to_np64(yq[0]), 2e-2, "varlen y vs single sequence %d" % q)
        assert_close(st[q], to_np64(sq[0]), 2e-2, "varlen state vs single sequence %d" % q)


@pytest.mark.parametrize("N", [128, 256])   # 256: two state slices, whose sum must skip unowned tokens too
def test_varlen_leaves_unowned_tokens_alone_and_rejects_bad_boundaries(ssd, N):
    H, L = 4, 64
    T = 400
    cfg = cfg_of(1, T, H, 64, N, 1, L, "bf16")
    assert ssd.prefill_path(ssd.make_shape(2, T, H, 64, N, 1, L, torch.bfloat16)) == "mfma_bf16"
    inp = inputs.make_prefill_inputs(cfg, seed=37)
    dev = {k: (v[0] if k in ("x", "dt", "B", "C") else v).cuda() for k, v in inp.items()}
    # tokens [0, 10) and [300, 400) belong to no sequence
    cu = torch.tensor([10, 100, 300], dtype=torch.int32).cuda()
    y = torch.full_like(dev["x"], 7.0)
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cu, L, y=y)
    torch.cuda.synchronize()
    assert (y[:10] == 7.0).all() and (y[300:] == 7.0).all()
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"],
                                              np.array([10, 100, 300], dtype=np.int32))
    assert_close(y[10:300], y_ref[10:300], 2e-2, "varlen y with unowned tokens")
    assert_close(st, st_ref, 2e-2, "varlen states with unowned tokens")
    # boundaries that decrease, or run past the token count: the call is a no-op
    for bad in ([0, 200, 100], [0, 100, 401], [-1, 100, 300]):
        y2 = torch.full_like(dev["x"], 7.0)
        st2 = torch.full((2, H, 64, N), 5.0, device="cuda")
        ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                               torch.tensor(bad, dtype=torch.int32).cuda(), L, y=y2, final_state=st2)
        torch.cuda.synchronize()
        assert (y2 == 7.0).all() and (st2 == 5.0).all(), bad


# ---- step-size activation fused into the prefill ---------------------------------------------
@pytest.mark.parametrize("case", [
    # Bt, T, H, P, N, G, L, io, bias, softplus, limit
    (2, 300, 8, 64, 128, 1, 128, "bf16", True, True, (1e-3, 1e-1)),     # MFMA family: fused in the block preparation
    (1, 1000, 4, 64, 128, 1, 256, "bf16", True, True, None),
    (1, 200, 4, 64, 128, 1, 64, "bf16", False, False, (2e-3, 5e-2)),    # clamp only
    (2, 100, 4, 32, 16, 2, 32, "f32", True, True, (1e-3, 1e-1)),        # generic family
    (1, 65, 2, 16, 8, 1, 64, "bf16", True, False, None),                # bias only
], ids=lambda c: "x".join(str(v) for v in c))
def test_prefill_with_fused_dt_transform(ssd, case):
    Bt, T, H, P, N, G, L, io, with_bias, softplus, limit = case
    cfg = cfg_of(Bt, T, H, P, N, G, L, io)
    inp = inputs.make_prefill_inputs(cfg, seed=71)
    g = torch.Generator().manual_seed(72)
    # raw values: what a projection would emit before the activation
    raw = 0.5 * torch.randn((Bt, T, H), generator=g) + (inputs.DT_BIAS if softplus else 0.02)
    bias = 0.3 * torch.randn((H,), generator=g) if with_bias else None
    if not softplus and limit is None:
        raw = raw.abs() * 0.05 + 0.02     # stay positive without an activation
        bias = bias.abs() * 0.01 if bias is not None else None
    print("dt transform case", case, flush=True)
    dev = {k: v.cuda() for k, v in inp.items()}
    y, st = ssd.ssd_prefill(dev["x"], raw.cuda(), dev["A"], dev["B"], dev["C"], dev["D"], L,
                            dt_bias=None if bias is None else bias.cuda(), dt_softplus=softplus, dt_limit=limit)
    torch.cuda.synchronize()
    dt_ref = ssd_oracle.dt_transform(raw, bias, softplus, limit)
    assert dt_ref.min() > 0
    y_ref, st_ref = ssd_oracle.prefill(inp["x"], dt_ref, inp["A"], inp["B"], inp["C"], inp["D"])
    assert_close(y, y_ref, TOL[io], "fused dt: y")
    assert_close(st, st_ref, TOL[io], "fused dt: state")


@pytest.mark.parametrize("case", [
    # lengths, H, P, N, G, L, io
    ([300, 64, 1, 500], 4, 64, 128, 1, 128, "bf16"),      # MFMA family
    ([70, 7, 100], 3, 24, 20, 3, 16, "f32"),              # generic family
], ids=lambda c: "x".join(str(v) for v in c[1:]) + "-n%d" % len(c[0]))
def test_varlen_prefill_with_fused_dt_transform(ssd, case):
    lens, H, P, N, G, L, io = case
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    cfg = cfg_of(1, T, H, P, N, G, L, io)
    inp = inputs.make_prefill_inputs(cfg, seed=73)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    g = torch.Generator().manual_seed(74)
    raw = 0.5 * torch.randn((T, H), generator=g) + inputs.DT_BIAS
    bias = 0.3 * torch.randn((H,), generator=g)
    limit = (1e-3, 1e-1)
    print("varlen dt transform case", case, flush=True)
    dev = {k: v.cuda() for k, v in pk.items()}
    y, st = ssd.ssd_prefill_varlen(dev["x"], raw.cuda(), dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), L, dt_bias=bias.cuda(), dt_softplus=True, dt_limit=limit)
    torch.cuda.synchronize()
    dt_ref = ssd_oracle.dt_transform(raw, bias, True, limit)
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], dt_ref, pk["A"], pk["B"], pk["C"], pk["D"], cu)
    assert_close(y, y_ref, TOL[io], "varlen fused dt: y")
    assert_close(st, st_ref, TOL[io], "varlen fused dt: states")


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("case", [
    # Ly, Bt, H, P, N, G, steps, bias, softplus, limit
    (3, 2, 8, 64, 128, 2, 6, True, True, (1e-3, 1e-1)),     # vector kernel / register-resident multi-step kernel
    (2, 1, 5, 7, 6, 5, 3, True, True, None),                # any-shape kernel, per-step launches
    (1, 2, 4, 64, 64, 1, 5, False, False, (2e-3, 5e-2)),    # clamp only
], ids=lambda c: "x".join(str(v) for v in c))
def test_decode_with_fused_dt_transform(ssd, case, io):
    """Alg. 2, "Discretise": the decode entry points apply the step-size activation themselves."""
    Ly, Bt, H, P, N, G, S, with_bias, softplus, limit = case
    iod = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator().manual_seed(75)
    state = torch.randn((Ly, Bt, H, P, N), generator=g)
    x = torch.randn((S, Ly, Bt, H, P), generator=g).to(iod)
    raw = 0.5 * torch.randn((S, Ly, Bt, H), generator=g) + (inputs.DT_BIAS if softplus else 0.02)
    bias = 0.3 * torch.randn((Ly, H), generator=g) if with_bias else None
    A = -(torch.rand((Ly, H), generator=g) * 15 + 1)
    D = torch.randn((Ly, H), generator=g)
    B = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).to(iod)
    C = (0.25 * torch.randn((S, Ly, Bt, G, N), generator=g)).to(iod)
    # bias has a layer axis: broadcast (Ly, 1, H) against raw (S, Ly, Bt, H)
    dt_ref = ssd_oracle.dt_transform(raw, None if bias is None else bias[:, None, :], softplus, limit)
    y_ref, st_ref = ssd_oracle.decode_steps_layers(state, x, dt_ref, A, B, C, D)
    kw = dict(dt_bias=None if bias is None else bias.cuda(), dt_softplus=softplus, dt_limit=limit)
    print("decode dt transform case", case, io, flush=True)
    dev = [t.cuda() for t in (x, raw, A, B, C, D)]
    sd = state.cuda().clone()
    y = ssd.ssd_decode_steps_layers(sd, *dev, **kw)
    torch.cuda.synchronize()
    assert_close(y, y_ref, TOL[io], "multi-step decode, fused dt: y")
    assert_close(sd, st_ref, 1e-4, "multi-step decode, fused dt: state")
    s1 = state.cuda().clone()
    for s in range(S):
        ys = ssd.ssd_decode_step_layers(s1, dev[0][s].clone(), dev[1][s].clone(), dev[2], dev[3][s].clone(),
                                        dev[4][s].clone(), dev[5], **kw)
        torch.cuda.synchronize()
        assert_close(ys, y_ref[s], TOL[io], "single decode step %d, fused dt: y" % s)
    assert_close(s1, st_ref, 1e-4, "single decode steps, fused dt: state")


GENERIC_VARLEN_CASES = [
    # lengths, H, P, N, G, L, io, with h0
    ([5, 0, 33, 64, 1, 100], 4, 32, 16, 2, 32, "f32", True),      # fp32 io: the 1e-4 tolerance family
    ([70, 7], 3, 24, 20, 3, 7, "f32", False),                      # nothing is a multiple of any tile
    ([130, 0, 300], 2, 72, 40, 1, 128, "bf16", True),              # bf16, head shape outside the MFMA family
    ([200, 57, 64], 4, 64, 100, 1, 64, "bf16", True),              # dstate not a multiple of 8: generic kernels
    ([1000], 2, 16, 8, 1, 2048, "f32", False),                     # chunk longer than everything
]


@pytest.mark.parametrize("case", GENERIC_VARLEN_CASES, ids=lambda c: "x".join(str(v) for v in c[1:]) + "-n%d" % len(c[0]))
def test_varlen_prefill_generic_family_matches_oracle(ssd, case):
    lens, H, P, N, G, L, io, with_h0 = case
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, nseq = int(cu[-1]), len(lens)
    cfg = cfg_of(1, T, H, P, N, G, L, io)
    inp = inputs.make_prefill_inputs(cfg, seed=83)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    h0 = inputs.make_state(cfg_of(nseq, 1, H, P, N, G, L, io), seed=83) if with_h0 else None
    print("generic varlen case", case, flush=True)
    dev = {k: v.cuda() for k, v in pk.items()}
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), L, h0=None if h0 is None else h0.cuda())
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, h0=h0)
    assert_close(y, y_ref, TOL[io], "generic varlen y")
    assert_close(st, st_ref, TOL[io], "generic varlen final states")


def test_varlen_families_agree_and_bad_boundaries_are_a_no_op_on_both(ssd):
    lens = [100, 0, 300, 65]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = cfg_of(1, int(cu[-1]), 4, 64, 128, 1, 64, "bf16")
    inp = inputs.make_prefill_inputs(cfg, seed=89)
    dev = {k: (v[0] if k in ("x", "dt", "B", "C") else v).cuda() for k, v in inp.items()}
    cud = torch.from_numpy(cu).cuda()
    y1, s1 = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cud, 64)
    ssd.set_knob("force_generic", 1)
    y2, s2 = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cud, 64)
    torch.cuda.synchronize()
    assert_close(y1, to_np64(y2), 2e-2, "varlen: MFMA vs generic y")
    assert_close(s1, to_np64(s2), 2e-2, "varlen: MFMA vs generic state")
    y3 = torch.full_like(dev["x"], 7.0)
    s3 = torch.full((4, 4, 64, 128), 5.0, device="cuda")
    ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                           torch.tensor([0, 200, 100, 300, 465], dtype=torch.int32).cuda(), 64, y=y3, final_state=s3)
    torch.cuda.synchronize()
    assert (y3 == 7.0).all() and (s3 == 5.0).all()


def test_prefill_replayed_from_a_hip_graph(ssd):
    """The library allocates nothing and never synchronises, so a prefill (plain and packed) can be
    captured into a HIP graph; every replay, with eager work and synchronisations in between and the
    inputs changed in place, equals the eager call on the same inputs."""
    cfg = cfg_of(2, 1000, 8, 64, 128, 1, 256, "bf16")
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        torch.bfloat16)
    dev = {k: v.cuda() for k, v in inputs.make_prefill_inputs(cfg, seed=91).items()}
    pk = {k: (v.reshape((-1,) + tuple(v.shape[2:])) if k in ("x", "dt", "B", "C") else v) for k, v in dev.items()}
    cu = torch.tensor([0, 700, 700, 1300, 2000], dtype=torch.int32).cuda()
    y, st = torch.empty_like(dev["x"]), torch.empty((2, 8, 64, 128), device="cuda")
    yv, stv = torch.empty_like(pk["x"]), torch.empty((4, 8, 64, 128), device="cuda")
    ws = torch.empty((ssd.prefill_workspace_bytes(sh),), dtype=torch.uint8, device="cuda")
    shv = ssd.make_shape(4, 2000, 8, 64, 128, 1, 256, torch.bfloat16)
    wsv = torch.empty((ssd.raw().ssd_prefill_varlen_workspace_bytes(shv),), dtype=torch.uint8, device="cuda")

    def both(y, st, yv, stv):
        ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk, y=y, final_state=st,
                        workspace=ws)
        ssd.ssd_prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, cfg.chunk, y=yv,
                               final_state=stv, workspace=wsv)

    both(y, st, yv, stv)  # warm-up outside the capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            both(y, st, yv, stv)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        dev["x"].mul_(-0.5 if rep else 1.0)          # new inputs in the same buffers (pk views them)
        dev["dt"].mul_(1.1).clamp_(1e-3, 1e-1)
        y.zero_(), st.zero_(), yv.zero_(), stv.zero_()
        graph.replay()
        torch.cuda.synchronize()
        ye, se, yve, sve = torch.empty_like(y), torch.empty_like(st), torch.empty_like(yv), torch.empty_like(stv)
        both(ye, se, yve, sve)
        torch.cuda.synchronize()
        assert torch.equal(y, ye) and torch.equal(st, se), "plain prefill, replay %d" % rep
        assert torch.equal(yv, yve) and torch.equal(stv, sve), "packed prefill, replay %d" % rep


def test_peak_probes_run_and_the_copy_probe_copies(ssd):
    from paper_2603_09555_amd import measure
    a = torch.arange(1 << 22, dtype=torch.int32, device="cuda")          # 16 MiB
    b = torch.zeros_like(a)
    rate, ms = measure.peak_probe("copy", a, b, reps=2)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and rate > 1e11 and ms > 0
    odd = torch.arange(1000 * 4 + 4, dtype=torch.int32, device="cuda")    # not a multiple of the 32 KB slabs
    out = torch.zeros_like(odd)
    measure.peak_probe("copy", odd, out)
    torch.cuda.synchronize()
    assert torch.equal(odd, out)
    for kind in ("read", "write", "read_nt", "write_nt"):
        rate, _ = measure.peak_probe(kind, a, b, reps=2)
        assert rate > 1e11
    b.zero_()
    measure.peak_probe("copy_nt", a, b)
    measure.peak_probe("copy_nt", odd, out.zero_())
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(odd, out)
    rate, _ = measure.peak_probe("mfma", a, None, iters=50, reps=2)
    assert rate > 1e13


def _random_cases(seed, n):
    """Seeded random shapes: MFMA-family and generic-family, plain and packed, with and without h0."""
    r = np.random.default_rng(seed)
    out = []
    for i in range(n):
        mfma = bool(i % 2)
        if mfma:
            P = int(r.choice([64, 128]))
            N = int(r.choice([32, 64, 128, 192, 256]))
            G = int(r.choice([1, 2]))
            H = G * int(r.choice([4, 8])) if P == 64 else G * int(r.choice([2, 4]))
            L = int(r.choice([64, 128, 256]))
            io = "bf16"
        else:
            P = int(r.integers(1, 80))
            N = int(r.integers(1, 70))
            G = int(r.choice([1, 2, 3]))
            H = G * int(r.integers(1, 4))
            L = int(r.integers(1, 200))
            io = str(r.choice(["f32", "bf16"]))
        nseq = int(r.integers(1, 5))
        lens = [int(v) for v in r.integers(0, 400 if mfma else 150, nseq)]
        if sum(lens) == 0:
            lens[0] = 1 + int(r.integers(0, 100))
        out.append((lens, H, P, N, G, L, io, bool(r.integers(0, 2)), int(r.integers(0, 3))))
    return out


@pytest.mark.parametrize("case", _random_cases(2024, 24), ids=lambda c: "%s-%dx%dx%dx%dx%d-%s-h0%d-seg%d" % (
    "+".join(map(str, c[0])), c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8]))
def test_random_shapes_plain_and_packed(ssd, case):
    """Each random case runs packed (all sequences in one call) and plain (the longest sequence alone,
    batch 1): both against the oracle."""
    lens, H, P, N, G, L, io, with_h0, seg = case
    if seg:
        ssd.set_knob("seg_chunks", seg)
    tol = TOL[io]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, nseq = int(cu[-1]), len(lens)
    cfg = cfg_of(1, T, H, P, N, G, L, io)
    inp = inputs.make_prefill_inputs(cfg, seed=sum(lens) + H)
    pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
    h0 = inputs.make_state(cfg_of(nseq, 1, H, P, N, G, L, io), seed=3, scale=0.5) if with_h0 else None
    print("random case", case, flush=True)
    dev = {k: v.cuda() for k, v in pk.items()}
    y, st = ssd.ssd_prefill_varlen(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"],
                                   torch.from_numpy(cu).cuda(), L, h0=None if h0 is None else h0.cuda())
    torch.cuda.synchronize()
    y_ref, st_ref = ssd_oracle.prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, h0=h0)
    assert_close(y, y_ref, tol, "packed y")
    assert_close(st, st_ref, tol, "packed states")
    q = int(np.argmax(lens))
    a, b = int(cu[q]), int(cu[q + 1])
    # (clones: a slice of a contiguous tensor is a view at an offset that need not be 16-byte aligned)
    yq, sq = ssd.ssd_prefill(dev["x"][None, a:b].clone(), dev["dt"][None, a:b].clone(), dev["A"],
                             dev["B"][None, a:b].clone(), dev["C"][None, a:b].clone(), dev["D"], L,
                             h0=None if h0 is None else h0[q:q + 1].cuda())
    torch.cuda.synchronize()
    assert_close(yq[0], y_ref[a:b], tol, "plain y")
    assert_close(sq[0], st_ref[q], tol, "plain state")
