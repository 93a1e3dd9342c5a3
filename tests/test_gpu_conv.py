"""GPU parity of the depthwise causal convolution (the step in front of the SSD core) against
the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import ssd_oracle
from parity import TOL, assert_close, to_np64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ssd():
    from paper_2603_09555_amd import ssd as binding
    return binding


def draw(Bt, T, C, k, io, seed):
    g = torch.Generator().manual_seed(seed)
    iod = torch.float32 if io == "f32" else torch.bfloat16
    u = torch.randn((Bt, T, C), generator=g).to(iod)
    w = torch.randn((C, k), generator=g) / k
    b = 0.1 * torch.randn((C,), generator=g)
    st = torch.randn((Bt, C, k - 1), generator=g).to(iod)
    return u, w, b, st


CONV_CASES = [
    # Bt, T, C (as split), k, activation, with cache, with bias
    (1, 64, (256,), 4, "silu", False, True),
    (2, 100, (128, 32, 32), 4, "silu", True, True),      # three outputs, ragged run of tokens
    (2, 33, (24, 8, 8), 4, "none", True, False),
    (1, 2, (64,), 4, "silu", True, True),                # prompt shorter than the cache
    (3, 70, (37,), 4, "silu", True, True),               # channel count not a multiple of 8
    (2, 45, (20, 3, 3), 3, "none", True, True),          # scalar path with three outputs
    (1, 200, (512, 128, 128), 2, "silu", False, False),
    (1, 90, (64, 8, 8), 8, "silu", True, True),
    (2, 1, (5376,), 4, "silu", True, True),              # one token through the prompt kernel
]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_conv_prefill_and_step_match_oracle(ssd, case, io):
    Bt, T, split, k, act, with_state, with_bias = case
    C = sum(split)
    u, w, b, st = draw(Bt, T, C, k, io, seed=61)
    print("conv case", case, io, flush=True)
    outs, new_st = ssd.ssd_conv1d_prefill(u.cuda(), w.cuda(), b.cuda() if with_bias else None,
                                          st.cuda() if with_state else None, split=split, activation=act)
    torch.cuda.synchronize()
    z_ref, st_ref = ssd_oracle.conv1d_prefill(u, w, b if with_bias else None, st if with_state else None, act)
    assert [tuple(o.shape) for o in outs] == [(Bt, T, s) for s in split]
    assert_close(torch.cat(outs, dim=2), z_ref, TOL[io], "conv z")
    assert np.array_equal(to_np64(new_st), st_ref), "the cache is a copy of inputs: exact"
    # one more token through the step entry point, from the cache the prompt left
    u1 = torch.randn((Bt, C), generator=torch.Generator().manual_seed(62)).to(u.dtype)
    cache = new_st.clone()
    outs1 = ssd.ssd_conv1d_step(cache, u1.cuda(), w.cuda(), b.cuda() if with_bias else None, split=split,
                                activation=act)
    torch.cuda.synchronize()
    z1_ref, st1_ref = ssd_oracle.conv1d_step(st_ref, u1, w, b if with_bias else None, act)
    assert_close(torch.cat(outs1, dim=1), z1_ref, TOL[io], "conv step z")
    assert np.array_equal(to_np64(cache), st1_ref)


def test_conv_feeds_the_ssd_core(ssd):
    """The x | B | C ranges of the convolution output go straight into ssd_prefill as three dense
    tensors; the result matches the oracle run on the oracle's convolution output."""
    Bt, T, H, P, N, G, k = 2, 300, 8, 64, 128, 1, 4
    C = H * P + 2 * G * N
    u, w, b, _ = draw(Bt, T, C, k, "bf16", seed=63)
    g = torch.Generator().manual_seed(64)
    dt = torch.rand((Bt, T, H), generator=g) * 0.05 + 1e-3
    A = -(torch.rand((H,), generator=g) * 8 + 0.5)
    D = torch.randn((H,), generator=g)
    (zx, zB, zC), _ = ssd.ssd_conv1d_prefill(u.cuda(), w.cuda(), b.cuda(), None, split=(H * P, G * N, G * N))
    y, st = ssd.ssd_prefill(zx.view(Bt, T, H, P), dt.cuda(), A.cuda(), zB.view(Bt, T, G, N), zC.view(Bt, T, G, N),
                            D.cuda(), 256)
    torch.cuda.synchronize()
    # the oracle of the core consumes what the core consumed: the bf16-rounded convolution output
    y_ref, st_ref = ssd_oracle.prefill(zx.view(Bt, T, H, P).cpu(), dt, A, zB.view(Bt, T, G, N).cpu(),
                                       zC.view(Bt, T, G, N).cpu(), D)
    assert_close(y, y_ref, 2e-2, "ssd on conv output: y")
    assert_close(st, st_ref, 2e-2, "ssd on conv output: state")
    z_ref, _ = ssd_oracle.conv1d_prefill(u, w, b, None)
    assert_close(torch.cat([zx, zB, zC], dim=2), z_ref, 2e-2, "conv z")


def test_conv_prefill_replayed_from_a_graph_equals_eager(ssd):
    """The convolution enqueues one kernel and nothing else (the run length per thread comes from a host-side
    occupancy query, no device work), so it can be captured; replays equal the eager call bit for bit."""
    Bt, T, split, k = 2, 3000, (512, 64, 64), 4
    C = sum(split)
    u, w, b, st = draw(Bt, T, C, k, "bf16", seed=64)
    ud, wd, bd, sd = u.cuda(), w.cuda(), b.cuda(), st.cuda()
    eager, eager_cache = ssd.ssd_conv1d_prefill(ud, wd, bd, sd, split=split, activation="silu")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs, cache = ssd.ssd_conv1d_prefill(ud, wd, bd, sd, split=split, activation="silu")
    for rep in range(3):
        for o in outs:
            o.zero_()
        cache.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, e) for a, e in zip(outs, eager)), "replay %d" % rep
        assert torch.equal(cache, eager_cache)
