"""``ssd_prefill_static`` -- the prefill on the library's own static scratch buffer, for callers that cannot
allocate -- against ``ssd_prefill`` with a caller-provided workspace, through the C ABI: the same kernels
run on the same inputs, so outputs must agree bit for bit (which also puts them inside the oracle
tolerance that ``ssd_prefill`` is held to); two calls in a row, the second on a smaller input, and a shape
beyond the buffer, which must be refused."""
import ctypes

import pytest
import torch

from oracle import ssd_oracle
from paper_2603_09555_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ssd():
    from paper_2603_09555_amd import ssd as binding
    return binding


def _both(ssd, cfg, seed, with_h0):
    inp = inputs.make_prefill_inputs(cfg, seed=seed)
    dev = {k: v.cuda() for k, v in inp.items()}
    h0 = inputs.make_state(cfg, seed=seed + 1, scale=0.1) if with_h0 else None
    h0d = None if h0 is None else h0.cuda()
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        cfg.torch_io_dtype)
    assert ssd.prefill_workspace_bytes(sh) <= ssd.STATIC_SCRATCH_BYTES
    y_ref, st_ref = ssd.ssd_prefill(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk, h0=h0d)
    y = torch.full_like(dev["x"], float("nan"))
    st = torch.full((cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), float("nan"), device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    print("static prefill", cfg, flush=True)
    ssd.ssd_prefill_static(dev["x"], dev["dt"], dev["A"], dev["B"], dev["C"], dev["D"], cfg.chunk, y, st, h0=h0d)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(y, y_ref) and torch.equal(st, st_ref)
    return inp, h0, y, st


def test_static_prefill_equals_prefill_two_calls_in_a_row(ssd):
    big = inputs.SSDConfig("static_big", 1, 2048, 24, 64, 128, 1, 256, "bf16")        # configs[1]: several segments
    small = inputs.SSDConfig("static_small", 2, 300, 4, 64, 128, 1, 64, "bf16")
    tiny = inputs.SSDConfig("static_f32", 1, 100, 4, 32, 16, 2, 32, "f32")            # the generic fp32 kernels
    _both(ssd, big, 3, False)
    inp, h0, y, st = _both(ssd, small, 5, True)     # smaller, on what the first call left in the buffer
    y_o, st_o = ssd_oracle.prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], h0=h0)
    assert_close(y, y_o, 2e-2, "static prefill y vs the oracle")
    assert_close(st, st_o, 2e-2, "static prefill state vs the oracle")
    _both(ssd, tiny, 7, False)
    _both(ssd, big, 9, True)


def test_static_prefill_refuses_what_does_not_fit(ssd):
    cfg = inputs.CONFIGS["c3_2p7b_long"]
    sh = ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                        cfg.torch_io_dtype)
    assert ssd.prefill_workspace_bytes(sh) > ssd.STATIC_SCRATCH_BYTES
    lib = ssd.raw()
    one = ctypes.c_void_p(256)   # never dereferenced: the call must return before any HIP call
    st = lib.ssd_prefill_static(ctypes.byref(sh), one, one, one, one, one, one, None, one, one, None)
    assert st == -8 and "scratch" in ssd.status_string(st)
