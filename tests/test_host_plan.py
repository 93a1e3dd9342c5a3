"""Host-side tests of how the library cuts a prefill up (``ssd_testing_prefill_plan``: host arithmetic only, no
GPU): the choices the design notes state for the benchmark shapes, the effect of the test-only knobs, and the
invariants the kernels rely on, over a grid of shapes."""
import itertools

import pytest
import torch

from paper_2603_09555_amd import inputs, ssd


@pytest.fixture(autouse=True)
def _reset():
    ssd.reset_knobs()
    yield
    ssd.reset_knobs()


def shape_of(c):
    return ssd.make_shape(c.batch, c.seqlen, c.nheads, c.headdim, c.dstate, c.ngroups, c.chunk, c.torch_io_dtype)


def test_plans_of_the_benchmark_shapes():
    plan = {n: ssd.prefill_plan(shape_of(c)) for n, c in inputs.CONFIGS.items() if not c.decode_steps}
    # config 0: fp32 MFMA kernel, eight time segments of one block (four workgroups would leave the chip idle)
    assert plan["c0_tiny_f32"]["path"] == "mfma_f32" and plan["c0_tiny_f32"]["f32_segments"] == 8
    # config 1: 32 blocks -> 16 segments of 2; a chain of 15 slots is not folded
    assert plan["c1_130m"] == dict(path="mfma_bf16", seg_blocks=2, segments=16, parts=1, fold=False, f32_segments=0)
    # config 2: x (201 MB) does not survive in the memory-side cache -> 36 + 28 blocks; the states pass in two
    # pieces; a chain of two slots is summed by the full scan itself
    assert plan["c2_780m_b8"] == dict(path="mfma_bf16", seg_blocks=36, segments=2, parts=2, fold=True, f32_segments=0)
    # config 3: 256 blocks -> 12 segments of 22 (240 workgroups)
    assert plan["c3_2p7b_long"] == dict(path="mfma_bf16", seg_blocks=22, segments=12, parts=1, fold=False, f32_segments=0)


def test_knobs_and_aliasing_change_the_plan():
    sh = shape_of(inputs.CONFIGS["c2_780m_b8"])
    assert ssd.prefill_plan(sh)["fold"]
    assert not ssd.prefill_plan(sh, h0_aliases_final_state=True)["fold"]   # h0 and final_state in one buffer
    ssd.set_knob("fold_max_slots", 0)
    assert not ssd.prefill_plan(sh)["fold"]
    ssd.set_knob("fold_max_slots", 1)
    p = ssd.prefill_plan(sh)                                                # (the choice of lengths knows the limit)
    assert p["fold"] == ((p["segments"] - 1) * p["parts"] <= 1)
    ssd.set_knob("seg_blocks", 36)
    ssd.set_knob("seg_parts", 2)
    assert not ssd.prefill_plan(sh)["fold"]                                 # a chain of two slots is over the limit
    ssd.reset_knobs()
    ssd.set_knob("seg_parts", 1)
    assert ssd.prefill_plan(sh) == dict(path="mfma_bf16", seg_blocks=36, segments=2, parts=1, fold=True, f32_segments=0)
    ssd.reset_knobs()
    ssd.set_knob("seg_blocks", 16)
    p = ssd.prefill_plan(sh)
    assert (p["seg_blocks"], p["segments"]) == (16, 4)
    ssd.reset_knobs()
    ssd.set_knob("force_generic", 1)
    assert ssd.prefill_plan(sh)["path"] == "generic_f32"
    ssd.reset_knobs()
    c0 = shape_of(inputs.CONFIGS["c0_tiny_f32"])
    ssd.set_knob("f32_segments", 3)
    assert ssd.prefill_plan(c0)["f32_segments"] == 3
    ssd.set_knob("f32_segments", 100)                                       # at most one per block
    assert ssd.prefill_plan(c0)["f32_segments"] == 8


GRID = list(itertools.product([1, 2, 3, 8, 16], [1, 64, 1000, 2048, 4096, 16384, 50000], [4, 8, 24, 48, 80, 128],
                              [64, 128], [256, 64]))


def test_plan_invariants_over_a_grid_of_shapes():
    base = inputs.CONFIGS["c3_2p7b_long"]
    for Bt, T, H, P, L in GRID:
        c = base.with_(batch=Bt, seqlen=T, nheads=H, headdim=P, chunk=L)
        sh = shape_of(c)
        p = ssd.prefill_plan(sh)
        assert p["path"] == "mfma_bf16", (Bt, T, H, P, L)
        nblocks = (T + 63) // 64
        assert 1 <= p["seg_blocks"] and p["segments"] == (nblocks + p["seg_blocks"] - 1) // p["seg_blocks"]
        assert p["parts"] >= 1 and p["seg_blocks"] % p["parts"] == 0
        assert p["segments"] > 1 or p["parts"] == 1
        # the workspace holds one state slot per piece and head: its size must cover the plan whatever it is
        slots = (p["segments"] - 1) * p["parts"] + 1
        per_slot = Bt * H * P * 128 * 4
        assert ssd.prefill_workspace_bytes(sh) >= slots * per_slot, (Bt, T, H, P, L, p)
        assert p["fold"] == (p["segments"] >= 2 and (p["segments"] - 1) * p["parts"] <= 3)
        assert not ssd.prefill_plan(sh, True)["fold"]


def test_f32_time_segments_over_a_grid_of_shapes():
    base = inputs.CONFIGS["c0_tiny_f32"]
    for Bt, T, H, P, N in itertools.product([1, 2, 8], [1, 64, 65, 512, 4096], [2, 4, 24, 80], [32, 64], [16, 64, 128]):
        c = base.with_(batch=Bt, seqlen=T, nheads=H, headdim=P, dstate=N)
        ssd.set_knob("force_mfma_f32", 1)
        p = ssd.prefill_plan(shape_of(c))
        assert p["path"] == "mfma_f32"
        nblocks, wgs = (T + 63) // 64, Bt * H * (P // 32)
        s = p["f32_segments"]
        assert 1 <= s <= max(1, nblocks)
        assert s == 1 or wgs * s <= 256          # the library cuts only as far as the workgroups run side by side
        if wgs * 2 <= 256 and nblocks >= 2:
            assert s >= 2                        # and does cut when half the chip would idle
