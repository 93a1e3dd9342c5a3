#!/usr/bin/env python3
"""Benchmark of the SSD layer core on one MI355X.

A "step" is one pass of the whole hot path on one batch of synthetic input: ``ssd_prefill``
over the prompt (segsum, intra-chunk masked product, chunk states, inter-chunk pass,
state-to-output, final state) followed by one ``ssd_decode_step`` on the state it returned.
Inputs are resident in HBM before the timed region.  The headline value is prefill
throughput in TFLOP/s by the *algorithmic, causal-only* FLOP count at the configured chunk
length (work the method must do: no per-head recomputation of C.B^T, no padding, no masked
upper triangle); the dense-convention figure is printed beside it.  The decode workload
(64 stacked layers, 1024 back-to-back steps, batch 16 and batch 1) is timed in a second
region and reported as HBM GB/s under ``decode`` (with the HIP-graph replay and the many-steps-per-
launch variant beside it).  Further objects of the same line, none of them part of the timed step:
``other_configs`` (configs 0-2), ``sweeps`` (chunk length, groups, head shapes), ``varlen`` (packed
ragged batches, piecewise prompts), ``conv`` (the depthwise convolution), ``measured_peaks`` (the
library's MFMA and streaming probes).  One JSON line is printed last.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # dense bf16 MFMA, MI355X
PEAK_VALU_F32_TFLOPS = 157.3     # fp32 vector, the published figure (counts packed fp32: 256 CUs x 4 SIMDs x 16
                                 # lanes x 2 (packed) x 2 (fma) x 2.4 GHz); the peak every "alu" fraction here uses
PEAK_VALU_F32_NON_PACKED = 78.6  # the same without packed instructions, which this build does not emit
PEAK_HBM_GBS = 8000.0


# ---- algorithmic work: what the method must compute, independent of how a kernel does it -------
def chunk_lengths(T, L):
    L = min(L, T)
    full, tail = divmod(T, L)
    return [L] * full + ([tail] if tail else [])


def prefill_flops(cfg, causal=True):
    """FLOPs one prefill must perform, split by step of Alg. 1 (per call, all batch rows)."""
    H, P, N, G = cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    out = dict(scores=0.0, intra=0.0, states=0.0, state_pass=0.0, state_out=0.0, skip=0.0)
    for ln in chunk_lengths(cfg.seqlen, cfg.chunk):
        k = (ln + 1) / (2.0 * ln) if causal else 1.0
        out["scores"] += G * 2.0 * ln * ln * N * k          # C.B^T, once per group
        out["intra"] += H * 2.0 * ln * ln * P * k           # (G o L).(dt o x)
        out["states"] += H * 2.0 * ln * P * N               # chunk-end states
        out["state_out"] += H * 2.0 * ln * N * P            # C.H_c
        out["state_pass"] += H * 2.0 * P * N                # H_{c+1} = decay*H_c + S_c
        out["skip"] += H * 2.0 * ln * P                     # + D x
    return {k: v * cfg.batch for k, v in out.items()}


def io_size(cfg):
    return 4 if cfg.io_dtype == "f32" else 2


def prefill_bytes(cfg):
    """Compulsory HBM traffic of one prefill: every input read once, every output written once."""
    Bt, T, H, P, N, G = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    sz = io_size(cfg)
    return 2 * Bt * T * H * P * sz + 4 * Bt * T * H + 2 * Bt * T * G * N * sz + 8 * H + 4 * Bt * H * P * N


def decode_bytes(cfg, nlayers):
    """Compulsory HBM traffic of one decode step over nlayers stacked layers."""
    Bt, H, P, N, G = cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    sz = io_size(cfg)
    per_layer = 2 * 4 * Bt * H * P * N + Bt * (2 * H * P * sz + 4 * H + 2 * G * N * sz) + 8 * H
    return nlayers * per_layer


def decode_flops(cfg, nlayers):
    return nlayers * cfg.batch * cfg.nheads * cfg.headdim * (5.0 * cfg.dstate + 3.0)


# HBM bytes per launch of a kernel come from the committed summary of the rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this file, profiles/hbm_traffic_fetch_write_size.txt: its "TRAFFIC <workload> <kernel>
# fetch_kib=.. write_kib=.." lines, scaled by the factors a copy of known size gives on this chip
# (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0; stated in the same file).  Nothing is typed in here; a kernel
# without a line reports null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_fetch_write_size.txt")
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0


def read_traffic(path=TRAFFIC_FILE):
    """{(workload, kernel): HBM bytes per launch} from the TRAFFIC lines of the counter summary."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 5 and w[0] == "TRAFFIC" and w[3].startswith("fetch_kib=") and w[4].startswith("write_kib="):
                    fetch, write = float(w[3].split("=")[1]), float(w[4].split("=")[1])
                    out[(w[1], w[2])] = int((FETCH_SCALE * fetch + WRITE_SCALE * write) * 1024)
    except OSError:
        pass
    return out


# Which algorithmic FLOPs each kernel of a prefill call is responsible for.
KERNEL_WORK = {
    # generic fp32 family
    "chunk_cumsum": (),
    "chunk_states": ("states",),
    "state_pass": ("state_pass",),
    "chunk_output": ("scores", "intra", "state_out", "skip"),
    # MFMA family
    "block_prep": ("scores",),
    "segment_states": (),          # re-computation: carries no algorithmic FLOPs of its own
    "segment_pass": ("state_pass",),
    "prefill_f32": ("scores", "intra", "states", "state_pass", "state_out", "skip"),   # fp32 MFMA: one kernel
    "chunk_scan": ("intra", "states", "state_out", "skip"),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--preheat-ms", type=float, default=100.0,
                    help="before the warm-up steps of every timed loop the same call is repeated for this long: after "
                         "an idle gap (input generation, the previous leg's teardown) the GPU takes some 30 ms of "
                         "sustained work to return to its steady clocks, which is the state a serving process is in")
    ap.add_argument("--workload", default="c3_2p7b_long",
                    help="prefill configuration of the timed step (see paper_2603_09555_amd.inputs.CONFIGS)")
    ap.add_argument("--decode-steps", type=int, default=1024)
    ap.add_argument("--decode-layers", type=int, default=64)
    ap.add_argument("--decode-block", type=int, default=64,
                    help="steps per HIP graph and per multi-step launch in the decode comparison")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the decode step")
    ap.add_argument("--no-peaks", action="store_true", help="skip the MFMA / streaming peak probes")
    ap.add_argument("--no-varlen", action="store_true")
    ap.add_argument("--no-conv", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-configs", action="store_true")
    ap.add_argument("--no-segment-model", action="store_true",
                    help="skip the check of the library's segment-length choice on shapes it was not fitted to")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (counter calibration for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
                 "--gpus %d is not supported, use --gpus 1" % args.gpus)

    import torch
    from paper_2603_09555_amd import inputs, measure, ssd

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    dev = "cuda"
    log = lambda *a: print(*a, file=sys.stderr, flush=True)

    def preheat(fn):
        """Repeats fn (a call that only enqueues) until --preheat-ms of wall time have passed."""
        t_end = time.perf_counter() + args.preheat_ms * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(8):
                fn()
            torch.cuda.synchronize()

    def shape_of(cfg):
        return ssd.make_shape(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups,
                              cfg.chunk, cfg.torch_io_dtype)

    def time_prefill(cfg, steps, warmup, with_decode=True, profile=True):
        """Times `steps` whole steps; then the same number of profiled steps for per-kernel times."""
        inp = inputs.make_prefill_inputs(cfg, seed=0, device=dev)
        nxt = inputs.make_decode_inputs(cfg, 1, seed=0, device=dev)
        nxt = {k: v[0].contiguous() for k, v in nxt.items()}
        y = torch.empty_like(inp["x"])
        st = torch.empty((cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
        yd = torch.empty_like(nxt["x"])
        ws = torch.empty((max(ssd.prefill_workspace_bytes(shape_of(cfg)), 256),), dtype=torch.uint8, device=dev)

        def step(profile=None):
            if profile is None:
                ssd.ssd_prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], cfg.chunk, y=y,
                                final_state=st, workspace=ws)
            else:  # the measurement library's copy of the same call, an event after every kernel
                profile.extend(measure.prefill_profile(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"],
                                                       cfg.chunk, y, st, ws))
            if with_decode:
                ssd.ssd_decode_step(st, nxt["x"], nxt["dt"], inp["A"], nxt["B"], nxt["C"], inp["D"], y=yd)

        preheat(step)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        kern = {}
        for _ in range(steps if profile else 0):
            prof = []
            step(profile=prof)
            for name, kms in prof:
                kern.setdefault(name, []).append(kms)
        torch.cuda.synchronize()
        kern = {k: sum(v) / len(v) for k, v in kern.items()}
        return ms, kern, inp

    def time_step_cold(cfg, reps=9, dirty=True):
        """The same step with the caches overwritten before every call (512 MiB of unrelated dirty data:
        twice the memory-side cache), timed per call with events; the median.  The back-to-back loop above
        finds part of x cached from the step before, as a layer finds the x its convolution just wrote;
        this is the other end of the range."""
        inp = inputs.make_prefill_inputs(cfg, seed=0, device=dev)
        nxt = {k: v[0].contiguous() for k, v in inputs.make_decode_inputs(cfg, 1, seed=0, device=dev).items()}
        y = torch.empty_like(inp["x"])
        st = torch.empty((cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
        yd = torch.empty_like(nxt["x"])
        ws = torch.empty((max(ssd.prefill_workspace_bytes(shape_of(cfg)), 256),), dtype=torch.uint8, device=dev)
        junk = torch.empty((512 << 20,), dtype=torch.uint8, device=dev)
        evs = []
        for i in range(reps + 2):
            if dirty:
                junk.fill_(i & 1)       # the caches end up full of modified lines that must be written back
            else:
                junk.sum()              # read only: the caches end up full of unrelated clean lines
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ssd.ssd_prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], cfg.chunk, y=y,
                            final_state=st, workspace=ws)
            ssd.ssd_decode_step(st, nxt["x"], nxt["dt"], inp["A"], nxt["B"], nxt["C"], inp["D"], y=yd)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in evs[2:])
        return ts[len(ts) // 2]

    def prefill_report(cfg, ms, kern):
        fl_c, fl_d = prefill_flops(cfg, True), prefill_flops(cfg, False)
        tot_c, tot_d = sum(fl_c.values()), sum(fl_d.values())
        path = ssd.prefill_path(shape_of(cfg))
        peak = PEAK_MFMA_BF16_TFLOPS if path == "mfma_bf16" else PEAK_VALU_F32_TFLOPS
        ai = tot_c / prefill_bytes(cfg)
        attainable = min(peak, ai * PEAK_HBM_GBS / 1e3)
        return dict(workload=cfg.name, path=path, ms=ms, tflops_causal=tot_c / ms / 1e9,
                    tflops_dense=tot_d / ms / 1e9, frac_of_peak=tot_c / ms / 1e9 / peak, peak_tflops=peak,
                    frac_of_attainable=tot_c / ms / 1e9 / attainable,
                    hbm_gbs_compulsory=prefill_bytes(cfg) / ms / 1e6,
                    kernels_ms={k: round(v, 5) for k, v in kern.items()})

    if args.calibrate_copy_mib > 0:
        # a copy of known size: its FETCH_SIZE / WRITE_SIZE readings give the counters' scale
        src = torch.empty((args.calibrate_copy_mib << 20,), dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ---- measured machine peaks (the library's own probe kernels), for scale -------------------
    peaks = {}
    if not args.no_peaks:
        pa = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).fill_(1)
        pb = torch.empty_like(pa)
        for kind in ("copy", "read", "write", "copy_nt", "read_nt", "write_nt"):
            rate, ms = measure.peak_probe(kind, pa, pb, reps=10)
            peaks["stream_%s_gbs" % kind] = round(rate / 1e9, 1)
        for label, iters in (("short", 300), ("long", 4000)):
            rate, ms = measure.peak_probe("mfma", pa, None, iters=iters, reps=3)
            peaks["mfma_bf16_tflops_%s" % label] = round(rate / 1e12, 1)
            peaks["mfma_%s_ms" % label] = round(ms, 3)
        for kind, label in (("mfma_f32", "mfma_f32_32x32x2_tflops"), ("mfma_f32_16x16x4", "mfma_f32_16x16x4_tflops")):
            rate, ms = measure.peak_probe(kind, pa, None, iters=1000, reps=3)
            peaks[label] = round(rate / 1e12, 1)
        log("[bench] measured peaks: %s" % peaks)
        del pa, pb
        torch.cuda.empty_cache()

    # ---- headline: the timed step --------------------------------------------------------
    cfg = inputs.CONFIGS[args.workload]
    log("[bench] workload %s, path %s" % (cfg.name, ssd.prefill_path(shape_of(cfg))))
    ms_step, kern, _ = time_prefill(cfg, args.steps, args.warmup)
    head = prefill_report(cfg, ms_step, kern)
    log("[bench] %s: %.3f ms/step, %.1f TFLOP/s (causal count), kernels %s" %
        (cfg.name, ms_step, head["tflops_causal"], head["kernels_ms"]))
    head["cold_cache_ms"] = round(time_step_cold(cfg), 5)
    head["cold_cache_tflops_causal"] = round(sum(prefill_flops(cfg, True).values()) / head["cold_cache_ms"] / 1e9, 1)
    log("[bench] %s with the caches overwritten before every step: %.3f ms/step, %.1f TFLOP/s" %
        (cfg.name, head["cold_cache_ms"], head["cold_cache_tflops_causal"]))
    head["cold_clean_cache_ms"] = round(time_step_cold(cfg, dirty=False), 5)
    log("[bench] %s with the caches filled with unrelated clean data before every step: %.3f ms/step" %
        (cfg.name, head["cold_clean_cache_ms"]))

    # roofline of the dominant kernel of the step
    dom = max(kern, key=kern.get)
    fl_c = prefill_flops(cfg, True)
    dom_flops = sum(fl_c[k] for k in KERNEL_WORK.get(dom, ()))
    if head["path"] == "mfma_bf16":
        bound, peak = "mfma", PEAK_MFMA_BF16_TFLOPS
    else:
        bound, peak = "alu", PEAK_VALU_F32_TFLOPS
    achieved = dom_flops / kern[dom] / 1e9
    roofline = dict(bound=bound, kernel=dom, achieved=round(achieved, 3), peak=peak, unit="TFLOP/s",
                    frac=round(achieved / peak, 5), traffic=read_traffic().get((cfg.name, dom)),
                    kernel_ms=round(kern[dom], 5), flops_per_launch=dom_flops)
    # the whole prefill call (every kernel of it) beside its dominant kernel: the metric is the prefill
    kern_total = sum(kern.values())
    tot_c = sum(fl_c.values())
    roofline["prefill"] = dict(
        kernels_ms=round(kern_total, 5), tflops_causal=round(tot_c / kern_total / 1e9, 1),
        frac_of_peak=round(tot_c / kern_total / 1e9 / peak, 5),
        frac_of_attainable=round(tot_c / kern_total / 1e9 / min(peak, tot_c / prefill_bytes(cfg) * PEAK_HBM_GBS / 1e3), 5),
        step_frac_of_peak=round(head["frac_of_peak"], 5), step_frac_of_attainable=round(head["frac_of_attainable"], 5),
        cold_cache_step_frac_of_peak=round(head["cold_cache_tflops_causal"] / peak, 5),
        note="kernels_ms: sum of the call's kernels by events; step_*: the timed step (prefill + one decode step)")
    if bound == "mfma" and dom == "chunk_scan":
        # what the kernel actually issues: 38 v_mfma_f32_32x32x16_bf16 per wave and 64-token block, two waves
        # per 64-column head slice (confirmed by SQ_INSTS_MFMA, profiles/prefill_c3_sq_counters.txt)
        nblk = (cfg.seqlen + 63) // 64
        waves = cfg.batch * cfg.nheads * (cfg.headdim // 64) * 2 * ((cfg.dstate + 127) // 128)
        roofline["executed_mfma_flops_per_launch"] = 38 * 32768 * nblk * waves
        roofline["executed_tflops"] = round(38 * 32768 * nblk * waves / kern[dom] / 1e9, 1)
    if peaks.get("mfma_bf16_tflops_long") and bound == "mfma":
        roofline["peak_measured"] = peaks["mfma_bf16_tflops_long"]
        roofline["frac_of_measured"] = round(achieved / peaks["mfma_bf16_tflops_long"], 5)

    # ---- the other prefill configurations (reported, not the headline) -------------------------
    extra = {}
    if not args.no_extra_configs:
        for name in ("c0_tiny_f32", "c1_130m", "c2_780m_b8", "c3_2p7b_long"):
            if name == cfg.name:
                continue
            c = inputs.CONFIGS[name]
            ms, k, _ = time_prefill(c, max(5, args.steps // 2), 2, with_decode=False)
            extra[name] = prefill_report(c, ms, k)
            log("[bench] %s: %.4f ms, %.1f TFLOP/s causal" % (name, ms, extra[name]["tflops_causal"]))
            torch.cuda.empty_cache()

    # ---- chunk-length and group-count sweeps at the headline shape (not measured by the paper) -----
    sweeps = {}
    if not args.no_extra_configs and cfg.headdim == 64 and cfg.dstate == 128:
        for label, c in [("chunk_%d" % L, cfg.with_(chunk=L)) for L in (64, 128, 256, 512, 1024)] + \
                        [("ngroups_%d" % G, cfg.with_(ngroups=G)) for G in (4, 20) if cfg.nheads % (4 * G) == 0] + \
                        [("headdim_128", cfg.with_(headdim=128, nheads=cfg.nheads // 2)),
                         ("dstate_64", cfg.with_(dstate=64)), ("dstate_256", cfg.with_(dstate=256))]:
            ms, k, _ = time_prefill(c, max(5, args.steps // 4), 2, with_decode=False)
            rep = prefill_report(c, ms, k)
            sweeps[label] = dict(path=rep["path"], ms=round(ms, 5), tflops_causal=round(rep["tflops_causal"], 1),
                                 tflops_dense=round(rep["tflops_dense"], 1))
            log("[bench] sweep %s (%s): %.4f ms, %.1f TFLOP/s causal" % (label, rep["path"], ms, rep["tflops_causal"]))
            torch.cuda.empty_cache()

    # ---- the library's choice of segment length on shapes its cost model was not fitted to -------------
    # (the model's constants come from the three bf16 benchmark shapes).  For each shape: the time with the
    # library's own choice, and with forced lengths around it; a choice more than 10 % behind the best
    # forced length is a miss.
    segment_model = {}
    if not args.no_segment_model and not args.no_extra_configs:
        unseen = [("b2_t8192_h32", cfg.with_(batch=2, seqlen=8192, nheads=32)),
                  ("b1_t32768_h16", cfg.with_(batch=1, seqlen=32768, nheads=16)),
                  ("b4_t4096_h64", cfg.with_(batch=4, seqlen=4096, nheads=64)),
                  ("b4_t2048_h128", cfg.with_(batch=4, seqlen=2048, nheads=128)),
                  ("b1_t16384_h8", cfg.with_(batch=1, seqlen=16384, nheads=8)),
                  ("b16_t1024_h48", cfg.with_(batch=16, seqlen=1024, nheads=48)),
                  ("b1_t8192_h24_p128", cfg.with_(batch=1, seqlen=8192, nheads=24, headdim=128)),
                  ("b3_t3000_h20", cfg.with_(batch=3, seqlen=3000, nheads=20))]
        for label, c in unseen:
            nblk = (c.seqlen + 63) // 64
            ms0, _, _ = time_prefill(c, 40, 5, with_decode=False, profile=False)
            forced = {}
            for blocks in sorted({nblk, max(4, nblk // 2), max(4, nblk // 4), max(4, nblk // 8), max(4, nblk // 16), 8, 4}):
                if blocks > nblk:
                    continue
                ssd.set_knob("seg_blocks", blocks)
                forced[blocks], _, _ = time_prefill(c, 40, 5, with_decode=False, profile=False)
            ssd.set_knob("seg_blocks", 0)
            # the library's own choice once more, after the forced ones: the first leg on a new shape also pays
            # for first touches of fresh allocations; the better of the two is its figure
            ms0 = min(ms0, time_prefill(c, 40, 5, with_decode=False, profile=False)[0])
            best = min(forced, key=forced.get)
            segment_model[label] = dict(batch=c.batch, seqlen=c.seqlen, nheads=c.nheads, headdim=c.headdim,
                                        chosen_ms=round(ms0, 5), best_forced_blocks=best,
                                        best_forced_ms=round(forced[best], 5),
                                        forced_ms={str(k): round(v, 5) for k, v in forced.items()},
                                        behind_best=round(ms0 / forced[best] - 1.0, 4), miss=bool(ms0 > 1.05 * forced[best]))
            log("[bench] segment model %s: chosen %.4f ms, best forced %d blocks %.4f ms (%+.1f %%)" %
                (label, ms0, best, forced[best], 100 * (ms0 / forced[best] - 1)))
            torch.cuda.empty_cache()

    # ---- ragged batches and piecewise prompts (same token count and head shape as the headline) -----
    varlen = {}
    if not args.no_varlen and head["path"] == "mfma_bf16" and cfg.batch == 1:
        import numpy as np
        inp = inputs.make_prefill_inputs(cfg, seed=0, device=dev)
        pk = {k: (v[0] if k in ("x", "dt", "B", "C") else v) for k, v in inp.items()}
        T = cfg.seqlen
        y = torch.empty_like(pk["x"])

        def ragged_lengths(nseq, seed):
            """nseq lengths summing to T: log-uniform over a 64x range, rounded, the rest to the longest."""
            r = np.random.default_rng(seed)
            w = np.exp(r.uniform(0.0, np.log(64.0), nseq))
            ln = np.maximum(1, np.floor(w / w.sum() * T).astype(np.int64))
            ln[np.argmax(ln)] += T - ln.sum()
            return ln

        for label, lens in (("1x%d" % T, np.array([T])), ("16_ragged", ragged_lengths(16, 7)),
                            ("64_ragged", ragged_lengths(64, 8)), ("256x64", np.full(T // 64, 64))):
            cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
            nseq = len(lens)
            st = torch.empty((nseq, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
            shp = ssd.make_shape(nseq, T, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk,
                                 cfg.torch_io_dtype)
            ws = torch.empty((ssd.raw().ssd_prefill_varlen_workspace_bytes(shp),), dtype=torch.uint8, device=dev)
            run = lambda: ssd.ssd_prefill_varlen(pk["x"], pk["dt"], pk["A"], pk["B"], pk["C"], pk["D"], cu, cfg.chunk,
                                                 y=y, final_state=st, workspace=ws)
            preheat(run)
            for _ in range(3):
                run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                run()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            fl = sum(sum(prefill_flops(cfg.with_(seqlen=int(n)), True).values()) for n in lens if n > 0)
            varlen[label] = dict(nseq=nseq, min_len=int(lens.min()), max_len=int(lens.max()), ms=round(ms, 5),
                                 tflops_causal=round(fl / ms / 1e9, 1))
            log("[bench] varlen %s: %.4f ms, %.1f TFLOP/s causal" % (label, ms, fl / ms / 1e9))
            del ws, st
        # the headline prompt fed in four pieces, each continuing from the state the previous one left
        pieces = 4
        Tp = T // pieces
        st = torch.zeros((1, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
        cfgp = cfg.with_(seqlen=Tp)
        ws = torch.empty((max(ssd.prefill_workspace_bytes(shape_of(cfgp)), 256),), dtype=torch.uint8, device=dev)
        sl = [{k: inp[k][:, i * Tp:(i + 1) * Tp].contiguous() for k in ("x", "dt", "B", "C")} for i in range(pieces)]
        yp = torch.empty_like(sl[0]["x"])

        def run_pieces():
            for i in range(pieces):
                ssd.ssd_prefill(sl[i]["x"], sl[i]["dt"], inp["A"], sl[i]["B"], sl[i]["C"], inp["D"], cfg.chunk,
                                h0=None if i == 0 else st, y=yp, final_state=st, workspace=ws)
        preheat(run_pieces)
        for _ in range(3):
            run_pieces()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_pieces()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        varlen["continuation_4x%d" % Tp] = dict(pieces=pieces, ms=round(ms, 5),
                                                tflops_causal=round(sum(prefill_flops(cfg, True).values()) / ms / 1e9, 1))
        log("[bench] prompt in %d pieces with carried state: %.4f ms" % (pieces, ms))
        del inp, pk, y, sl, yp, ws, st
        torch.cuda.empty_cache()

    # ---- the depthwise convolution in front of the core, at the headline shape ---------------------
    conv = {}
    if not args.no_conv:
        k = 4
        split = (cfg.nheads * cfg.headdim, cfg.ngroups * cfg.dstate, cfg.ngroups * cfg.dstate)
        C = sum(split)
        io = cfg.torch_io_dtype
        g = torch.Generator(device=dev)
        g.manual_seed(4321)
        u = torch.randn((cfg.batch, cfg.seqlen, C), generator=g, device=dev).to(io)
        wgt = torch.randn((C, k), generator=g, device=dev) / k
        bia = 0.1 * torch.randn((C,), generator=g, device=dev)
        for _ in range(3):
            ssd.ssd_conv1d_prefill(u, wgt, bia, None, split=split)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        # outputs are allocated by the binding; allocate once outside the timed region instead
        outs = [torch.empty((cfg.batch, cfg.seqlen, w_), dtype=io, device=dev) for w_ in split]
        cache = torch.empty((cfg.batch, C, k - 1), dtype=io, device=dev)
        import ctypes as _ct
        i3 = (_ct.c_int32 * 3)(*split)
        vp = lambda t: _ct.c_void_p(t.data_ptr())
        call = lambda: ssd.raw().ssd_conv1d_prefill(cfg.batch, cfg.seqlen, k, 1 if io == torch.bfloat16 else 0, i3, vp(u),
                                                    vp(wgt), vp(bia), None, vp(outs[0]), vp(outs[1]), vp(outs[2]),
                                                    vp(cache), 1, _ct.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert call() == 0
        preheat(call)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.steps
        nbytes = 2 * u.numel() * u.element_size()
        zc = torch.empty_like(u)  # a plain device copy of the same tensor, for scale
        preheat(lambda: zc.copy_(u))
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            zc.copy_(u)
        e1.record()
        torch.cuda.synchronize()
        copy_us = e0.elapsed_time(e1) * 1e3 / args.steps
        del zc
        conv["prefill"] = dict(copy_same_size_us=round(copy_us, 2), batch=cfg.batch, seqlen=cfg.seqlen, channels=C, ksize=k, us=round(us, 2),
                               bytes=nbytes, hbm_gbs=round(nbytes / us / 1e3, 1),
                               frac_of_hbm_peak=round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4))
        log("[bench] conv1d prefill (%d x %d channels): %.1f us, %.0f GB/s" % (cfg.seqlen, C, us, nbytes / us / 1e3))
        # the pair as a layer runs it: the convolution's outputs are the core's x, B and C
        pin = inputs.make_prefill_inputs(cfg, seed=0, device=dev)
        xv = outs[0].view(cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim)
        Bv = outs[1].view(cfg.batch, cfg.seqlen, cfg.ngroups, cfg.dstate)
        Cv = outs[2].view(cfg.batch, cfg.seqlen, cfg.ngroups, cfg.dstate)
        yp = torch.empty_like(xv)
        stp = torch.empty((cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), dtype=torch.float32, device=dev)
        wsp = torch.empty((max(ssd.prefill_workspace_bytes(shape_of(cfg)), 256),), dtype=torch.uint8, device=dev)

        def pair():
            call()
            ssd.ssd_prefill(xv, pin["dt"], pin["A"], Bv, Cv, pin["D"], cfg.chunk, y=yp, final_state=stp, workspace=wsp)
        preheat(pair)
        for _ in range(3):
            pair()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            pair()
        e1.record()
        torch.cuda.synchronize()
        pair_us = e0.elapsed_time(e1) * 1e3 / args.steps
        conv["prefill"]["conv_then_ssd_prefill_us"] = round(pair_us, 2)
        log("[bench] conv1d prefill followed by ssd_prefill on its outputs: %.1f us" % pair_us)
        # the same pair with the other cache policy for y (the library chooses from the size of x; the
        # test-only knob overrides the choice)
        other = {}
        for pol in ("0", "1", "0", "1"):   # twice each, the better one kept: clocks drift over the legs of a run
            ssd.set_knob("y_stream", int(pol))
            for _ in range(3):
                pair()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                pair()
            e1.record()
            torch.cuda.synchronize()
            other[pol] = min(other.get(pol, 1e30), round(e0.elapsed_time(e1) * 1e3 / args.steps, 2))
        ssd.set_knob("y_stream", -1)
        conv["prefill"]["pair_us_y_stores_cached"] = other["0"]
        conv["prefill"]["pair_us_y_stores_non_temporal"] = other["1"]
        log("[bench] the pair with y stored through the caches %.1f us, non-temporally %.1f us" % (other["0"], other["1"]))
        del u, outs, cache, pin, xv, Bv, Cv, yp, stp, wsp
        torch.cuda.empty_cache()

    # ---- decode: 64 stacked layers, states seeded by a 2048-token prefill, 1024 steps ---------
    decode = {}
    if not args.no_decode:
        for name in ("c4_decode_b16", "c4_decode_b1"):
            c = inputs.CONFIGS[name]
            Ly, nsteps = args.decode_layers, args.decode_steps
            state = torch.empty((Ly, c.batch, c.nheads, c.headdim, c.dstate), dtype=torch.float32, device=dev)
            A = torch.empty((Ly, c.nheads), dtype=torch.float32, device=dev)
            D = torch.empty_like(A)
            ws = torch.empty((max(ssd.prefill_workspace_bytes(shape_of(c)), 256),), dtype=torch.uint8,
                             device=dev)
            ytmp = None
            for l in range(Ly):
                inp = inputs.make_prefill_inputs(c, seed=0, layer=l, device=dev)
                if ytmp is None:
                    ytmp = torch.empty_like(inp["x"])
                ssd.ssd_prefill(inp["x"], inp["dt"], inp["A"], inp["B"], inp["C"], inp["D"], c.chunk, y=ytmp,
                                final_state=state[l], workspace=ws)
                A[l], D[l] = inp["A"], inp["D"]
            torch.cuda.synchronize()
            del ytmp, ws, inp
            # per-step inputs for all layers: (steps, Ly, Bt, ...)
            g = torch.Generator(device=dev)
            g.manual_seed(1234)
            io = c.torch_io_dtype
            xs = torch.randn((nsteps, Ly, c.batch, c.nheads, c.headdim), generator=g, device=dev,
                             dtype=torch.float32).to(io) if c.batch == 1 else None
            if xs is None:  # batch 16: 10.7 GB in bf16; draw per step block to bound the fp32 temporary
                xs = torch.empty((nsteps, Ly, c.batch, c.nheads, c.headdim), dtype=io, device=dev)
                for i in range(0, nsteps, 64):
                    xs[i:i + 64] = torch.randn((min(64, nsteps - i),) + tuple(xs.shape[1:]), generator=g,
                                               device=dev, dtype=torch.float32).to(io)
            dts = torch.nn.functional.softplus(
                0.5 * torch.randn((nsteps, Ly, c.batch, c.nheads), generator=g, device=dev) + inputs.DT_BIAS
            ).clamp_(inputs.DT_MIN, inputs.DT_MAX)
            Bs = (inputs.BC_SCALE * torch.randn((nsteps, Ly, c.batch, c.ngroups, c.dstate), generator=g,
                                                device=dev)).to(io)
            Cs = (inputs.BC_SCALE * torch.randn((nsteps, Ly, c.batch, c.ngroups, c.dstate), generator=g,
                                                device=dev)).to(io)
            yd = torch.empty((Ly, c.batch, c.nheads, c.headdim), dtype=io, device=dev)
            for i in range(3):
                ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=yd)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(9)]
            e0.record()
            for i in range(nsteps):
                if i % (nsteps // 8 or 1) == 0 and i // (nsteps // 8 or 1) < 9:
                    marks[i // (nsteps // 8 or 1)].record()
                ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=yd)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / nsteps
            nmarks = min(9, (nsteps + (nsteps // 8 or 1) - 1) // (nsteps // 8 or 1))
            eighths = [marks[i].elapsed_time(marks[i + 1]) * 1e3 / (nsteps // 8 or 1) for i in range(nmarks - 1)]
            bytes_step = decode_bytes(c, Ly)
            gbs = bytes_step / us / 1e3
            decode[name] = dict(layers=Ly, batch=c.batch, steps=nsteps, us_per_step=round(us, 3),
                                bytes_per_step=bytes_step, hbm_gbs=round(gbs, 1),
                                frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4),
                                gflops=round(decode_flops(c, Ly) / us / 1e3, 1),
                                us_per_step_by_eighth=[round(v, 3) for v in eighths],
                                state_bytes=state.numel() * 4,
                                note=("state (%.0f MB) fits the 256 MB Infinity Cache: not a pure HBM figure"
                                      % (state.numel() * 4 / 1e6)) if state.numel() * 4 < 256e6 else
                                "state streams from HBM")
            log("[bench] decode %s: %.2f us/step, %.0f GB/s (%.1f%% of HBM peak)" %
                (name, us, gbs, 100 * gbs / PEAK_HBM_GBS))
            # the other cache policy for the state (the library streams it past the caches when the states
            # of a call exceed the memory-side cache; the test-only knob overrides that)
            for pol, key in (("0", "us_per_step_state_cached"), ("1", "us_per_step_state_non_temporal")):
                ssd.set_knob("decode_stream", int(pol))
                nshort = min(nsteps, 64)
                for i in range(3):
                    ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=yd)
                torch.cuda.synchronize()
                e0.record()
                for i in range(nshort):
                    ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=yd)
                e1.record()
                torch.cuda.synchronize()
                decode[name][key] = round(e0.elapsed_time(e1) * 1e3 / nshort, 3)
            ssd.set_knob("decode_stream", -1)
            log("[bench] decode %s: state through the caches %.2f us/step, non-temporal %.2f us/step" %
                (name, decode[name]["us_per_step_state_cached"], decode[name]["us_per_step_state_non_temporal"]))
            # the same stacked launches replayed from a HIP graph (the launch work done once), and all
            # steps of a block in ONE launch with the state kept on chip between the steps
            nb = min(nsteps, args.decode_block)
            us_graph = None
            if not args.no_graph:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    with torch.cuda.graph(graph, stream=side):
                        for i in range(nb):
                            ssd.ssd_decode_step_layers(state, xs[i], dts[i], A, Bs[i], Cs[i], D, y=yd)
                torch.cuda.current_stream().wait_stream(side)
                graph.replay()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(max(1, nsteps // nb)):
                    graph.replay()
                e1.record()
                torch.cuda.synchronize()
                us_graph = e0.elapsed_time(e1) * 1e3 / (max(1, nsteps // nb) * nb)
                del graph
            nrep = max(1, nsteps // nb)
            ys_blk = torch.empty((nb, Ly, c.batch, c.nheads, c.headdim), dtype=io, device=dev)
            ssd.ssd_decode_steps_layers(state, xs[:nb], dts[:nb], A, Bs[:nb], Cs[:nb], D, y=ys_blk)
            torch.cuda.synchronize()
            e0.record()
            for k in range(nrep):
                o = (k * nb) % (nsteps - nb + 1)
                ssd.ssd_decode_steps_layers(state, xs[o:o + nb], dts[o:o + nb], A, Bs[o:o + nb], Cs[o:o + nb], D,
                                            y=ys_blk)
            e1.record()
            torch.cuda.synchronize()
            us_fused = e0.elapsed_time(e1) * 1e3 / (nrep * nb)
            io_b = 2 if c.io_dtype == "bf16" else 4
            fused_bytes = (2 * 4 * state.numel() / nb + Ly * c.batch * (2 * c.nheads * c.headdim * io_b +
                                                                       4 * c.nheads + 2 * c.ngroups * c.dstate * io_b))
            decode[name].update(
                graph_us_per_step=None if us_graph is None else round(us_graph, 3),
                graph_hbm_gbs=None if us_graph is None else round(bytes_step / us_graph / 1e3, 1), steps_per_graph=nb,
                multi_step=dict(steps_per_launch=nb, us_per_step=round(us_fused, 3),
                                speedup_vs_stacked=round(us / us_fused, 2),
                                bytes_per_step=int(fused_bytes), hbm_gbs=round(fused_bytes / us_fused / 1e3, 1),
                                gflops=round(decode_flops(c, Ly) / us_fused / 1e3, 1),
                                bound="alu", peak_tflops=PEAK_VALU_F32_TFLOPS,
                                frac_of_fp32_valu_peak=round(decode_flops(c, Ly) / us_fused / 1e6 / PEAK_VALU_F32_TFLOPS, 4),
                                frac_of_non_packed_fp32_peak=round(decode_flops(c, Ly) / us_fused / 1e6 / PEAK_VALU_F32_NON_PACKED, 4)))
            log("[bench] decode %s: graph replay %s us/step; %d steps per launch %.2f us/step (%.1fx)" %
                (name, "-" if us_graph is None else "%.2f" % us_graph, nb, us_fused, us / us_fused))
            del ys_blk
            if c.batch == 1:
                # per-layer launches (64 per step), the host-driven analogue
                n2 = min(nsteps, 128)
                torch.cuda.synchronize()
                e0.record()
                for i in range(n2):
                    for l in range(Ly):
                        ssd.ssd_decode_step(state[l], xs[i, l], dts[i, l], A[l], Bs[i, l], Cs[i, l], D[l], y=yd[l])
                e1.record()
                torch.cuda.synchronize()
                us2 = e0.elapsed_time(e1) * 1e3 / n2
                decode[name]["per_layer_launch_us_per_step"] = round(us2, 2)
                decode[name]["per_layer_launch_hbm_gbs"] = round(bytes_step / us2 / 1e3, 1)
            del state, xs, dts, Bs, Cs, yd
            torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample of the headline workload --
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ssd_oracle
        cores = ssd_oracle.max_threads()
        hc = inputs.make_prefill_inputs(cfg, seed=0)  # host copy of the headline workload
        flops_per_pair = sum(prefill_flops(cfg.with_(batch=1, nheads=1), True).values())
        # nheads=1 would count C.B^T once per head; remove it and add the group's share
        sc = prefill_flops(cfg.with_(batch=1, nheads=1), True)["scores"]
        flops_per_pair = flops_per_pair - sc + sc * cfg.ngroups / cfg.nheads
        all_pairs = [(b, h) for b in range(cfg.batch) for h in range(cfg.nheads)]
        probe = all_pairs[:cores]
        pa = ssd_oracle.gather_pairs(hc["x"], hc["dt"], hc["A"], hc["B"], hc["C"], hc["D"], None, probe)
        t0 = time.perf_counter()
        ssd_oracle.scan_pairs(*pa)
        t_probe = time.perf_counter() - t0
        rounds = int(max(1, min(len(all_pairs) // cores, args.cpu_seconds / max(t_probe, 1e-3))))
        sample = all_pairs[:rounds * cores]
        pa = ssd_oracle.gather_pairs(hc["x"], hc["dt"], hc["A"], hc["B"], hc["C"], hc["D"], None, sample)
        # the sample is scanned repeatedly until about --cpu-seconds of CPU work has been timed
        t_cpu, reps = 0.0, 0
        while t_cpu < args.cpu_seconds and reps < 200:
            t0 = time.perf_counter()
            ssd_oracle.scan_pairs(*pa)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cpu = dict(value=round(flops_per_pair * len(sample) * reps / t_cpu / 1e12, 6), unit="TFLOP/s", cores=cores,
                   kind="oracle", seconds=round(t_cpu, 2),
                   sample="%d of %d (batch,head) sequences of %s, all %d tokens each, scanned %d times; fp64 token "
                          "recurrence; same algorithmic FLOP count as the GPU figure" % (len(sample), len(all_pairs),
                                                                                       cfg.name, cfg.seqlen, reps))
        log("[bench] cpu oracle: %.4f TFLOP/s on %d threads (%.1f s)" % (cpu["value"], cores, t_cpu))
        # the oracle's decode step on the batch-1 decode workload (64 layers, state streamed from DRAM in
        # fp64), a few steps: the like-for-like CPU figure for the decode GB/s
        import numpy as np
        c4 = inputs.CONFIGS["c4_decode_b1"]
        Ly = min(args.decode_layers, 64)
        r = np.random.default_rng(5)
        st = r.standard_normal((Ly, c4.batch, c4.nheads, c4.headdim, c4.dstate))
        xs = r.standard_normal((Ly, c4.batch, c4.nheads, c4.headdim))
        dts = r.uniform(1e-3, 1e-1, (Ly, c4.batch, c4.nheads))
        Al = -r.uniform(1, 16, (Ly, c4.nheads))
        Dl = r.standard_normal((Ly, c4.nheads))
        Bl = 0.25 * r.standard_normal((Ly, c4.batch, c4.ngroups, c4.dstate))
        Cl = 0.25 * r.standard_normal((Ly, c4.batch, c4.ngroups, c4.dstate))
        ssd_oracle.decode_step_layers(st, xs, dts, Al, Bl, Cl, Dl)
        t0 = time.perf_counter()
        nst = 3
        for _ in range(nst):
            _, st = ssd_oracle.decode_step_layers(st, xs, dts, Al, Bl, Cl, Dl)
        t_dec = (time.perf_counter() - t0) / nst
        cpu["decode"] = dict(layers=Ly, batch=c4.batch, steps=nst, us_per_step=round(t_dec * 1e6, 1),
                             state_gbs_fp64=round(2 * 8 * st.size / t_dec / 1e9, 2),
                             note="fp64 state read and written once per step, as the oracle stands (it also "
                                  "copies the state once per layer and step)")
        log("[bench] cpu oracle decode: %.0f us/step, %.1f GB/s of fp64 state" % (t_dec * 1e6, 2 * 8 * st.size / t_dec / 1e9))

    out = {
        "metric": "ssd_prefill_tflops", "value": round(head["tflops_causal"], 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.io_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "seqlen": cfg.seqlen, "nheads": cfg.nheads,
                   "headdim": cfg.headdim, "dstate": cfg.dstate, "ngroups": cfg.ngroups, "chunk": cfg.chunk,
                   "step": "ssd_prefill + one ssd_decode_step", "flop_count": "algorithmic, causal-only",
                   "preheat_ms": args.preheat_ms},
        "prefill": head, "roofline": roofline, "cpu_baseline": cpu, "decode": decode, "other_configs": extra,
        "varlen": varlen, "sweeps": sweeps, "segment_model": segment_model, "conv": conv, "measured_peaks": peaks,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
