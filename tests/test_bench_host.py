"""Host-side checks of ``bench.py``: the HBM-traffic figure of the roofline object comes from the committed
counter summary under ``profiles/`` (nothing typed into the script), and the algorithmic FLOP count of the
headline configuration is the closed form of the chunked algorithm."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2603_09555_amd import inputs  # noqa: E402


def test_traffic_comes_from_the_committed_counter_summary(tmp_path):
    t = bench.read_traffic()
    key = ("c3_2p7b_long", "chunk_scan")
    assert key in t, "the headline kernel has no TRAFFIC line in profiles/"
    cfg = inputs.CONFIGS["c3_2p7b_long"]
    xy = 2 * cfg.batch * cfg.seqlen * cfg.nheads * cfg.headdim * 2
    assert xy <= t[key] < 1.5 * xy       # at least x + y, not wildly more
    # the parser: scale factors, malformed lines ignored, a missing file gives an empty table
    f = tmp_path / "s.txt"
    f.write_text("TRAFFIC w k fetch_kib=1.5 write_kib=2\nTRAFFIC broken\nnoise\n")
    assert bench.read_traffic(str(f)) == {("w", "k"): int((2.0 * 1.5 + 2.0) * 1024)}
    assert bench.read_traffic(str(tmp_path / "absent")) == {}


def test_algorithmic_flop_count_of_the_headline_configuration():
    cfg = inputs.CONFIGS["c3_2p7b_long"]
    fl = bench.prefill_flops(cfg, causal=True)
    L, T, H, P, N, G = cfg.chunk, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    k = (L + 1) / (2 * L)
    per_chunk = G * 2 * L * L * N * k + H * (2 * L * L * P * k + 4 * L * P * N) + H * (2 * P * N + 2 * L * P)
    assert abs(sum(fl.values()) - per_chunk * (T // L)) < 1e-6 * per_chunk * (T // L)
    assert 64e9 < sum(fl.values()) < 67e9
