"""bench.py's work model and its reading of the committed profile, without a GPU: the flops and bytes the roofline
fractions are computed from are the per-matrix formulas summed over the workload's shapes (checked here against sums
written out by hand for LLaMA-7B, r = 1024), and the traffic figure comes with the digest of the kernel sources it
was profiled at."""
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2407_08296_amd import inputs as I  # noqa: E402


def test_llama7b_work_per_launch():
    shapes = [(m, n, r) for (_, _, m, n, r) in I.config_matrices(4)]
    assert len(shapes) == 224
    h, f, layers, r = 4096, 11008, 32, 1024
    mn = layers * (4 * h * h + 3 * h * f)                   # weight elements: q, k, v, o; gate, up, down
    rn = layers * r * (4 * h + 2 * h + f)                   # low-rank elements: n = h six times, n = f once
    mr = layers * r * (4 * h + 2 * f + h)                   # projection elements: m = h five times, m = f twice
    assert mn == 6_476_005_376 and rn == 1_166_016_512 and mr == 1_392_508_928
    flops, proj, adam, bp = bench.algorithmic_work(shapes)
    assert flops == 2 * mn * r                              # 13.26 TFLOP per GEMM launch
    assert adam == 22 * rn                                  # R 4, M 4 + 4, V 4 + 4, N 2 bytes per element
    p_bytes = mr // 2 + 4 * (mr // 256)                     # INT4 codes + one fp32 scale per 256 (m*r is a multiple of 256)
    assert proj == 2 * mn + p_bytes + 4 * rn
    assert bp == 2 * mn + 8 * (mn // 256) + p_bytes + 2 * rn     # W codes and scales read and written, P, N
    mfma_ms, hbm_ms = bench.step_bounds(shapes)
    assert abs(mfma_ms - 2 * flops / 2.5e15 * 1e3) < 1e-9
    assert 10.5 < mfma_ms < 10.7 and 6.0 < hbm_ms < 7.6


def test_small_configs_have_their_shapes():
    counts = {0: 1, 1: 84, 2: 168, 3: 168}
    for c, k in counts.items():
        shapes = [(m, n, r) for (_, _, m, n, r) in I.config_matrices(c)]
        assert len(shapes) == k
        flops, proj, adam, bp = bench.algorithmic_work(shapes)
        assert flops == sum(2 * m * n * r for m, n, r in shapes) and adam == sum(22 * r * n for m, n, r in shapes)
    assert [(m, n, r) for (_, _, m, n, r) in I.config_matrices(0)] == [(512, 512, 128)]


def test_committed_traffic_figure_names_the_sources_it_was_profiled_at():
    traffic, stamp = bench.measured_traffic("k_backproject_many", 4)
    assert isinstance(traffic, int) and stamp
    digest, date = stamp.split()[:2]
    assert re.fullmatch(r"[0-9a-f]{12}", digest) and re.fullmatch(r"\d{4}-\d{2}-\d{2}", date)
    assert re.fullmatch(r"[0-9a-f]{12}", bench.kernel_source_digest())
    shapes = [(m, n, r) for (_, _, m, n, r) in I.config_matrices(4)]
    _, _, _, bp = bench.algorithmic_work(shapes)
    assert bp <= traffic <= 2 * bp                          # measured HBM bytes: at least the algorithmic ones
    assert bench.measured_traffic("k_backproject_many", 1) == (None, None)     # only the 7B workload was profiled
