"""Host-side checks of bench.py's contract (no GPU): the one-GPU rule, the roofline roll-up from
per-site records, and the committed counter summaries it reads."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_1302_1690_amd import workloads as wl  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_roofline_roll_up():
    """Two matrix sites and the two pool sites: the dominant site is the one with the most time, its peak
    follows its instruction, achieved = sum of flops / sum of durations, the pool entry sums both kernels."""
    stats = [
        dict(name="conv_fwd_mfma", layer=2, launches=4, ms_total=4.0, flops=100e9, bytes=1e9),
        dict(name="conv_fwd_mfma", layer=4, launches=4, ms_total=8.0, flops=200e9, bytes=1e9),
        dict(name="wgrad_bm", layer=2, launches=4, ms_total=2.0, flops=500e9, bytes=1e9),
        dict(name="maxfilter_fwd", layer=1, launches=4, ms_total=1.0, flops=0.0, bytes=1e9),
        dict(name="maxfilter_bwd", layer=1, launches=4, ms_total=1.0, flops=0.0, bytes=2e9),
        dict(name="class_layer", layer=9, launches=0, ms_total=0.0, flops=0.0, bytes=0.0),
    ]
    roofs, by_name = bench.rooflines(stats, steps=4, ms_per_step=5.0, workload="no_such_workload")
    r = roofs["roofline"]
    assert r["kernel"] == "conv_fwd_mfma" and r["peak"] == bench.PEAK_FP32_MFMA and r["bound"] == "mfma"
    want = (4 * 100e9 + 4 * 200e9) / 12e-3 / 1e12
    assert abs(r["achieved"] - want) < 1e-3 and abs(r["frac"] - want / bench.PEAK_FP32_MFMA) < 1e-4
    assert r["launches_per_step"] == 2 and r["traffic"] is None
    assert r["all_matrix_sites"]["wgrad_bm"]["frac"] == round(4 * 500e9 / 2e-3 / 1e12 / bench.PEAK_BF16_MFMA, 4)
    h = roofs["roofline_hbm"]
    assert h["bound"] == "hbm" and h["peak"] == bench.PEAK_HBM
    assert abs(h["achieved"] - (4 * 1e9 + 4 * 2e9) / 2e-3 / 1e9) < 0.1
    assert "class_layer" not in by_name


def test_committed_counter_summaries_cover_the_benched_sites():
    """profiles/traffic_<workload>.txt: one line per launch site with the HBM-side bytes per launch; the
    headline's matrix sites and the pool sites must be there, and near or above the algorithmic bytes."""
    for idx in (1, 2, 3, 4):
        cfg = wl.CONFIGS[idx]
        path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % cfg.name)
        assert os.path.exists(path), path
        for site in ("maxfilter_fwd", "maxfilter_bwd", "conv_fwd_bm" if cfg.dtype == "bf16" else "conv_fwd_mfma"):
            v = bench.read_traffic(path, site)
            assert v is not None and v > 0, (path, site)
    assert bench.read_traffic(os.path.join(ROOT, "profiles", "no_such_file.txt"), "x") is None


def test_every_profile_names_its_command():
    """A summary under profiles/ states the rocprofv3 command that made it (committed files only)."""
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        text = open(os.path.join(ROOT, "profiles", name)).read()
        if name.startswith("traffic_"):
            assert "derived from hbm_traffic_" in text, name
            continue
        assert "rocprofv3" in text and "bench.py" in text, name
        assert "_work" not in text, name
