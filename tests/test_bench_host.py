"""Host-side checks of bench.py: the byte accounting, the one-GPU rule, and that the committed
profile summaries were measured with the kernel sources in the tree (otherwise bench.py withholds
`roofline.traffic`)."""
import glob
import os
import re
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench                                                   # noqa: E402
from paper_2509_15038_amd import workloads as wl               # noqa: E402


def test_algorithmic_bytes_of_the_headline_step():
    cfg = wl.CONFIGS["c3"]
    b = wl.budgets_for(cfg, 0.1)
    ab = bench.algorithmic_bytes(cfg, b)
    # per head: K and V once (512 n), scores written and read (8 n), indices written and read
    # (8 k), kept rows read and written (1024 k); n = 32768, k = 3276, 256 heads
    per_head = 520 * 32768 + 1032 * 3276
    assert per_head == 20420192
    assert ab["total"] == 256 * per_head == 5227569152
    assert ab["scan"] == 256 * 32768 * 512
    assert ab["scores"] + ab["select"] + ab["compact"] == ab["total"]
    # key-only reads one tensor; fp32 rows are twice as long
    assert bench.algorithmic_bytes(cfg, b, source="k")["scan"] == ab["scan"] // 2
    f32 = wl.scaled(cfg, dtype="fp32")
    assert bench.algorithmic_bytes(f32, b)["scan"] == 2 * ab["scan"]
    assert bench.algorithmic_bytes(f32, b)["compact"] == int(b.astype(np.int64).sum()) * (4 + 2048)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)


def test_profile_summaries_match_the_kernel_sources():
    sha = bench.kernel_sources_sha16()
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md")))
    assert files
    for f in files:
        m = re.search(r"kernel_sources_sha16:\s*([0-9a-f]{16})", open(f).read())
        assert m, f"{os.path.basename(f)} records no kernel_sources_sha16"
        assert m.group(1) == sha, (f"{os.path.basename(f)} was measured with other kernel sources "
                                   f"({m.group(1)}, tree {sha}): re-run the profile passes")


def test_traffic_figures_exist_for_every_workload_of_the_default_run():
    c3 = wl.CONFIGS["c3"]
    heads = c3.layers * c3.kv_heads
    for cfg_name, keep in (("c3", 0.1), ("c3", 0.2), ("c3", 0.5), ("c4", 0.1)):
        fused = keep * 100 <= bench.FUSED_GATHER_MAX_PERCENT
        t, src = bench.measured_traffic(cfg_name, keep, fused, heads)
        assert isinstance(t, int) and t > 0, (cfg_name, keep, src)
        alg = bench.algorithmic_bytes(wl.CONFIGS[cfg_name], wl.budgets_for(wl.CONFIGS[cfg_name], keep))["total"]
        assert 0.97 < t / alg < 1.03, (cfg_name, keep, t, alg)     # no re-reads: traffic = algorithmic bytes
    t, _ = bench.measured_traffic("c5", wl.CONFIGS["c5"].keep[0], False, heads)
    assert isinstance(t, int) and t > 0
