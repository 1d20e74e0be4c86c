"""Host-side parts of the benchmark's contract (no GPU): the one-GPU rule, the FLOP accounting, the
profile summary it reads, and that nothing of the product path reaches into the oracle."""
import ast
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2407_09105_amd import workloads as wl  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and p.stdout.strip() == ""
    assert "ONE GPU" in p.stderr and "--gpus 2" in p.stderr


def test_flop_accounting_counts_unmasked_pairs():
    # useful FLOPs: 4d forward + 10d backward per unmasked (i, j) pair and query head, pairs = sum L(L+1)/2
    w = wl.make_workload(1, tensors=False)
    assert w.stats["pairs"] == sum(L * (L + 1) // 2 for L in (3, 5, 1, 7))
    f, b = bench.flops(w.cfg, w.stats["pairs"])
    assert f == 4 * w.cfg.d * w.cfg.hq * w.stats["pairs"] and b == 10 * w.cfg.d * w.cfg.hq * w.stats["pairs"]
    w2 = wl.make_workload(2, tensors=False)
    assert w2.cfg.n_tokens == 8192 and sum(w2.lengths[0]) == 8192
    assert w2.stats["pairs"] == sum(L * (L + 1) // 2 for L in w2.lengths[0])


def test_roofline_bound_follows_algorithmic_intensity():
    # configs 2 and 5: the slowest kernel (dK/dV) lies above the ridge of 2500 TFLOP/s over 8 TB/s -> MFMA-bound,
    # quoted in TFLOP/s; config 4 (examples of 8..128 tokens) lies far below it -> HBM-bound, quoted in GB/s
    stages = {"pack": 0.01, "fwd": 0.1, "bwd_dQ": 0.15, "bwd_dKdV": 0.25}
    for cfg_id, bound, unit, peak in ((2, "mfma", "TFLOP/s", 2500.0), (5, "mfma", "TFLOP/s", 2500.0), (4, "hbm", "GB/s", 8000.0)):
        w = wl.make_workload(cfg_id, tensors=False)
        r = bench.roofline_of(w.cfg, w.stats["pairs"], stages, cfg_id)
        assert (r["kernel"], r["bound"], r["unit"], r["peak"]) == ("dkdv_mfma_kernel", bound, unit, peak)
        assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
        c, pairs = w.cfg, w.stats["pairs"]
        assert r["algorithmic_flops"] == 8 * c.d * c.hq * pairs
        # Q, dO read; K, V read; dK, dV written (2 bytes each); LSE and D read (4 bytes each)
        assert r["algorithmic_bytes"] == c.n_tokens * (2 * c.d * (2 * c.hq + 4 * c.hkv) + 8 * c.hq)
        want = r["algorithmic_flops"] / 0.25e-3 / 1e12 if bound == "mfma" else r["algorithmic_bytes"] / 0.25e-3 / 1e9
        assert abs(r["achieved"] - want) < 1e-9 * want
    # the three kernels' FLOPs add up to the useful FLOPs of the step
    w = wl.make_workload(2, tensors=False)
    work = bench.algorithmic_work(w.cfg, w.stats["pairs"])
    assert sum(f for f, _ in work.values()) == sum(bench.flops(w.cfg, w.stats["pairs"]))


def test_traffic_summary_is_parsed(tmp_path, monkeypatch):
    # bench.py reads "<kernel>: <bytes> ..." lines from profiles/hbm_traffic_cfgN.txt; the parser is checked on a
    # file written here (the tracked summaries are measurements: the test only asks that they parse)
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "hbm_traffic_cfg7.txt").write_text("header line\nfwd_mfma_kernel: 123456 bytes/launch  (read 0.1 MB)\n"
                                               "dq_mfma_kernel: not-a-number\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.read_traffic(7, "fwd_mfma_kernel") == 123456.0
    assert bench.read_traffic(7, "dq_mfma_kernel") is None
    assert bench.read_traffic(7, "no_such_kernel") is None and bench.read_traffic(8, "fwd_mfma_kernel") is None
    monkeypatch.undo()
    for cfg_id in (2, 3, 4, 5):
        for kernel in ("fwd_mfma_kernel", "dq_mfma_kernel", "dkdv_mfma_kernel"):
            t = bench.read_traffic(cfg_id, kernel)
            assert t is not None and t > 0, (cfg_id, kernel)


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2407_09105_amd")
    for name in os.listdir(pkg):
        if not name.endswith(".py"):
            continue
        tree = ast.parse(open(os.path.join(pkg, name)).read())
        for node in ast.walk(tree):
            mods = []
            if isinstance(node, ast.Import):
                mods = [a.name for a in node.names]
            elif isinstance(node, ast.ImportFrom):
                mods = [node.module or ""]
            assert not any(m == "oracle" or m.startswith("oracle.") for m in mods), name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        text = open(os.path.join(pkg, "csrc", name)).read()
        assert "oracle" not in text.lower(), name
    # and the oracle imports nothing of the package
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c")):
            assert "paper_2407_09105_amd" not in open(os.path.join(ROOT, "oracle", name)).read(), name


def test_padded_layout_groups_of_four():
    lay = wl.padded_layout([[3, 9, 4, 6, 2, 8]], group=4)
    assert lay == [(3, 9), (9, 9), (4, 9), (6, 9), (2, 8), (8, 8)]
    assert np.sum([p for _, p in lay]) == 52
