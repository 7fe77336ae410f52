"""Host-side pieces of bench.py (no GPU): the byte model, the figures derived per projection, and the counter
summaries under profiles/ that roofline.traffic is read from."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2603_02599_amd import workloads as wl  # noqa: E402


def test_algorithmic_bytes_of_the_headline_workload():
    work = wl.make_workload("cfg2")
    a = bench.algorithmic_bytes(work.shape, work, None)
    s = work.shape
    # weights once (bf16), every cached position's K and V once, the new entries, embedding rows, fp32 logits
    weights = (s.n_layers * (s.hidden * (s.q_dim + 2 * s.kv_dim) + s.q_dim * s.hidden + 3 * s.hidden * s.ffn) + s.vocab * s.hidden) * 2
    kv = int((work.seq_lens.astype(np.int64) + 1).sum()) * 2 * s.n_layers * s.kv_dim * 2
    assert a["weights"] == weights and a["kv_read"] == kv
    assert a["kv_write"] == work.batch * 2 * s.n_layers * s.kv_dim * 2
    assert abs(a["total"] - 33.19e9) < 0.02e9
    q = bench.algorithmic_bytes(s, work, "asym")
    assert abs(q["weights"] - (s.body_params * 0.53125 + s.vocab * s.hidden * 2)) < 1 and q["kv_read"] == kv
    assert bench.w4_bytes_per_weight("sym_noz") == 0.515625


def test_traffic_figures_come_from_the_profiles():
    for name, tokens in (("cfg2", 138411), ("cfg3", 459145)):
        t = bench.measured_traffic_bytes(name, None)
        assert t is not None and 1.0 < t / (tokens * 4096) < 1.2       # a little above the algorithmic bytes
        assert wl.make_workload(name).kv_tokens_read == tokens
    assert bench.measured_traffic_bytes("cfg2", "asym") is None        # not counted: reported as null
    assert bench.measured_traffic_bytes("small", None) is None


def test_projection_figures():
    work = wl.make_workload("cfg3")
    kernels = {"gate_up_proj": {"avg_us": 100.0}, "lm_head": {"avg_us": 500.0}}
    bench.projection_figures(work.shape, work, None, kernels)
    g = kernels["gate_up_proj"]
    n, k = 2 * work.shape.ffn, work.shape.hidden
    assert abs(g["TFLOPs"] - 2.0 * 256 * n * k / 100e-6 / 1e12) < 1e-6
    assert abs(g["frac_of_mfma_peak"] - g["TFLOPs"] / 2500.0) < 1e-12 and g["mfma_operands"] == "bf16"
    assert abs(g["weight_GBps"] - n * k * 2 / 100e-6 / 1e9) < 1e-6 and g["bound"] == "hbm"
    kq = {"gate_up_proj": {"avg_us": 100.0}, "lm_head": {"avg_us": 500.0}}
    bench.projection_figures(work.shape, work, "asym", kq)
    assert kq["gate_up_proj"]["mfma_operands"] == "int8" and kq["gate_up_proj"]["bound"] == "mfma"
    assert abs(kq["gate_up_proj"]["frac_of_mfma_peak"] - g["TFLOPs"] / 5000.0) < 1e-12
    assert kq["lm_head"]["mfma_operands"] == "bf16"                    # stays dense (Appendix A.1)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
