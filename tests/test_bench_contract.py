"""bench.py's host-side contract, checked without a GPU: the one-GPU rule, the
algorithmic byte counts it divides by, and the rule that counter-measured HBM
traffic is reported only for the kernel sources it was measured on."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2410_15651_amd import workloads as wl  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_are_the_stated_formulas():
    # log-prob/KL: two logit rows per position, the token id and two fp32 results
    assert bench.logprob_bytes(131072, 128256, 2) == 131072 * (2 * 128256 * 2 + 12) == 67_244_654_592
    assert bench.logprob_bytes(1024, 50272, 4) == 1024 * (2 * 50272 * 4 + 12)
    # decode attention: K and V of every cached token once, q in and out once, a page id per page, a length per row
    cfg = wl.config(5)
    lens = np.array([16, 17, 1, 4096] + [0] * (cfg.batch - 4), dtype=np.int32)
    kv = 2 * int(lens.sum()) * cfg.n_kv_heads * cfg.head_dim * 2
    qo = 2 * cfg.batch * cfg.n_q_heads * cfg.head_dim * 2
    ids = 4 * (1 + 2 + 1 + 256) + 4 * cfg.batch
    assert bench.attention_bytes(lens, cfg) == kv + qo + ids
    # append of one token per sequence: its K and V rows read and written
    assert bench.append_bytes(cfg) == 2 * 2 * cfg.batch * cfg.n_kv_heads * cfg.head_dim * 2


def test_measured_traffic_holds_only_for_the_sources_it_was_taken_on(tmp_path, monkeypatch, capsys):
    good = bench.sources_hash("decode_attn")
    prof = tmp_path / "traffic.txt"
    prof.write_text("some header\n"
                    f"traffic decode_attn workload=5 bytes=1624689530 sha256={good}\n"
                    f"traffic logprob_kl workload=5 bytes=7 sha256={'0' * 64}\n")
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(prof))
    assert bench.measured_traffic("decode_attn", 5) == 1624689530
    assert bench.measured_traffic("decode_attn", 4) is None          # a workload the summary does not cover
    capsys.readouterr()
    assert bench.measured_traffic("logprob_kl", 5) is None           # other sources: said on stderr, not silently
    assert "has changed since its HBM counters were taken" in capsys.readouterr().err
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic("decode_attn", 5) is None
    assert "is missing" in capsys.readouterr().err


def test_the_hash_covers_every_source_a_kernel_is_built_from():
    for name, files in bench.TRAFFIC_SOURCES.items():
        for f in files:
            assert os.path.exists(os.path.join(ROOT, "paper_2410_15651_amd", "csrc", f)), (name, f)
    # an edit to a shared header changes every kernel's hash
    assert "device_ops.h" in bench.TRAFFIC_SOURCES["logprob_kl"]
    assert "device_ops.h" in bench.TRAFFIC_SOURCES["decode_attn"]
    assert "device_ops.h" in bench.TRAFFIC_SOURCES["prefill_attn"]
