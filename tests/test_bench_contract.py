"""The parts of bench.py's contract that need no GPU: more than one GPU is refused with a message (this build
measures one GPU), the host-only mode prints one JSON line, and the traffic figure is only passed on while the
fingerprint in the committed profile matches the kernel and planner sources."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=600)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_host_only_mode_prints_one_json_line():
    r = run("--only", "simulate")
    assert r.returncode == 0, r.stderr
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["only"] == "simulate" and {"remote", "local", "adaptive"} <= set(d)


def test_traffic_figure_follows_the_source_fingerprint():
    t, note = bench.committed_traffic("attn_kernel_cfg2_prefill_counters.md")
    sha = bench.sources_sha16()
    measured_on_these_sources = sha in open(os.path.join(ROOT, "profiles", "attn_kernel_cfg2_prefill_counters.md")).read()
    assert len(sha) == 16
    if measured_on_these_sources:
        assert t is not None and 5e8 < t < 1e9 and "profiles/" in note
    else:
        assert t is None          # a figure measured on other sources is never passed on
