"""Host-side contract of bench.py that needs no GPU: more than one GPU is refused with a message, and the
stored hardware-counter traffic is tied to the kernel sources it was measured with."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_is_reported_only_for_the_sources_it_was_measured_with(monkeypatch):
    b = _bench_module()
    assert len(b.TRAFFIC_GEMM_STORE["sources_sha256"]) == 64
    monkeypatch.setattr(b, "kernel_sources_digest", lambda: b.TRAFFIC_GEMM_STORE["sources_sha256"])
    t = b.measured_traffic("gemm_store_kernel")
    assert t == b.TRAFFIC_GEMM_STORE["read_bytes"] + b.TRAFFIC_GEMM_STORE["write_bytes"] and 1e9 < t < 1e11
    assert b.measured_traffic("lmhead_fwd_kernel") is None              # counters were taken for one kernel only
    monkeypatch.setattr(b, "kernel_sources_digest", lambda: "0" * 64)   # the kernel has changed since
    assert b.measured_traffic("gemm_store_kernel") is None
    assert b.PEAK_BF16_TFLOPS == 2500.0
