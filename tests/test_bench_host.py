"""Host-side parts of bench.py (no GPU): the one-GPU rule, the algorithmic work it prices the kernels with, and the
readers of the committed rocprofv3 summaries that fill `roofline.traffic` and the matrix-core counters."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_work_is_the_stated_formulas():
    sys.path.insert(0, ROOT)
    import bench
    p, q, r = 4096, 11008, 512
    w = bench.algorithmic_work([(p, q, r)])
    assert w["down"] == dict(bytes=2 * p * q + 4 * p * r + 4 * r * q, flops=2 * p * q * r)        # bf16 G, Q, g out
    assert w["adam"] == dict(bytes=24 * r * q, flops=0)                                            # g, u, v in; u, v, N out
    assert w["up"] == dict(bytes=8 * p * q + 4 * p * r + 4 * r * q, flops=2 * p * q * r)          # W read and written, Q, N
    assert w["outer"] == dict(bytes=24 * p * q, flops=0)                                           # Delta, anchor, b in; b, W, anchor out
    b16 = bench.algorithmic_work([(p, q, r)], w_bytes=2)
    assert w["up"]["bytes"] - b16["up"]["bytes"] == 4 * p * q and w["outer"]["bytes"] - b16["outer"]["bytes"] == 2 * p * q
    ef = bench.algorithmic_work([(p, q, r)], ef=True, qhm_full=True)
    assert ef["down"]["bytes"] - w["down"]["bytes"] == 4 * p * q                                   # the residual is read
    assert ef["up"]["flops"] == 2 * w["up"]["flops"]                                               # residual launch and weight launch
    two = bench.algorithmic_work([(p, q, r), (q, p, r)])
    assert two["up"]["flops"] == 2 * w["up"]["flops"]


def test_committed_counter_summaries_are_read():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2602_04396_amd import synth
    shapes = synth.config_shapes("c4", None)
    work = bench.algorithmic_work(shapes)
    traffic = bench.measured_traffic("c4", None, "up")
    assert traffic is not None and work["up"]["bytes"] < traffic < 2 * work["up"]["bytes"]          # L2-boundary traffic: operand re-reads on top
    assert bench.measured_traffic("c4", None, "up", update="global") is None                         # no summary for that variant
    for kc in ("up", "down"):
        c = bench.measured_mfma_counters("c4", None, kc)
        assert 0.4 < c["mfma_busy_frac_of_elapsed_cycles"] < 1.0 and 1.0 < c["clock_GHz"] <= 2.4
    assert bench.measured_mfma_counters("c2", None, "up") == {}
    assert bench.measured_mfma_counters("c5", 1024, "up")["clock_GHz"] > 1.0
