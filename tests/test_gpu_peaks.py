"""The benchmark aid lococo_measure_peaks on a real GPU."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible():
    """A bare MFMA loop and a plain copy on this GPU land below the published peaks (2.5 PFLOP/s
    bf16, 8 TB/s) and within reach of them; bad arguments are refused."""
    from paper_2406_05317_amd import binding as lb
    scratch = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    tf, gbs = lb.lococo_measure_peaks(scratch)
    print(f"bare MFMA loop {tf:.0f} TFLOP/s, copy {gbs:.0f} GB/s")
    assert 800.0 < tf < 2600.0, tf
    assert 1000.0 < gbs < 8200.0, gbs
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_measure_peaks(scratch[:1 << 20])
    assert e.value.status == lb.LOCOCO_EINVAL
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_measure_peaks(scratch[1:(64 << 20) + 1])
    assert e.value.status == lb.LOCOCO_EINVAL


def test_the_bench_line_keeps_its_contract():
    """`bench.py` on the small target shape, a few steps, as a child process: one JSON line with the fields the
    harness reads, a roofline of the dominant kernel measured with events in the timed region, the oracle timed
    beside it, and the extra figures."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "cfg2", "--steps", "5", "--warmup",
                        "2", "--sustain-seconds", "0.2"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "tokens/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert d["config"]["workload"].startswith("cfg2") and "model" not in d["config"]
    assert abs(d["value"] - 3584 / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["peak"] == 2500.0 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.02 < roof["frac"] < 1.0
    assert roof["kernel"] == "compress_mfma" and roof["launches"] == 5
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    assert d["value"] > 100 * cpu["value"]
    assert d["sustained"]["value"] > 0 and d["hip_graph"]["value"] > 0 and d["measured_peaks"]["mfma_bf16_tflops"] > 0
