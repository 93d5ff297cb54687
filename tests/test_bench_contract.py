"""Host-side checks of bench.py that need no GPU: the command line the driver uses, the
refusal of more than one GPU, the pure helpers, and that every --op has a traffic summary
name and a bytes model."""
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", BENCH)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, BENCH, "--gpus", "2", "--steps", "1", "--warmup", "0"],
                          capture_output=True, text=True, cwd=ROOT)
    assert proc.returncode != 0
    assert "single-GPU" in proc.stderr and proc.stdout.strip() == ""


def test_help_lists_the_driver_flags_and_every_op():
    proc = subprocess.run([sys.executable, BENCH, "--help"], capture_output=True, text=True, cwd=ROOT)
    assert proc.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--op", "--profile-only", "--calib-copy", "--paper-shape"):
        assert flag in proc.stdout
    for op in ("rmsnorm", "softmax", "layernorm", "crossentropy", "rowsum"):
        assert op in proc.stdout


def test_trimmed_mean_and_roofline_object():
    b = load_bench()
    assert b.trimmed_mean([1.0] * 8 + [100.0, -100.0]) == 1.0            # 10 % cut from each end
    assert b.trimmed_mean([3.0]) == 3.0
    obj = b.roofline_object(8_000_000, 0.001, [1.0, 1.25, 1.25], traffic=8_100_000.0,
                            traffic_source="profiles/some_summary.txt", extra_field=1)
    assert obj["bound"] == "hbm" and obj["unit"] == "GB/s" and obj["peak"] == 8000.0
    assert obj["achieved"] == pytest.approx(8000.0) and obj["frac"] == pytest.approx(1.0)
    # the back-to-back region's time per launch, under a name that says what it is
    assert obj["region_us_per_launch"] == pytest.approx(1.0) and "kernel_mean_us" not in obj
    # the per-launch event-pair protocol beside it: 10 % trimmed mean and the fraction it gives
    assert obj["event_pair_trimmed_mean_us"] == pytest.approx(3.5 / 3, abs=1e-3)
    assert obj["frac_event_pair"] == pytest.approx(3 / 3.5, abs=1e-3)
    # counter-derived traffic, where it came from, and the rate it gives at this run's time
    assert obj["traffic"] == 8_100_000.0 and obj["traffic_source"] == "profiles/some_summary.txt"
    assert obj["traffic_gbps"] == pytest.approx(8100.0)
    assert obj["extra_field"] == 1
    bare = b.roofline_object(8_000_000, 0.001, [1.0])
    assert bare["traffic"] is None and bare["traffic_source"] is None and bare["traffic_gbps"] is None


def test_the_json_line_names_its_timing_protocol_and_its_settling_launches():
    """Every --op writes config.timing and settle_launches, and no op reaches the measurement
    copy through the RMSNorm library any more."""
    text = open(BENCH).read()
    assert text.count('"timing": "back_to_back_region"') == 5
    assert text.count('"settle_launches": settled') == 5
    assert "rmsnorm_calib_copy" not in text and text.count("measure.measure_copy(") == 5 and "measure.measure_staged_copy" in text
    b = load_bench()
    assert b.traffic_fields("rmsnorm")["traffic_source"] == "profiles/" + b.TRAFFIC_FILES["rmsnorm"]


def test_every_op_has_a_traffic_summary_that_parses():
    b = load_bench()
    assert sorted(b.TRAFFIC_FILES) == ["crossentropy", "layernorm", "rmsnorm", "rowsum", "softmax",
                                       "softmax_attention"]
    for op, name in b.TRAFFIC_FILES.items():
        path = os.path.join(ROOT, "profiles", name)
        assert os.path.exists(path), f"profiles/{name} is missing"
        traffic = b.read_traffic(op)
        assert traffic is not None and traffic > 0
        text = open(path).read()
        algorithmic = float([ln for ln in text.splitlines() if ln.startswith("algorithmic_bytes_per_launch:")][0].split()[1])
        assert 0.99 < traffic / algorithmic < 1.05, (op, traffic, algorithmic)


def test_bytes_models_of_the_benchmark_shapes():
    from paper_2603_21331_amd import inputs
    assert inputs.algorithmic_bytes(16384, 8192, inputs.BF16) == 536887296
    assert inputs.softmax_bytes(8192, 8192, inputs.FP16) == 268435456
    assert inputs.layernorm_bytes(8192, 4096, inputs.FP16) == 134234112
    assert inputs.crossentropy_bytes(8192, 32000, inputs.FP16) == 524288000
    assert inputs.rowsum_bytes(8192, 8192, inputs.FP16) == 134217728
