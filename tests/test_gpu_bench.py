"""bench.py end to end at reduced sizes: one JSON line with the contract's fields, for both workloads."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*flags):
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, res.stdout[-2000:]
    return json.loads(lines[0])


def check_contract(r):
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["value"] > 0 and r["ms_per_step"] > 0 and "workload" in r["config"]
    rf = r["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3


def test_attention_bench_small():
    r = run_bench("--layers", "2", "--batch", "3", "--kv", "512", "--steps", "3", "--warmup", "1", "--event-stride", "1", "--cpu-seqs", "1")
    check_contract(r)
    assert r["metric"] == "predict_verify_attn_hbm_gbps_b3_kv512"        # the label follows the configuration
    assert r["config"]["workload"].startswith("batch3_kv512_layers2") and "also" not in r
    cb = r["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and 1 <= cb["cores"] <= cb["cores_usable"] <= cb["nproc"]
    assert cb["single_thread"]["cores"] == 1 and cb["single_thread"]["value"] > 0
    rf = r["roofline"]
    assert rf["min_kernel_ms"] <= rf["median_kernel_ms"] and rf["min_kernel_ms"] <= rf["avg_kernel_ms"]
    assert set(rf["plain_read_gbps"]) == {"ordinary", "non_temporal"} and min(rf["plain_read_gbps"].values()) > 0 and rf["frac_of_plain_read"] > 0
    assert cb["gpu_vs_oracle_max_abs"] <= 2e-2 and cb["gpu_vs_oracle_mean_rel"] <= 1e-2 and cb["within_tolerance"] is True
    r = run_bench("--layers", "2", "--batch", "32", "--kv", "8192", "--steps", "2", "--warmup", "1", "--no-cpu-baseline", "--no-also")
    assert r["metric"] == "predict_verify_attn_hbm_gbps_b32_kv8k" and r["roofline"]["traffic"] is not None


def test_read_probe_reads_and_leaves_the_sink_alone():
    """The plain read kernel behind `plain_read_gbps`: any size and both load kinds run, nothing is written."""
    import torch

    from paper_2604_14889_amd import binding as M

    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for nbytes in (16, 4096 + 16, 3 * 256 * 16 * 2048 + 48, 64 << 20):
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda", generator=gen)
        for nt in (False, True):
            assert M.ms_hbm_read_probe(src, nt, sink) == nbytes // 32768 * 32768
    torch.cuda.synchronize()
    assert int(sink.count_nonzero()) == 0
    with pytest.raises(M.MsError):
        M.ms_hbm_read_probe(src[1:17], False, sink)      # not 16-byte aligned


def test_attention_bench_other_paths_small():
    """The host-side commit (accept lengths read back every step) and the fixed tile assignment stay runnable; 16 steps
    take the small caches through a compaction of the 56-token segment."""
    for flag in ("--host-commit", "--deterministic"):
        r = run_bench("--layers", "2", "--batch", "3", "--kv", "512", "--steps", "16", "--warmup", "1", "--event-stride", "1",
                      "--no-cpu-baseline", flag)
        check_contract(r)
    r = run_bench("--workload", "decode_step", "--layers", "1", "--batch", "3", "--kv", "128", "--steps", "2", "--warmup", "1", "--host-commit")
    check_contract(r)


def test_compaction_bench_small():
    r = run_bench("--workload", "compaction", "--layers", "3", "--batch", "4", "--steps", "3", "--warmup", "1")
    check_contract(r)
    cp = r["compaction"]
    assert cp["calls"] == 3 and cp["device_us_per_call"] > 0 and cp["kernel_launches_per_call"] >= 1
    assert cp["kv_row_bytes_written_per_call"] == 4 * 8 * 3 * 4 * 128 * 2 * 2


def test_wide_step_bench_small():
    r = run_bench("--workload", "wide_step", "--layers", "2", "--batch", "2", "--kv", "1000", "--queries", "41", "--steps", "2", "--warmup", "1")
    check_contract(r)
    assert r["kernel_launches_per_call"] == 1.0 and r["roofline"]["kernel"] == "pv_attn_mfma_wide"


def test_decode_step_bench_small():
    r = run_bench("--workload", "decode_step", "--layers", "1", "--batch", "3", "--kv", "128", "--steps", "2", "--warmup", "1")
    check_contract(r)
    assert r["attention_share_of_step"] > 0
    r = run_bench("--workload", "decode_step", "--layers", "1", "--batch", "1", "--kv", "128", "--steps", "2", "--warmup", "1",
                  "--fused-lm-head")
    check_contract(r)


def test_projections_bench_small():
    r = run_bench("--workload", "projections", "--rows", "63", "--steps", "2", "--warmup", "1")
    assert r["roofline"]["bound"] == "mfma" and r["roofline"]["peak"] == 2500.0 and len(r["projections"]) == 5
    assert all(p["us"] > 0 for p in r["projections"]) and r["config"]["workload"] == "qwen2.5-7b_projections_rows63"


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120, cwd=ROOT)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr) or "single" in (res.stdout + res.stderr).lower()
