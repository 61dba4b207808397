"""bench.py's contract with the driver: one JSON line with the agreed keys, and a refusal of
more than one GPU (this build has no sharded path)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, BENCH], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


@pytest.mark.gpu
@pytest.mark.parametrize("config,bound,unit", [("cfg3_mixtral_decode", "hbm", "GB/s"),
                                               ("cfg4_finegrained", "mfma", "TFLOP/s")])
def test_bench_prints_one_json_line_with_the_contract_keys(config, bound, unit):
    r = subprocess.run([sys.executable, BENCH, "--config", config, "--steps", "3", "--warmup", "1",
                        "--cpu-sample-tokens", "8"], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config", "roofline",
                "cpu_baseline"):
        assert key in d, key
    assert d["metric"] == "moe_layer_tokens_per_sec" and d["unit"] == "tokens/s"
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["config"]["workload"] == config and "model" not in d["config"]
    assert d["value"] == pytest.approx(d["config"]["tokens"] / (d["ms_per_step"] * 1e-3), rel=1e-6)
    rf = d["roofline"]
    assert rf["bound"] == bound and rf["unit"] == unit
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], rel=1e-9)
    assert 0 < rf["frac"] < 1 and rf["kernel_ms"] > 0
    lr = d["layer_roofline"]                       # the same bound over the whole step
    assert lr["bound"] == bound and lr["unit"] == unit and 0 < lr["frac"] < 1
    assert lr["frac"] == pytest.approx(lr["achieved"] / lr["peak"], rel=1e-9)
    assert rf["traffic"] is None or rf["traffic"] > 0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["value"] > 0 and cb["cores"] >= 1
    assert "sample" in cb and "8" in cb["sample"]
    assert set(d["measured_ceilings"]) == {"mfma_bf16_constant_operands_tflops",
                                           "mfma_bf16_random_operands_tflops", "hbm_read_gbs",
                                           "hbm_read_nontemporal_gbs"}


@pytest.mark.gpu
def test_bench_options_show_up_in_the_config_it_reports():
    r = subprocess.run([sys.executable, BENCH, "--config", "cfg3_mixtral_decode", "--steps", "3", "--warmup", "1",
                        "--mask", "random", "--weight-layout", "row_major", "--no-cpu-baseline", "--no-ceilings"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip())
    c = d["config"]
    assert c["mask"] == "random" and c["weight_layout"] == "row_major" and c["local_experts"] == 5
    assert 0 <= c["tokens_with_a_remote_slot"] <= c["tokens"]
    assert c["n_local"] + c["n_remote"] == c["tokens"] * c["top_k"]
    assert "cpu_baseline" not in d and "measured_ceilings" not in d


@pytest.mark.gpu
def test_bench_with_another_batch_size_says_so():
    r = subprocess.run([sys.executable, BENCH, "--config", "cfg3_mixtral_decode", "--tokens", "100", "--steps", "3",
                        "--warmup", "1", "--no-cpu-baseline", "--no-ceilings"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip())
    assert d["config"]["tokens"] == 100 and "100 tokens" in d["config"]["workload"]
    assert d["roofline"]["bound"] == "hbm" and d["roofline"]["traffic"] is None
    assert d["value"] == pytest.approx(100 / (d["ms_per_step"] * 1e-3), rel=1e-6)


@pytest.mark.gpu
def test_default_run_carries_both_halves_of_the_metric():
    """No --config: the prefill batch is the line's value, the decode batch of the same layer sits
    under `decode`, each with the dominant kernel's and the whole layer's roofline fraction."""
    r = subprocess.run([sys.executable, BENCH, "--steps", "3", "--warmup", "1", "--cpu-sample-tokens", "8",
                        "--no-ceilings"], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["config"]["workload"] == "cfg2_mixtral_prefill" and d["steps"] == 3
    assert d["roofline"]["bound"] == "mfma" and d["layer_roofline"]["bound"] == "mfma"
    assert d["value"] == pytest.approx(4096 / (d["ms_per_step"] * 1e-3), rel=1e-6)
    dec = d["decode"]
    assert dec["workload"] == "cfg3_mixtral_decode" and dec["config"]["tokens"] == 32
    assert dec["config"]["weight_copies_rotated"] == 4
    for key in ("roofline", "layer_roofline"):
        assert dec[key]["bound"] == "hbm" and dec[key]["unit"] == "GB/s" and 0 < dec[key]["frac"] < 1
    assert dec["layer_roofline"]["achieved"] == pytest.approx(
        dec["layer_roofline"]["algorithmic_bytes_per_step"] / (dec["ms_per_step"] * 1e-3) / 1e9, rel=1e-6)
    assert dec["tokens_per_s"] == pytest.approx(32 / (dec["ms_per_step"] * 1e-3), rel=1e-6)


@pytest.mark.gpu
def test_migration_workload_reports_every_phase():
    base = [sys.executable, BENCH, "--config", "cfg5_dsv2lite_migration", "--steps", "3", "--warmup", "1",
            "--no-cpu-baseline", "--no-ceilings"]
    r = subprocess.run(base, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip())
    ph = d["phases"]
    assert [p["workload"] for p in ph] == ["cfg5_dsv2lite_migration phase 0", "cfg5_dsv2lite_migration phase 1"]
    for p in ph:
        c = p["config"]
        assert sum(p["counts"]) == 8192 * 6 and c["n_local"] + c["n_remote"] == 8192 * 6
        assert c["remote_bytes_each_way"] == c["n_remote"] * 2048 * 2
        assert p["tokens_per_s"] == pytest.approx(8192 / (p["ms_per_step"] * 1e-3), rel=1e-6)
    assert ph[0]["counts"] != ph[1]["counts"]                     # the popularity ranking was reshuffled
    total_ms = sum(p["ms_per_step"] for p in ph) * 3
    assert d["value"] == pytest.approx(2 * 8192 * 3 / (total_ms * 1e-3), rel=1e-6)
    assert d["migration"] == {"experts_admitted": 16, "experts_evicted": 16,
                              "bytes_loaded": 16 * 3 * 2048 * 1408 * 2, "changed_entries_eq3": 32}
    r = subprocess.run(base + ["--phase", "1"], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    one = json.loads(r.stdout.strip())
    assert "phases" not in one and one["config"]["workload"] == "cfg5_dsv2lite_migration"
    assert one["config"]["n_remote"] == ph[1]["config"]["n_remote"]
