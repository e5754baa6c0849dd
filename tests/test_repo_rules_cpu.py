"""Host-side checks of the rules the repository keeps: the product never reaches for the oracle or for a CPU
fallback, bench.py names every configuration of the benchmark spec with the shapes it states, and refuses more than one
GPU."""
import importlib.util
import json
import os
import re
import subprocess
import sys

from paper_2601_05524_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def product_sources():
    pkg = os.path.join(ROOT, "paper_2601_05524_amd")
    for d, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                yield os.path.join(d, f)
    for f in os.listdir(os.path.join(ROOT, "include")):
        yield os.path.join(ROOT, "include", f)


def test_product_never_imports_or_names_the_oracle():
    for path in product_sources():
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "dbl_oracle" not in text and "liborc" not in text, path


def test_oracle_never_imports_the_product():
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"^\s*(import|from)\s+paper_2601_05524_amd\b", text, re.M), f
            assert "libdbl.so" not in text and "binding" not in text, f


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2601_05524_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libdbl.so"))
    try:
        B.lib()
    except B.DblError as e:
        assert "no fallback" in str(e)
    else:
        raise AssertionError("binding.lib() returned without a library")


def test_nothing_committed_reaches_into_the_working_folder():
    r = subprocess.run(["git", "ls-files"], cwd=ROOT, capture_output=True, text=True)
    if r.returncode == 0 and r.stdout.strip():
        tracked = r.stdout.split()
        assert not [p for p in tracked if p.startswith("_work/") or p.startswith("gpurun_out/")]
    else:   # a copy of the tree without its history: every source file outside the ignored folders
        tracked = [os.path.relpath(os.path.join(d, f), ROOT) for d, _, fs in os.walk(ROOT) for f in fs
                   if not os.path.relpath(d, ROOT).split(os.sep)[0] in ("_work", "gpurun_out", ".git", ".pytest_cache")]
    for p in tracked:
        if p.endswith((".py", ".h", ".hip", ".c", ".sh")) and p != "tests/test_repo_rules_cpu.py":
            assert "_work/" not in open(os.path.join(ROOT, p)).read(), p


def test_bench_workloads_are_the_baseline_configurations():
    bench = load_bench()
    cfgs = json.load(open(os.path.join(ROOT, "BASELINE.json")))["configs"]
    assert len(cfgs) == 5
    W = bench.WORKLOADS

    def shape(name):
        return synth.CONFIGS[W[name][0]]

    # config 0: the tiny fp32 model, 256-token history, k = 4
    t = shape("tiny_ctx256_k4_b1_greedy")
    assert (t["n_layers"], t["d_model"], t["n_q_heads"], t["n_kv_heads"], t["head_dim"], t["d_ffn"], t["vocab"], t["dtype"]) == \
        (2, 256, 4, 2, 64, 688, 2048, 0)
    assert W["tiny_ctx256_k4_b1_greedy"][1:5] == (256, 4, 1, "greedy")
    # config 1: the 1B-shaped draft model, 1024-token history, k = 8
    s = shape("llama1b_ctx1024_k8_b1_greedy")
    assert (s["n_layers"], s["d_model"], s["n_q_heads"], s["n_kv_heads"], s["head_dim"], s["d_ffn"], s["vocab"], s["dtype"]) == \
        (16, 2048, 32, 8, 64, 8192, 128256, 1)
    assert W["llama1b_ctx1024_k8_b1_greedy"][1:5] == (1024, 8, 1, "greedy")
    # config 2: the 70B-shaped target, 2048 cached tokens, k = 8, greedy -- the configuration the metric is quoted on
    s = shape("llama70b_ctx2048_k8_b1_greedy")
    assert (s["n_layers"], s["d_model"], s["n_q_heads"], s["n_kv_heads"], s["head_dim"], s["d_ffn"], s["vocab"], s["dtype"]) == \
        (80, 8192, 64, 8, 128, 28672, 128256, 1)
    assert W["llama70b_ctx2048_k8_b1_greedy"][1:5] == (2048, 8, 1, "greedy")
    assert "llama70b_ctx2048_k8_b1_greedy" in open(os.path.join(ROOT, "bench.py")).read().split('"--workload", default=')[1][:60]
    # config 3: the 32B-shaped target with q/k-norm, 8192 cached tokens, k = 16, sampling at 0.7
    s = shape("qwen32b_ctx8192_k16_b1_sample")
    assert (s["n_layers"], s["d_model"], s["n_q_heads"], s["n_kv_heads"], s["head_dim"], s["d_ffn"], s["vocab"], s["qk_norm"]) == \
        (64, 5120, 64, 8, 128, 25600, 151936, 1)
    assert W["qwen32b_ctx8192_k16_b1_sample"][1:6] == (8192, 16, 1, "sample", 0.7)
    # config 4: long-context stress, 32768 tokens, batch 4, k in {4, 8, 16, 32}, sampling at 1.0
    for k in (4, 8, 16, 32):
        w = W["llama70b_ctx32768_k%d_b4_sample" % k]
        assert w[0] == "llama70b" and w[1:6] == (32768, k, 4, "sample", 1.0)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
