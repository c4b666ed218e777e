"""Host-side logic of bench.py (no GPU): algorithmic byte counts against the closed forms of the
workload definitions, the workload table against the configurations it stands for, and the refusal
of more than one GPU."""
import json
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _fake(name, lens, stride, paged=False):
    wl = dict(bench.WORKLOADS[name]); wl.update(bench.COMMON)
    return dict(wl=wl, ctx_len=torch.tensor(lens, dtype=torch.int32), stride=stride, paged=paged)


def test_algorithmic_bytes_cfg2_closed_form():
    # batch 32, 32768 tokens, one query token: keys 128 B + one fp32 score per token, queries 64 x (128 + 4) B
    W = _fake("cfg2", [32768] * 32, 1152)
    ab = bench.algorithmic_bytes(W, 0)
    assert ab["index_score"] == 32 * 32768 * 132 + 32 * 64 * 132 == 138_682_368
    assert ab["topk"] == 32 * 32768 * 4 + 32 * 2048 * 4
    assert ab["attention_rows"] == 32 * 2048 * 1152 + 32 * 128 * (576 * 2 + 512 * 2 + 4)
    assert ab["fill"] == 0


def test_algorithmic_bytes_two_tokens_paged_and_fill():
    # two query tokens read every key once and write two scores; paged keys carry a 4-byte scale
    W = _fake("cfg5", [131072] * 128, 656, paged=True)
    ab = bench.algorithmic_bytes(W, 1000.0)
    assert ab["index_score"] == 128 * 131072 * (128 + 4 + 8) + 128 * 2 * 64 * 132
    assert ab["attention_rows"] == 128 * 2 * 2048 * 656 + 128 * 2 * 128 * (576 * 2 + 512 * 2 + 4)
    assert ab["fill"] == 656_000


def test_workload_table_matches_the_configurations():
    cfgs = json.load(open(os.path.join(ROOT, "BASELINE.json")))["configs"]
    want = {"cfg2": ("batch 32", "context 32768"), "cfg3": ("batch 64", "context 32768"),
            "cfg4": ("batch 64", "context 131072"), "cfg5": ("batch 128", "context 131072")}
    for name, (b, ctx) in want.items():
        wl = bench.WORKLOADS[name]
        text = cfgs[wl["cfg"] - 1]
        assert b in text and ctx in text, (name, text)
        assert "batch %d" % wl["B"] == b and "context %d" % wl["L"] == ctx
    assert bench.WORKLOADS["cfg4"]["lens"] == (98304, 131072) and bench.WORKLOADS["cfg4"]["ratio"] == 0.10
    assert bench.WORKLOADS["cfg3"]["ratio"] == 0.25 and bench.WORKLOADS["cfg3"]["rho"] == 0.8
    assert bench.WORKLOADS["cfg5"]["T"] == 2 and bench.WORKLOADS["cfg5"]["layers"] == 61
    assert bench.COMMON["k"] == 2048 and bench.COMMON["H"] == 128 and (bench.COMMON["Hi"], bench.COMMON["Di"]) == (64, 128)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_median_of_step_times():
    assert bench._median([3.0, 1.0, 2.0]) == 2.0
    assert bench._median([4.0, 1.0, 2.0, 3.0]) == 2.5
