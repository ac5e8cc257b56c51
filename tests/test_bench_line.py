"""bench.py's JSON line, assembled on the CPU: the rig that owns the GPU buffers is replaced by a
stand-in with fixed timings, so every side leg fails (there is no GPU here) and the line must still
come out whole, with the contract's keys and each failed leg reported in its place."""
import json
import sys
import types

import pytest

import bench
from paper_2508_04257_amd import pipeline, synth
from paper_2508_04257_amd.traffic import decode_algorithmic_bytes, quantize_algorithmic_bytes


class StandInRig:
    def __init__(self, w, slots, dev):
        self.w, self.slots, self.dev = w, slots, dev
        self.bufs = [types.SimpleNamespace(desc=pipeline.desc_for(w)) for _ in range(slots)]
        self.inputs = [(None, None)] * slots
        self.q = None
        self.nnz = None
        self.dec_bytes = decode_algorithmic_bytes(w, w.keep_cap)
        self.qnt_bytes = quantize_algorithmic_bytes(w)

    def timed_steps(self, steps, warmup):
        return {"ms_step": 0.2, "ms_predict": 0.01, "ms_quant": 0.13, "ms_decode": 0.03,
                "ms_decode_estimates": [0.029, 0.031]}

    def back_to_back(self, reps):
        return 0.028

    def stream_ceiling(self, reps=40):
        return {"ms": 0.0225, "achieved": 0.0, "frac": 0.0, "note": "stand-in"}


@pytest.fixture
def line(monkeypatch, capsys):
    import torch

    def run(*argv):
        monkeypatch.setattr(bench, "Rig", StandInRig)
        monkeypatch.setattr(torch.cuda, "set_device", lambda *_: None)
        monkeypatch.setattr(sys, "argv", ["bench.py", "--no-cpu-baseline", *argv])
        rc = bench.main()
        out = capsys.readouterr().out.strip().splitlines()
        return rc, out
    return run


def test_the_line_survives_every_side_leg_failing(line):
    rc, out = line("--steps", "7", "--warmup", "2")
    assert rc == 0 and len(out) == 1                       # ONE line, nothing else on stdout
    r = json.loads(out[0])
    w = synth.WORKLOADS["cfg1"]
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in r, key
    assert (r["n_gpus"], r["steps"], r["warmup"], r["vs_baseline"], r["data"]) == (1, 7, 2, None, "synthetic")
    assert r["config"]["workload"].startswith("cfg1") and "model" not in r["config"]
    # value = algorithmic bytes / the decode duration the rig reported
    assert r["value"] == pytest.approx(decode_algorithmic_bytes(w, w.keep_cap) / 0.03e-3 / 1e9, rel=1e-4)
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], abs=1e-4)
    assert roof["algorithmic_bytes"] == 143425536
    # the legs had no GPU to run on: each says so where its result would be
    for leg in ("graph_replay", "growing_cache", "static_quantisation", "per_token_keys", "int8"):
        assert "error" in r[leg], leg
    assert set(r["configs"]) == set(bench.OTHER_CONFIGS) - {"cfg1"} >= {"cfg2", "cfg3", "cfg4"}
    assert all(isinstance(v, dict) for v in r["configs"].values())


def test_no_configs_and_the_sparse_workload(line):
    rc, out = line("--workload", "cfg4", "--no-configs")
    r = json.loads(out[0])
    assert rc == 0 and "configs" not in r and "cpu_baseline" not in r
    assert "error" in r["layers32"]
    assert "isolated outliers" in r["roofline"]["kernel"]
    assert r["roofline"]["traffic"] is None                # counters were taken on the headline workload only


def test_more_than_one_gpu_is_refused(line, capsys):
    rc, out = line("--gpus", "2")
    assert rc == 2 and out == []
