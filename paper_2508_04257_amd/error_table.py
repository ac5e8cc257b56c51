"""Quantisation-error table with the structure of the paper's Table 1 (Section 4.1), on synthetic
data: MSE x 100 of per-token Keys, per-token Values and per-channel Keys, dynamic (overall, groups
without a sink token, groups with one) and static (overall with the sinks calibrated and
quantised, and with the sinks excluded from both).  Every number comes from the library calls
(kvs_quantize_kv, kvs_calibrate, kvs_static_params, kvs_quantize_kv_static, kvs_quant_error).

    python -m paper_2508_04257_amd.error_table [--group 32]

The paper's figures are measured on LLaMA2-7B activations with group size 16; this prints the same
rows for a seeded synthetic tensor (sink rows suppressed x0.1 except for two extreme entries, Key
outlier channels with a mean far from zero) and group sizes the library supports, as a sanity
analysis of the same effects.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as kb
from . import pipeline, synth


def _mse(r, which):
    sse0, n0, sse1, n1 = r
    if which == "overall":
        return 100.0 * (sse0 + sse1) / max(n0 + n1, 1)
    if which == "without":
        return 100.0 * sse0 / max(n0, 1)
    return 100.0 * sse1 / max(n1, 1)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--group", type=int, default=32)
    args = ap.parse_args()
    dev = "cuda"
    base = synth.Workload("table", B=4, n=2048, Hq=8, Hkv=8, bits=4, group=args.group, k_sinks=2,
                          key_channel_offset=40.0, sink_kv_spike=120.0)
    K, V = synth.make_kv(base, dev)
    sinks = torch.zeros((base.B, base.n), dtype=torch.uint8, device=dev)
    for b, row in enumerate(synth.sink_positions(base)):
        sinks[b, torch.as_tensor(row, device=dev)] = 1
    none = torch.zeros_like(sinks)
    print("| scheme | bits | per-token K: overall | w/o sinks | w/ sinks | per-token V: overall | w/o sinks | w/ sinks "
          "| per-channel K: overall | w/o sinks | w/ sinks |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for static in (False, True):
        for bits in (4, 3, 2):
            cells = {}
            for kpt in (True, False):
                w = base.scaled(bits=bits, key_per_token=kpt)
                desc = pipeline.desc_for(w)
                cache, ws = kb.alloc_cache(desc, dev), kb.alloc_workspace(desc, dev)
                if not static:
                    kb.kvs_quantize_kv(desc, K, V, none, cache, ws)          # the sinks are quantised too
                    r = kb.kvs_quant_error(desc, K, V, cache, sinks)
                    cells[kpt] = {t: [_mse(r[t], c) for c in ("overall", "without", "with")] for t in ("k", "v")}
                else:
                    out = {}
                    for label, mask in (("overall", none), ("without", sinks)):
                        calib = kb.alloc_calibration(desc, dev)
                        kb.kvs_calibrate(desc, K, V, mask, calib)
                        ks, vs = kb.kvs_static_params(desc, calib)
                        kb.kvs_quantize_kv_static(desc, K, V, mask, ks, vs, cache, ws)
                        out[label] = kb.kvs_quant_error(desc, K, V, cache, sinks)
                    cells[kpt] = {t: [_mse(out["overall"][t], "overall"), _mse(out["without"][t], "overall"), None]
                                  for t in ("k", "v")}
            row = cells[True]["k"] + cells[True]["v"] + cells[False]["k"]
            print("| %s | %d | %s |" % ("static" if static else "dynamic", bits,
                                        " | ".join("-" if x is None else "%.3f" % x for x in row)))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
