"""Decode and quantise timings over the grid of supported shapes.

``python -m paper_2508_04257_amd.shape_sweep [--pairs 256] [--n 4096]`` prints two markdown
tables (per-channel and per-token Keys): bit width x group size x query heads per KV head, for a
cache of ``pairs`` (sequence, KV head) pairs of ``n`` tokens each, i.e. the same cache bytes in
every row of one bit width.  Calls run back to back over three rotating caches (every stream
comes from HBM); the percentage is algorithmic bytes / time against 8 TB/s, so a shape whose heads
take several launches - each streams the codes again - shows a low figure by construction.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as kb
from . import pipeline, synth
from .traffic import decode_algorithmic_bytes, quantize_algorithmic_bytes

HBM_PEAK = 8e12
SLOTS = 3


def _time(fn, iters):
    for i in range(6):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e-3          # seconds per call


def measure(bits, group, rep, key_per_token, pairs, n, dev="cuda:0"):
    """(decode seconds, quantise seconds, decode bytes, quantise bytes, launches' splits)."""
    Hkv = 32 // rep
    w = synth.Workload("sweep", B=pairs // Hkv, n=n, Hq=32, Hkv=Hkv, bits=bits, group=group, k_sinks=5,
                       key_per_token=key_per_token)
    hidden, q = synth.make_hidden(w, dev), synth.make_query(w, dev)
    bufs, kvs = [], []
    for s in range(SLOTS):
        K, V = synth.make_kv(w, dev, layer=s)
        b = pipeline.alloc_step(w, dev)
        pipeline.run_step(w, hidden, K, V, q, b)
        bufs.append(b)
        kvs.append((K, V))
    t_dec = _time(lambda i: pipeline.decode(q, bufs[i % SLOTS]), 60)
    t_qnt = _time(lambda i: pipeline.quantize(kvs[i % SLOTS][0], kvs[i % SLOTS][1], bufs[i % SLOTS]), 30)
    out = (t_dec, t_qnt, decode_algorithmic_bytes(w, w.keep_cap), quantize_algorithmic_bytes(w),
           kb.kvs_decode_splits(bufs[0].desc))
    del bufs, kvs
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--pairs", type=int, default=256, help="(sequence, KV head) pairs; a multiple of 32")
    ap.add_argument("--n", type=int, default=4096, help="tokens per sequence; a multiple of 128")
    ap.add_argument("--shape", default=None, metavar="BITS,G,HEADS,PER_TOKEN",
                    help="time one shape only, e.g. 4,128,8,0")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("the sweep needs a GPU")
    if args.shape:
        bits, group, rep, kpt = (int(x) for x in args.shape.split(","))
        t_dec, t_qnt, b_dec, b_qnt, splits = measure(bits, group, rep, bool(kpt), args.pairs, args.n)
        print(f"bits {bits} G {group} heads per KV head {rep} per-token Keys {kpt}: decode {t_dec * 1e6:.1f} us "
              f"({100 * b_dec / t_dec / HBM_PEAK:.1f} % of 8 TB/s, {splits} part(s)), quantise {t_qnt * 1e6:.1f} us "
              f"({100 * b_qnt / t_qnt / HBM_PEAK:.1f} %)")
        return
    for kpt in (False, True):
        print(("Per-token Keys" if kpt else "Per-channel Keys") +
              f", {args.pairs} (sequence, KV head) pairs x {args.n} tokens; decode: time, % of 8 TB/s\n")
        print("| bits | G | Hq/Hkv = 1 | 2 | 4 | 8 | quantise |")
        print("|---|---|---|---|---|---|---|")
        for bits in (2, 3, 4, 8):
            for group in (32, 64, 128):
                cells, qs = [], []
                for rep in (1, 2, 4, 8):
                    t_dec, t_qnt, b_dec, b_qnt, _ = measure(bits, group, rep, kpt, args.pairs, args.n)
                    cells.append(f"{t_dec * 1e6:.0f} us, {100 * b_dec / t_dec / HBM_PEAK:.0f} %")
                    qs.append((t_qnt * 1e6, 100 * b_qnt / t_qnt / HBM_PEAK))
                print(f"| {bits} | {group} | " + " | ".join(cells) +
                      f" | {min(t for t, _ in qs):.0f}-{max(t for t, _ in qs):.0f} us, "
                      f"{min(p for _, p in qs):.0f}-{max(p for _, p in qs):.0f} % |", flush=True)
        print()


if __name__ == "__main__":
    main()
