"""Benchmark of the KVSink hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: kvs_predict_sinks on the hidden
state, kvs_decode_attn of one query per sequence and head over a cache, kvs_quantize_kv of one
layer's K and V into a cache.  The step quantises into cache slot i and decodes from slot i + 1
(quantised several steps earlier), and the K/V inputs rotate over distinct copies, so every
stream comes from HBM rather than from the 256 MB last-level cache.  Decode runs between
predict and quantise: it has no data dependence on this step's quantise.

Prints ONE JSON line.  value = effective HBM GB/s of kvs_decode_attn on the headline workload
(algorithmic bytes of the call / its mean duration inside the step); quantize tokens/s is reported
next to it, the other workloads are timed the same way under "configs", and the 32-layer
dense-and-sparse workload under "configs.cfg4.layers32".  Inputs are resident in HBM before the
timed region.  The CPU oracle is timed first, before the GPU is touched.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2508_04257_amd.traffic import decode_algorithmic_bytes, quantize_algorithmic_bytes  # noqa: E402

HBM_PEAK_GBPS = 8000.0
OTHER_CONFIGS = ("cfg0_kvsink", "cfg2", "cfg3", "cfg4")

# HBM bytes per kvs_decode_attn launch on the cfg1 workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE; profiles/pmc_cfg1_hbm_traffic.md), each scaled by what the same counter
# reads for a plain copy of known size.  Valid for the decode kernel's sources whose hash is given:
# once any of them changes the benchmark reports "traffic": null until the counters are taken again.
DECODE_TRAFFIC = {
    "workload": "cfg1",
    "sources": ["decode_mfma_impl.h", "decode_mfma_b4.hip", "decode_finish.h"],
    "sha256_16": "a9fa369b22b50917",
    "fetch_bytes": 144057580,
    "write_bytes": 73728,
}


def measured_decode_traffic(workload_name: str):
    import hashlib
    if workload_name != DECODE_TRAFFIC["workload"] or not DECODE_TRAFFIC["sha256_16"]:
        return None
    h = hashlib.sha256()
    try:
        for f in DECODE_TRAFFIC["sources"]:
            with open(os.path.join(ROOT, "paper_2508_04257_amd", "csrc", f), "rb") as fh:
                h.update(fh.read())
    except OSError:
        return None
    if h.hexdigest()[:16] != DECODE_TRAFFIC["sha256_16"]:
        return None
    return DECODE_TRAFFIC["fetch_bytes"] + DECODE_TRAFFIC["write_bytes"]


class HipEvent:
    """A HIP timing event recorded on torch's current stream (the stream every library call is
    launched on).  Created without the system-scope release fence that a default event carries:
    that fence writes back and invalidates the caches between two kernels and would be charged
    to whichever kernel is being timed."""

    _hip = None
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self):
        import ctypes
        if HipEvent._hip is None:
            HipEvent._hip = ctypes.CDLL("libamdhip64.so")
        self.h = ctypes.c_void_p()
        rc = HipEvent._hip.hipEventCreateWithFlags(ctypes.byref(self.h), HipEvent.DISABLE_SYSTEM_FENCE)
        assert rc == 0, f"hipEventCreateWithFlags failed: {rc}"

    def record(self):
        import ctypes
        import torch
        rc = HipEvent._hip.hipEventRecord(self.h, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, f"hipEventRecord failed: {rc}"

    def elapsed_time(self, other: "HipEvent") -> float:
        import ctypes
        ms = ctypes.c_float()
        rc = HipEvent._hip.hipEventElapsedTime(ctypes.byref(ms), self.h, other.h)
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return float(ms.value)


# ------------------------------------------------------------------------------------------------
# one workload: rotating inputs and caches, the timed steps
# ------------------------------------------------------------------------------------------------
class Rig:
    """Inputs, caches and buffers of one workload on the GPU, `slots` rotating copies of each."""

    def __init__(self, w, slots, dev):
        import torch

        from paper_2508_04257_amd import pipeline, synth

        self.w, self.slots, self.dev = w, slots, dev
        self.hidden = synth.make_hidden(w, dev)
        self.q = synth.make_query(w, dev)
        self.inputs = [synth.make_kv(w, dev, layer=s) for s in range(slots)]
        self.bufs = [pipeline.alloc_step(w, dev) for _ in range(slots)]
        # Fill every cache slot once so that the first timed decode reads real data.
        for s in range(slots):
            pipeline.run_step(w, self.hidden, self.inputs[s][0], self.inputs[s][1], self.q, self.bufs[s])
        torch.cuda.synchronize()
        self.nnz = None
        if w.sparse_frac > 0:                                   # entries the caches really hold
            rows = w.B * w.Hkv * w.n
            c = self.bufs[0].cache
            self.nnz = (int(c.k_rowptr[rows].cpu()), int(c.v_rowptr[rows].cpu()))
        self.dec_bytes = decode_algorithmic_bytes(w, w.keep_cap, self.nnz)
        self.qnt_bytes = quantize_algorithmic_bytes(w, self.nnz)

    def step(self, i, ev=None, mid_after_decode=False):
        """predict -> decode -> quantise.  ev = (start, middle, end) events; the middle one sits
        after predict or after decode (see the timing note in timed_steps)."""
        from paper_2508_04257_amd import pipeline

        cur, old = self.bufs[i % self.slots], self.bufs[(i + 1) % self.slots]
        K, V = self.inputs[i % self.slots]
        if ev:
            ev[0].record()
        pipeline.predict(self.w, self.hidden, cur)
        if ev and not mid_after_decode:
            ev[1].record()
        pipeline.decode(self.q, old)
        if ev and mid_after_decode:
            ev[1].record()
        pipeline.quantize(K, V, cur)
        if ev:
            ev[2].record()

    def timed_steps(self, steps, warmup):
        """Timing note.  A pair of HIP events around ONE launch measures the launch plus what the
        event packets themselves cost (an empty pair reads ~4 us on this machine), so a kernel is
        never bracketed on its own here.  Every step carries three events; the middle one alternates
        between "after predict" and "after decode", and a call's duration is a difference of
        brackets that hold real work only:
          decode   = mean[start -> after decode](odd steps) - mean[start -> after predict](even steps)
                   and mean[after predict -> end](even steps) - mean[after decode -> end](odd steps),
                   averaged (rocprofv3's kernel trace of the same run lies between the two)
          quantise = mean[after decode -> end](odd steps)
          predict  = mean[start -> after predict](even steps)"""
        import torch

        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        events = [[HipEvent() for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i, events[i], mid_after_decode=(i % 2 == 1))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        tagged = [(i % 2 == 1, events[i]) for i in range(steps)]
        while min(sum(k for k, _ in tagged), sum(not k for k, _ in tagged)) < 3:
            # too few timed steps for both kinds of bracket: untimed extra steps supply them
            kind = sum(k for k, _ in tagged) <= sum(not k for k, _ in tagged)
            ev = [HipEvent() for _ in range(3)]
            self.step(warmup + len(tagged), ev, mid_after_decode=kind)
            tagged.append((kind, ev))
        torch.cuda.synchronize()
        even = [e for is_odd, e in tagged if not is_odd]
        odd = [e for is_odd, e in tagged if is_odd]
        mean = lambda xs: sum(xs) / len(xs)
        ms_predict = mean([e[0].elapsed_time(e[1]) for e in even])
        ms_predict_decode = mean([e[0].elapsed_time(e[1]) for e in odd])
        ms_quant = mean([e[1].elapsed_time(e[2]) for e in odd])
        ms_decode_quant = mean([e[1].elapsed_time(e[2]) for e in even])
        front = ms_predict_decode - ms_predict     # the event's own cost falls on the bracket it closes,
        back = ms_decode_quant - ms_quant          # so the two differences err in opposite directions
        for b in self.bufs:
            assert int(b.cache.status.cpu()[0]) == 0, "capacity overflow reported by the library"
        return {"ms_step": 1e3 * (t1 - t0) / max(steps, 1), "ms_predict": ms_predict, "ms_quant": ms_quant,
                "ms_decode": 0.5 * (front + back), "ms_decode_estimates": [front, back]}

    def back_to_back(self, reps):
        """The same decode call back to back over the rotating (cold) caches, one event pair around
        the whole run: no event sits between kernels."""
        import torch

        from paper_2508_04257_amd import pipeline

        b0, b1 = HipEvent(), HipEvent()
        b0.record()
        for i in range(reps):
            pipeline.decode(self.q, self.bufs[i % self.slots])
        b1.record()
        torch.cuda.synchronize()
        return b0.elapsed_time(b1) / reps

    def stream_ceiling(self, reps=40):
        """A pure streaming read of as many bytes as one decode call moves, in the decode kernel's
        launch shape, over rotating cold buffers: what the memory system alone takes."""
        import torch

        from paper_2508_04257_amd import binding as kb

        n = (self.dec_bytes + 15) // 16 * 16
        src = [torch.ones(n, dtype=torch.uint8, device=self.dev) for _ in range(max(self.slots, 4))]
        sink = torch.zeros(4, dtype=torch.int32, device=self.dev)
        for s in src:
            kb.kvs_probe_stream_read(s, sink)
        torch.cuda.synchronize()
        e0, e1 = HipEvent(), HipEvent()
        e0.record()
        for i in range(reps):
            kb.kvs_probe_stream_read(src[i % len(src)], sink)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        return {"ms": round(ms, 4), "achieved": round(n / (ms * 1e-3) / 1e9, 2),
                "frac": round(n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "note": "kvs_probe_stream_read: the same bytes read once with no arithmetic, 256 workgroups x 8 waves, "
                        "back to back over rotating cold buffers"}


def decode_kernel_name(w, splits):
    if w.sparse_frac == 0:
        return ("kvs_decode_attn = decode_mfma_kernel<%d,%d,%d%s>" % (w.bits, w.group, w.Hq // w.Hkv,
                                                                     ",per-token Keys" if w.key_per_token else "")
                + ("" if splits == 1 else " (%d workgroups per (sequence, KV head), the last arriver merges)" % splits))
    return ("kvs_decode_attn = decode_mfma_kernel<%d,%d,%d,isolated outliers>" % (w.bits, w.group, w.Hq // w.Hkv)
            + ("" if splits == 1 else " (%d workgroups per (sequence, KV head), the last arriver merges)" % splits))


def workload_label(w):
    return (f"{w.name}: B={w.B} n={w.n} Hq={w.Hq} Hkv={w.Hkv} D={w.D} INT{w.bits} G={w.group} "
            f"keep=first{w.first_n}+top{w.k_sinks} sparse={w.sparse_frac}")


# ------------------------------------------------------------------------------------------------
# legs beside the headline numbers
# ------------------------------------------------------------------------------------------------
def growing_cache_leg(w, kv, q, dec_bytes):
    """The decoding-phase calls on the same shapes: a cache of capacity n holding n - 64 tokens
    (64 of them in the fp16 residual window), decode over it, then 128 appends (one of which
    completes and quantises a block).  Reported beside the headline numbers, not part of `value`."""
    import torch

    from paper_2508_04257_amd import binding as kb
    from paper_2508_04257_amd import pipeline

    dev = q.device
    K, V = kv
    desc = pipeline.desc_for(w)
    cache, ws = kb.alloc_cache(desc, dev), kb.alloc_workspace(desc, dev)
    n0 = w.n - 64
    mask = torch.zeros((w.B, n0), dtype=torch.uint8, device=dev)
    mask[:, 0] = 1
    kb.kvs_quantize_prefix(desc, K[:, :, :n0].contiguous(), V[:, :, :n0].contiguous(), mask, n0, cache, ws)
    out = torch.empty((w.B, w.Hq, w.D), dtype=torch.float16, device=dev)
    for _ in range(3):
        kb.kvs_decode_attn_n(desc, q, cache, n0, out, None, ws)
    torch.cuda.synchronize()
    reps = 30
    e0, e1 = HipEvent(), HipEvent()
    e0.record()
    for _ in range(reps):
        kb.kvs_decode_attn_n(desc, q, cache, n0, out, None, ws)
    e1.record()
    torch.cuda.synchronize()
    ms_decode = e0.elapsed_time(e1) / reps
    rows = [(K[:, :, t].contiguous(), V[:, :, t].contiguous()) for t in range(n0, w.n)]
    torch.cuda.synchronize()
    e0.record()
    for i, (k1, v1) in enumerate(rows):
        kb.kvs_append_kv(desc, k1, v1, n0 + i, cache, ws)
    e1.record()
    torch.cuda.synchronize()
    ms_append = e0.elapsed_time(e1) / len(rows)
    return {
        "n_tokens": n0, "capacity": w.n, "residual_rows": 64,
        "ms_decode_attn_n": round(ms_decode, 4),
        "decode_gbps": round((dec_bytes * ((n0 // 128) * 128) / w.n + 64 * w.B * w.Hkv * w.D * 4)
                             / (ms_decode * 1e-3) / 1e9, 2),
        "ms_append_kv_mean": round(ms_append, 4),
        "appends_timed": len(rows),
        "note": "decode over n - 64 tokens incl. 64 fp16 residual rows, back to back on one cache (last-level-cache "
                "resident); append = mean over 64 calls issued from Python (one 2 us copy kernel each, so this is the host's launch rate), "
                "the last of which quantises a completed block",
    }


def static_leg(w, inputs, bufs, qnt_bytes):
    """Calibration and fixed-parameter quantisation on the same shapes (rotating inputs and caches),
    reported beside the headline numbers."""
    import torch

    from paper_2508_04257_amd import binding as kb

    desc = bufs[0].desc
    calib = kb.alloc_calibration(desc, inputs[0][0].device)
    slots = len(inputs)
    for i in range(slots):
        kb.kvs_calibrate(desc, inputs[i][0], inputs[i][1], bufs[i].keep_mask, calib)
    ks, vs = kb.kvs_static_params(desc, calib)
    torch.cuda.synchronize()
    reps = 12
    e = [HipEvent() for _ in range(3)]
    e[0].record()
    for i in range(reps):
        kb.kvs_calibrate(desc, inputs[i % slots][0], inputs[i % slots][1], bufs[i % slots].keep_mask, calib)
    e[1].record()
    for i in range(reps):
        kb.kvs_quantize_kv_static(desc, inputs[i % slots][0], inputs[i % slots][1], bufs[i % slots].keep_mask, ks, vs,
                                  bufs[i % slots].cache, bufs[i % slots].workspace)
    e[2].record()
    torch.cuda.synchronize()
    ms_cal, ms_q = e[0].elapsed_time(e[1]) / reps, e[1].elapsed_time(e[2]) / reps
    read = 2 * w.B * w.Hkv * w.n * w.D * 2
    return {
        "ms_calibrate": round(ms_cal, 4), "calibrate_gbps": round(read / (ms_cal * 1e-3) / 1e9, 2),
        "ms_quantize_kv_static": round(ms_q, 4), "quantize_static_gbps": round(qnt_bytes / (ms_q * 1e-3) / 1e9, 2),
        "quantize_static_tokens_per_s": round(w.B * w.n / (ms_q * 1e-3), 1),
    }


def _variant_leg(wv, inputs, bufs, q):
    """Quantise and decode calls of a variant of the workload (same shapes, another scheme) over
    rotating inputs and caches of its own, back to back.  Returns (ms quantise, ms decode)."""
    import torch

    from paper_2508_04257_amd import binding as kb
    from paper_2508_04257_amd import pipeline

    dev = q.device
    desc = pipeline.desc_for(wv)
    slots = len(inputs)
    caches = [kb.alloc_cache(desc, dev) for _ in range(slots)]
    ws = kb.alloc_workspace(desc, dev)
    out = torch.empty((wv.B, wv.Hq, wv.D), dtype=torch.float16, device=dev)
    for i in range(slots):
        kb.kvs_quantize_kv(desc, inputs[i][0], inputs[i][1], bufs[i].keep_mask, caches[i], ws)
        kb.kvs_decode_attn(desc, q, caches[i], out, None, ws)
    torch.cuda.synchronize()
    reps = 12
    e = [HipEvent() for _ in range(3)]
    e[0].record()
    for i in range(reps):
        kb.kvs_quantize_kv(desc, inputs[i % slots][0], inputs[i % slots][1], bufs[i % slots].keep_mask, caches[i % slots], ws)
    e[1].record()
    for i in range(reps):
        kb.kvs_decode_attn(desc, q, caches[i % slots], out, None, ws)
    e[2].record()
    torch.cuda.synchronize()
    return e[0].elapsed_time(e[1]) / reps, e[1].elapsed_time(e[2]) / reps


def per_token_key_leg(w, inputs, bufs, q, dec_bytes, qnt_bytes):
    """The per-token Key scheme on the same shapes.  None where the scheme does not apply."""
    if w.key_per_token or w.sparse_frac > 0:
        return None
    ms_q, ms_d = _variant_leg(w.scaled(key_per_token=True), inputs, bufs, q)
    return {
        "ms_quantize_kv": round(ms_q, 4), "quantize_gbps": round(qnt_bytes / (ms_q * 1e-3) / 1e9, 2),
        "ms_decode_attn": round(ms_d, 4), "decode_gbps": round(dec_bytes / (ms_d * 1e-3) / 1e9, 2),
        "note": "same bytes per call as the per-channel scheme (the Key parameter array only changes shape); "
                "calls back to back over rotating cold caches",
    }


def eight_bit_leg(w, inputs, bufs, q):
    """The same shapes with 8-bit codes (twice the cache bytes per call).  None for 8-bit and
    dense-and-sparse workloads."""
    if w.bits == 8 or w.sparse_frac > 0:
        return None
    w8 = w.scaled(bits=8)
    ms_q, ms_d = _variant_leg(w8, inputs, bufs, q)
    dec_bytes, qnt_bytes = decode_algorithmic_bytes(w8, w8.keep_cap), quantize_algorithmic_bytes(w8)
    return {
        "ms_quantize_kv": round(ms_q, 4), "quantize_gbps": round(qnt_bytes / (ms_q * 1e-3) / 1e9, 2),
        "ms_decode_attn": round(ms_d, 4), "decode_gbps": round(dec_bytes / (ms_d * 1e-3) / 1e9, 2),
        "decode_frac_of_hbm_peak": round(dec_bytes / (ms_d * 1e-3) / 8e12, 4),
        "decode_algorithmic_bytes": dec_bytes,
        "note": "INT8 codes on the same shapes; calls back to back over rotating cold caches",
    }


def graph_leg(rig):
    """The same steps replayed from one HIP graph (all slots in sequence per replay): what the
    launch gaps of the eager loop cost."""
    import torch

    from paper_2508_04257_amd import pipeline

    graph = pipeline.capture_steps(rig.w, rig.hidden, rig.inputs, rig.q, rig.bufs)
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    reps = 10
    e0, e1 = HipEvent(), HipEvent()
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return {"ms_per_step": round(e0.elapsed_time(e1) / (reps * len(rig.bufs)), 4), "steps_per_replay": len(rig.bufs)}


def layers_leg(rig, layers):
    """The multi-layer form of a workload (Algorithm 1: the sink set is fixed once, at the
    emergence layer, and every later layer is quantised under it): one kvs_predict_sinks, then
    `layers` kvs_quantize_kv calls into `layers` distinct caches under that one mask, then one
    kvs_decode_attn per layer.  The K/V inputs rotate over the rig's slots (layer l reads input
    l mod slots); every layer has a cache of its own, so the decode stream of all layers together
    comes from HBM."""
    import torch

    from paper_2508_04257_amd import binding as kb
    from paper_2508_04257_amd import pipeline

    w, dev = rig.w, rig.dev
    desc = rig.bufs[0].desc
    caches = [kb.alloc_cache(desc, dev) for _ in range(layers)]
    ws = rig.bufs[0].workspace
    buf = rig.bufs[0]
    out = torch.empty((layers, w.B, w.Hq, w.D), dtype=torch.float16, device=dev)

    def run(ev=None):
        if ev:
            ev[0].record()
        pipeline.predict(w, rig.hidden, buf)                       # once: the mask every layer reuses
        if ev:
            ev[1].record()
        for l in range(layers):
            K, V = rig.inputs[l % rig.slots]
            kb.kvs_quantize_kv(desc, K, V, buf.keep_mask, caches[l], ws)
        if ev:
            ev[2].record()
        for l in range(layers):
            kb.kvs_decode_attn(desc, rig.q, caches[l], out[l], None, ws)
        if ev:
            ev[3].record()

    run()
    torch.cuda.synchronize()
    ev = [HipEvent() for _ in range(4)]
    run(ev)
    torch.cuda.synchronize()
    for c in caches:
        assert int(c.status.cpu()[0]) == 0, "capacity overflow reported by the library"
    ms_p, ms_q, ms_d = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), ev[2].elapsed_time(ev[3])
    cache_bytes = sum(t.numel() * t.element_size() for c in caches for t in c.tensors.values() if t is not None)
    given = {}
    if w.sparse_frac > 0:
        # The same quantise calls with outlier thresholds fixed beforehand (one search per distinct
        # input, outside the timed region), as a deployment with calibrated thresholds would run them.
        taus = [torch.zeros(2, dtype=torch.int32, device=dev) for _ in range(rig.slots)]
        for i, (K, V) in enumerate(rig.inputs):
            kb.kvs_outlier_thresholds(desc, K, V, buf.keep_mask, taus[i], ws)

        def run_given():
            for l in range(layers):
                K, V = rig.inputs[l % rig.slots]
                kb.kvs_quantize_kv_thresholds(desc, K, V, buf.keep_mask, taus[l % rig.slots], caches[l], ws)

        run_given()
        torch.cuda.synchronize()
        g0, g1 = HipEvent(), HipEvent()
        g0.record()
        run_given()
        g1.record()
        torch.cuda.synchronize()
        for c in caches:
            assert int(c.status.cpu()[0]) == 0, "capacity overflow reported by the library"
        ms_g = g0.elapsed_time(g1)
        given = {"ms_quantize_given_thresholds_total": round(ms_g, 3),
                 "ms_quantize_given_thresholds_per_layer": round(ms_g / layers, 4),
                 "quantize_given_thresholds_tokens_per_s_per_layer": round(w.B * w.n / (ms_g / layers * 1e-3), 1)}
    return {
        **given,
        "layers": layers, "caches_resident_gb": round(cache_bytes / 1e9, 2),
        "ms_predict_once": round(ms_p, 4),
        "ms_quantize_total": round(ms_q, 3), "ms_quantize_per_layer": round(ms_q / layers, 4),
        "quantize_tokens_per_s_per_layer": round(w.B * w.n / (ms_q / layers * 1e-3), 1),
        "ms_decode_total": round(ms_d, 3), "ms_decode_per_layer": round(ms_d / layers, 4),
        "decode_gbps": round(rig.dec_bytes / (ms_d / layers * 1e-3) / 1e9, 2),
        "decode_frac": round(rig.dec_bytes / (ms_d / layers * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "note": "one prediction, its mask reused by every layer's quantise call; a cache per layer, K/V inputs "
                f"rotating over {rig.slots} copies; one event pair around each phase",
    }


def guarded(leg, *args):
    """The leg's result, or a record of why it has none."""
    try:
        return leg(*args)
    except Exception as e:                                # noqa: BLE001 - anything a side leg can raise
        return {"error": f"{type(e).__name__}: {e}"[:300]}


def config_leg(name, steps, warmup, slots, dev):
    """One of the other workloads, timed like the headline one (same step, same event brackets)."""
    import gc

    import torch

    from paper_2508_04257_amd import binding as kb
    from paper_2508_04257_amd import synth

    w = synth.WORKLOADS[name]
    rig = Rig(w, slots, dev)
    t = rig.timed_steps(steps, warmup)
    b2b = rig.back_to_back(max(steps, 20))
    gbps = rig.dec_bytes / (t["ms_decode"] * 1e-3) / 1e9
    out = {
        "workload": workload_label(w),
        "kernel": decode_kernel_name(w, kb.kvs_decode_splits(rig.bufs[0].desc)),
        "steps": steps,
        "ms_decode": round(t["ms_decode"], 4), "decode_gbps": round(gbps, 2), "frac": round(gbps / HBM_PEAK_GBPS, 4),
        "ms_decode_back_to_back": round(b2b, 4),
        "frac_back_to_back": round(rig.dec_bytes / (b2b * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes": rig.dec_bytes,
        "ms_quantize": round(t["ms_quant"], 4),
        "quantize_tokens_per_s": round(w.B * w.n / (t["ms_quant"] * 1e-3), 1),
        "quantize_gbps": round(rig.qnt_bytes / (t["ms_quant"] * 1e-3) / 1e9, 2),
        "ms_predict": round(t["ms_predict"], 4),
    }
    if rig.nnz is not None:
        out["csr_entries"] = {"k": rig.nnz[0], "v": rig.nnz[1]}
    if w.layers > 1:
        out["layers%d" % w.layers] = guarded(layers_leg, rig, w.layers)
    del rig
    gc.collect()
    torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------------------------------------
# --sweep: every supported shape
# ------------------------------------------------------------------------------------------------
def sweep_shape(bits, group, rep, key_per_token, pairs, n, dev="cuda:0", slots=3):
    """(decode seconds, quantise seconds, decode bytes, quantise bytes, workgroups per (sequence,
    KV head)) of one shape: calls back to back over rotating caches."""
    import gc

    import torch

    from paper_2508_04257_amd import binding as kb
    from paper_2508_04257_amd import pipeline, synth

    Hkv = 32 // rep
    w = synth.Workload("sweep", B=pairs // Hkv, n=n, Hq=32, Hkv=Hkv, bits=bits, group=group, k_sinks=5,
                       key_per_token=key_per_token)
    rig = Rig(w, slots, dev)

    def timed(fn, iters):
        for i in range(6):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = HipEvent(), HipEvent()
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e-3

    t_dec = timed(lambda i: pipeline.decode(rig.q, rig.bufs[i % slots]), 60)
    t_qnt = timed(lambda i: pipeline.quantize(rig.inputs[i % slots][0], rig.inputs[i % slots][1], rig.bufs[i % slots]), 30)
    out = (t_dec, t_qnt, rig.dec_bytes, rig.qnt_bytes, kb.kvs_decode_splits(rig.bufs[0].desc))
    del rig
    gc.collect()
    torch.cuda.empty_cache()
    return out


def sweep(pairs, n):
    """Two markdown tables (per-channel and per-token Keys): bit width x group size x query heads
    per KV head, for a cache of `pairs` (sequence, KV head) pairs of `n` tokens, i.e. the same cache
    bytes in every row of one bit width.  The percentage is algorithmic bytes / time against
    8 TB/s, so a shape whose heads take several launches - each streams the codes again - shows a
    low figure by construction."""
    peak = HBM_PEAK_GBPS * 1e9
    for kpt in (False, True):
        print(("Per-token Keys" if kpt else "Per-channel Keys") +
              f", {pairs} (sequence, KV head) pairs x {n} tokens; decode: time, % of 8 TB/s\n")
        print("| bits | G | Hq/Hkv = 1 | 2 | 4 | 8 | quantise |")
        print("|---|---|---|---|---|---|---|")
        for bits in (2, 3, 4, 8):
            for group in (32, 64, 128):
                cells, qs = [], []
                for rep in (1, 2, 4, 8):
                    t_dec, t_qnt, b_dec, b_qnt, _ = sweep_shape(bits, group, rep, kpt, pairs, n)
                    cells.append(f"{t_dec * 1e6:.0f} us, {100 * b_dec / t_dec / peak:.0f} %")
                    qs.append((t_qnt * 1e6, 100 * b_qnt / t_qnt / peak))
                print(f"| {bits} | {group} | " + " | ".join(cells) +
                      f" | {min(t for t, _ in qs):.0f}-{max(t for t, _ in qs):.0f} us, "
                      f"{min(p for _, p in qs):.0f}-{max(p for _, p in qs):.0f} % |", flush=True)
        print()


# ------------------------------------------------------------------------------------------------
# the CPU oracle, timed before the GPU is touched
# ------------------------------------------------------------------------------------------------
def _cpu_slice(args):
    """One (sequence, KV head) slice of the workload at full length through the oracle, one
    thread.  Returns (seconds quantise, seconds decode)."""
    from threadpoolctl import threadpool_limits

    from oracle import kvsink_oracle as O
    from paper_2508_04257_amd import synth

    small, idx, q, mask = args
    with threadpool_limits(limits=1):
        K, V = synth.make_kv(small.scaled(seed=small.seed + idx))
        K, V = K.numpy(), V.numpy()
        t0 = time.perf_counter()
        cache = O.quantize_kv(K, V, mask, small.bits, small.group, max(small.keep_cap, 1),
                              key_per_token=small.key_per_token)
        t1 = time.perf_counter()
        O.decode_attn(q, cache, Hq=small.Hq)
        t2 = time.perf_counter()
    return t1 - t0, t2 - t1


def cpu_baseline(w, budget_s: float = 10.0):
    """The oracle as it stands, timed on this host on a bounded sample of the same workload:
    whole (sequence, head) slices at full length, first one at a time on one thread, then over
    all the host cores this process may use (one single-threaded worker process per core)."""
    import multiprocessing as mp

    import torch
    from threadpoolctl import threadpool_limits

    from oracle import kvsink_oracle as O
    from paper_2508_04257_amd import synth

    small = w.scaled(B=1, Hq=w.Hq // w.Hkv, Hkv=1)            # one (b, h) slice at the full n
    H = synth.make_hidden(small).numpy()
    q = synth.make_query(small).numpy()
    with threadpool_limits(limits=1):
        _, mask = O.predict_sinks(H, small.channels, small.k_sinks, small.first_n)
    total = w.B * w.Hkv
    done, t_quant, t_dec = 0, 0.0, 0.0
    t_start = time.perf_counter()
    torch.set_num_threads(1)
    while time.perf_counter() - t_start < budget_s and done < total:
        tq, td = _cpu_slice((small, done, q, mask))
        t_quant += tq
        t_dec += td
        done += 1
    slice_bytes = decode_algorithmic_bytes(small, small.keep_cap)
    out = {
        "value": round(done * slice_bytes / t_dec / 1e9, 6),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"{done} (sequence, KV head) slices of {w.name} at full length n={w.n} "
                  f"(of {total}); numpy oracle, single thread",
        "quantize_tokens_per_s": round(done * w.n / (w.Hkv * t_quant), 3),   # whole-layer equivalent
        "decode_ms_per_slice": round(1e3 * t_dec / done, 3),
        "quantize_ms_per_slice": round(1e3 * t_quant / done, 3),
    }
    # All cores: the same slices handed to one worker process per core (forked before this process
    # has touched the GPU); decode rate = bytes of all slices / (wall time x the decode share of
    # the workers' busy time).
    try:
        cores = min(len(os.sched_getaffinity(0)), 16)
    except AttributeError:
        cores = min(os.cpu_count() or 1, 16)
    if cores > 1:
        per_slice = (t_quant + t_dec) / done
        count = int(min(total, max(cores, budget_s * cores / max(per_slice, 1e-3))))
        with mp.get_context("fork").Pool(cores) as pool:
            pool.map(_cpu_slice, [(small, 10_000 + i, q, mask) for i in range(cores)])     # start-up, imports
            t0 = time.perf_counter()
            times = pool.map(_cpu_slice, [(small, i, q, mask) for i in range(count)], chunksize=1)
            wall = time.perf_counter() - t0
        busy_q, busy_d = sum(t[0] for t in times), sum(t[1] for t in times)
        out["all_cores"] = {
            "value": round(count * slice_bytes / (wall * busy_d / (busy_q + busy_d)) / 1e9, 6),
            "unit": "GB/s",
            "cores": cores,
            "quantize_tokens_per_s": round(count * w.n / (w.Hkv * wall * busy_q / (busy_q + busy_d)), 3),
            "sample": f"{count} slices over {cores} single-threaded worker processes, {wall:.1f} s wall "
                      "(input generation included in the wall time, excluded from the shares)",
        }
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--slots", type=int, default=4, help="rotating copies of inputs and caches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other workloads (\"configs\" in the JSON line)")
    ap.add_argument("--config-steps", type=int, default=20, help="timed steps of each other workload")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the JSON line: decode and quantise timings over the grid of supported shapes "
                         "(bits x group x heads per KV head x Key scheme) as two markdown tables")
    ap.add_argument("--sweep-pairs", type=int, default=256, help="--sweep: (sequence, KV head) pairs; a multiple of 32")
    ap.add_argument("--sweep-n", type=int, default=4096, help="--sweep: tokens per sequence; a multiple of 128")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain copy of known size (256 MiB read + 256 MiB written) a few times "
                         "before the steps: the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    from paper_2508_04257_amd import synth

    if args.sweep:
        import torch
        torch.cuda.set_device(0)
        sweep(args.sweep_pairs, args.sweep_n)
        return 0

    w = synth.WORKLOADS[args.workload]
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w)                        # before anything touches the GPU (it forks workers)

    import torch

    from paper_2508_04257_amd import binding as kb

    dev = "cuda:0"
    torch.cuda.set_device(0)
    slots = max(2, args.slots)

    if args.calibrate:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)              # one elementwise kernel: reads src once, writes dst once
        torch.cuda.synchronize()
        del src, dst

    rig = Rig(w, slots, dev)
    t = rig.timed_steps(args.steps, args.warmup)
    ms_decode, ms_quant = t["ms_decode"], t["ms_quant"]
    ms_decode_b2b = rig.back_to_back(max(args.steps, 20))
    dec_bytes, qnt_bytes = rig.dec_bytes, rig.qnt_bytes
    dec_gbps = dec_bytes / (ms_decode * 1e-3) / 1e9
    qnt_gbps = qnt_bytes / (ms_quant * 1e-3) / 1e9
    splits = kb.kvs_decode_splits(rig.bufs[0].desc)

    result = {
        "metric": "decode-attn effective HBM GB/s",
        "value": round(dec_gbps, 2),
        "unit": "GB/s",
        "pct_of_hbm_peak": round(100 * dec_gbps / HBM_PEAK_GBPS, 2),
        "quantize_tokens_per_s": round(w.B * w.n / (ms_quant * 1e-3), 1),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t["ms_step"], 4),
        "ms_predict": round(t["ms_predict"], 4),
        "ms_quantize": round(ms_quant, 4),
        "ms_decode": round(ms_decode, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "dtype_note": "decode: 2-8 bit codes as fp16 matrix-core operands, fp32 accumulation; quantise: fp32",
        "data": "synthetic",
        "config": {"workload": workload_label(w), "cache_slots": slots, "decode_splits": splits},
        "roofline": {
            "kernel": decode_kernel_name(w, splits),
            "bound": "hbm",
            "achieved": round(dec_gbps, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
            "traffic": measured_decode_traffic(w.name),
            "algorithmic_bytes": dec_bytes,
            "ms_kernel": round(ms_decode, 4),
            "ms_kernel_estimates": [round(x, 4) for x in t["ms_decode_estimates"]],
            "timing": "HIP events on the launch stream, never around the kernel alone: mean of "
                      "([predict+decode] - [predict]) and ([decode+quantise] - [quantise]), brackets of alternate steps",
            "back_to_back": {"ms": round(ms_decode_b2b, 4),
                             "achieved": round(dec_bytes / (ms_decode_b2b * 1e-3) / 1e9, 2),
                             "frac": round(dec_bytes / (ms_decode_b2b * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                             "note": "same call repeated over the rotating cold caches, no events between launches"},
            "stream_ceiling": rig.stream_ceiling(),
        },
        "roofline_quantize": {
            "kernel": ("kvs_quantize_kv = keep_index_fast_kernel + quantize_k%s_fast_kernel + quantize_v_fast_kernel"
                       % ("_token" if w.key_per_token else ""))
                      if w.sparse_frac == 0 else
                      "kvs_quantize_kv = sparse_hist_kernel x2 + quantize_{k,v}_fast_kernel<SPARSE> + scan + csr_move_kernel",
            "bound": "hbm",
            "achieved": round(qnt_gbps, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(qnt_gbps / HBM_PEAK_GBPS, 4),
            "traffic": None,
            "algorithmic_bytes": qnt_bytes,
        },
    }
    # The figures above are the line's contract; what follows are legs reported beside them.  A leg
    # that fails is reported as such and does not take the line with it.
    result["graph_replay"] = guarded(graph_leg, rig)
    if w.sparse_frac == 0:
        result["growing_cache"] = guarded(growing_cache_leg, w, rig.inputs[0], rig.q, dec_bytes)
        result["static_quantisation"] = guarded(static_leg, w, rig.inputs, rig.bufs, qnt_bytes)
        kpt = guarded(per_token_key_leg, w, rig.inputs, rig.bufs, rig.q, dec_bytes, qnt_bytes)
        if kpt is not None:
            result["per_token_keys"] = kpt
        int8 = guarded(eight_bit_leg, w, rig.inputs, rig.bufs, rig.q)
        if int8 is not None:
            result["int8"] = int8
    elif w.layers > 1:
        result["layers%d" % w.layers] = guarded(layers_leg, rig, w.layers)
    if not args.no_configs:
        import gc
        del rig
        gc.collect()
        guarded(torch.cuda.empty_cache)
        result["configs"] = {name: guarded(config_leg, name, args.config_steps, 3, slots, dev)
                             for name in OTHER_CONFIGS if name != w.name}
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
