"""One pass of the hot path for a synthetic workload: predict sinks -> quantise K, V -> decode
attention.  Orchestration only (buffer allocation and the three C-ABI calls); no arithmetic."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as kb
from .synth import Workload


def desc_for(w: Workload, sparse_cap: int = 0) -> kb.KvsDesc:
    if w.sparse_frac > 0 and sparse_cap == 0:
        # room for the requested fraction plus ties at the threshold
        sparse_cap = int(w.B * w.Hkv * w.n * w.D * w.sparse_frac * 1.25) + 4096
    return kb.make_desc(w.B, w.n, w.Hq, w.Hkv, w.bits, w.group, max(w.keep_cap, 1),
                        sparse_frac=w.sparse_frac, sparse_cap=sparse_cap, key_per_token=w.key_per_token)


@dataclass
class StepBuffers:
    desc: kb.KvsDesc
    cache: kb.CacheBuffers
    workspace: torch.Tensor
    sink_idx: Optional[torch.Tensor]
    predict_ws: Optional[torch.Tensor]
    keep_mask: torch.Tensor
    out: torch.Tensor
    lse: torch.Tensor


def alloc_step(w: Workload, device="cuda") -> StepBuffers:
    desc = desc_for(w)
    return StepBuffers(
        desc=desc,
        cache=kb.alloc_cache(desc, device),
        workspace=kb.alloc_workspace(desc, device),
        sink_idx=torch.empty((w.B, w.k_sinks), dtype=torch.int32, device=device) if w.k_sinks else None,
        predict_ws=(torch.empty(kb.kvs_predict_workspace_bytes(w.B, w.n, w.k_sinks), dtype=torch.uint8, device=device)
                    if kb.kvs_predict_workspace_bytes(w.B, w.n, w.k_sinks) else None),
        keep_mask=torch.empty((w.B, w.n), dtype=torch.uint8, device=device),
        out=torch.empty((w.B, w.Hq, w.D), dtype=torch.float16, device=device),
        lse=torch.empty((w.B, w.Hq), dtype=torch.float32, device=device),
    )


def predict(w: Workload, hidden: torch.Tensor, buf: StepBuffers) -> None:
    kb.kvs_predict_sinks(hidden, list(w.channels), w.k_sinks, w.first_n, buf.sink_idx, buf.keep_mask,
                         buf.predict_ws)


def quantize(K: torch.Tensor, V: torch.Tensor, buf: StepBuffers) -> None:
    kb.kvs_quantize_kv(buf.desc, K, V, buf.keep_mask, buf.cache, buf.workspace)


def decode(q: torch.Tensor, buf: StepBuffers) -> None:
    kb.kvs_decode_attn(buf.desc, q, buf.cache, buf.out, buf.lse, buf.workspace)


def run_step(w: Workload, hidden: torch.Tensor, K: torch.Tensor, V: torch.Tensor, q: torch.Tensor,
             buf: StepBuffers) -> None:
    predict(w, hidden, buf)
    quantize(K, V, buf)
    decode(q, buf)


def step_in_bench_order(w: Workload, hidden: torch.Tensor, K: torch.Tensor, V: torch.Tensor, q: torch.Tensor,
                        cur: StepBuffers, old: StepBuffers) -> None:
    """The order a serving loop runs them in: this step's prediction, decode over a cache quantised
    earlier (no dependence on this step), then this step's quantisation."""
    predict(w, hidden, cur)
    decode(q, old)
    quantize(K, V, cur)


def capture_steps(w: Workload, hidden: torch.Tensor, inputs, q: torch.Tensor, bufs) -> torch.cuda.CUDAGraph:
    """One HIP graph holding len(bufs) consecutive steps over the rotating slots (step i: predict
    and quantise into slot i, decode slot i + 1).  Every call of the library only launches kernels
    on the current stream - no allocation, copy or synchronisation - so the calls can be captured
    as they are; a replay then costs one launch for the whole sequence."""
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(len(bufs)):
            step_in_bench_order(w, hidden, inputs[i][0], inputs[i][1], q, bufs[i], bufs[(i + 1) % len(bufs)])
    return graph
