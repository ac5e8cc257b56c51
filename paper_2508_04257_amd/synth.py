"""Seeded synthetic inputs with the shapes and value structure of LLaMA-family KV caches.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
quantiser, no top-k, no attention): both the CPU oracle's tests and the HIP
path's tests/benchmarks consume the tensors it returns, so the two are fed the
same bytes without sharing any code of the method itself.

What the generator mimics (paper, Sections 3.1-3.2 and the stable-outlier table
of Appendix D): a handful of "sink" tokens per sequence carry extreme
activations (magnitude in the hundreds) in a few fixed hidden-state channels,
their Key/Value rows are strongly suppressed in norm, and Keys have a few
large-magnitude channels per head.  The real activations need model weights, so
the magnitudes are fixed numbers: outliers +-800, sink K/V rows x0.1, outlier
key channels x10.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np
import torch

# LLaMA2-7B row of the stable-outlier table (Appendix D): hidden size 4096,
# outlier channels 2533 and 1415, emergence layer 1.
LLAMA2_7B_HIDDEN = 4096
LLAMA2_7B_OUTLIER_CHANNELS = (1415, 2533)
OUTLIER_MAGNITUDE = 800.0
SINK_ROW_SCALE = 0.1
KEY_CHANNEL_SCALE = 10.0
KEY_OUTLIER_CHANNELS_PER_HEAD = 4


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: cache shape, quantiser setting and keep policy."""

    name: str
    B: int
    n: int
    Hq: int
    Hkv: int
    D: int = 128
    bits: int = 4
    group: int = 128
    k_sinks: int = 2          # sink tokens planted per sequence == top-k asked of the predictor
    first_n: int = 0          # Preserve-First-N part of the keep set
    sparse_frac: float = 0.0  # dense-and-sparse fp16 outlier fraction
    key_per_token: bool = False   # per-token Keys (the other Key scheme of Section 5.1)
    key_channel_offset: float = 0.0   # mean of the Key outlier channels (0: centred, as in the benchmark workloads)
    sink_kv_spike: float = 0.0        # magnitude of two spike channels in the sink tokens' K / V rows (0: none)
    layers: int = 1
    student_t: bool = False   # heavy-tailed K/V (Student-t, nu = 4) instead of N(0,1)
    d_hidden: int = LLAMA2_7B_HIDDEN
    channels: Tuple[int, ...] = LLAMA2_7B_OUTLIER_CHANNELS
    seed: int = 0

    @property
    def keep_cap(self) -> int:
        return self.k_sinks + self.first_n

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five workloads; 0 is the small worked-example case (sinks at tokens {0, 14} as in
# the paper's LLaMA2-7B prompt example), 1 is the one the headline metric is quoted on.
WORKLOADS = {
    "cfg0_kvsink": Workload("cfg0_kvsink", B=1, n=1024, Hq=32, Hkv=32, bits=4, group=128, k_sinks=2),
    "cfg0_pfn": Workload("cfg0_pfn", B=1, n=1024, Hq=32, Hkv=32, bits=4, group=128, k_sinks=0, first_n=1),
    "cfg1": Workload("cfg1", B=8, n=4096, Hq=32, Hkv=32, bits=4, group=128, k_sinks=5),
    "cfg2": Workload("cfg2", B=16, n=8192, Hq=32, Hkv=8, bits=3, group=64, k_sinks=4),
    "cfg3": Workload("cfg3", B=4, n=32768, Hq=32, Hkv=32, bits=2, group=32, k_sinks=8, first_n=16),
    "cfg1_per_token_keys": Workload("cfg1_per_token_keys", B=8, n=4096, Hq=32, Hkv=32, bits=4, group=128, k_sinks=5,
                                    key_per_token=True),
    "cfg1_int8": Workload("cfg1_int8", B=8, n=4096, Hq=32, Hkv=32, bits=8, group=128, k_sinks=5),
    "cfg4": Workload("cfg4", B=32, n=4096, Hq=32, Hkv=32, bits=3, group=128, k_sinks=5,
                     sparse_frac=0.01, layers=32, student_t=True),
}


def _np_rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def sink_positions(w: Workload, n_planted: int | None = None) -> np.ndarray:
    """Planted sink tokens, int64 [B, n_planted], ascending per sequence.

    Tokens 0 and 14 come first (the positions of the paper's worked example), the rest are
    distinct uniform-random positions in [16, n).
    """
    m = w.k_sinks if n_planted is None else n_planted
    rng = _np_rng(w.seed, 1)
    out = np.empty((w.B, m), np.int64)
    fixed = [0, 14][:m]
    for b in range(w.B):
        extra = rng.choice(np.arange(16, w.n), size=m - len(fixed), replace=False) if m > len(fixed) else []
        out[b] = np.sort(np.concatenate([np.asarray(fixed, np.int64), np.asarray(extra, np.int64)]))
    return out


def _torch_gen(device, seed: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1_000_003 + stream)
    return g


def make_hidden(w: Workload, device="cpu", sinks: np.ndarray | None = None) -> torch.Tensor:
    """Hidden state of the emergence layer, fp16 [B, n, d]: N(0,1) with +-800 planted in the
    outlier channels at each sequence's sink tokens (sign drawn from the seed)."""
    sinks = sink_positions(w) if sinks is None else sinks
    g = _torch_gen(device, w.seed, 11)
    H = torch.randn((w.B, w.n, w.d_hidden), generator=g, device=device, dtype=torch.float32).to(torch.float16)
    rng = _np_rng(w.seed, 2)
    for b in range(w.B):
        for t in sinks[b]:
            for c in w.channels:
                sign = 1.0 if rng.integers(0, 2) else -1.0
                # A little spread so that the magnitudes are distinct but all far above the N(0,1) bulk.
                H[b, int(t), c] = sign * (OUTLIER_MAGNITUDE + float(rng.integers(0, 64)))
    return H


def key_outlier_channels(w: Workload) -> np.ndarray:
    """int64 [Hkv, 4]: the large-magnitude key channels of each head (chosen once from the seed)."""
    rng = _np_rng(w.seed, 3)
    return np.stack([rng.choice(w.D, size=KEY_OUTLIER_CHANNELS_PER_HEAD, replace=False) for _ in range(w.Hkv)])


def make_kv(w: Workload, device="cpu", layer: int = 0,
            sinks: np.ndarray | None = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """K, V fp16 [B, Hkv, n, D] of one layer.

    N(0,1) (or Student-t with 4 degrees of freedom), four key channels per head x10 (plus an
    optional mean, so that a suppressed sink row lies outside the other tokens' range in those
    channels), and the K/V rows of the sink tokens x0.1.
    """
    sinks = sink_positions(w) if sinks is None else sinks
    shape = (w.B, w.Hkv, w.n, w.D)
    out = []
    for tensor_id in (0, 1):
        g = _torch_gen(device, w.seed, 100 + 2 * layer + tensor_id)
        X = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        if w.student_t:
            chi = torch.zeros(shape, device=device, dtype=torch.float32)
            for _ in range(4):
                chi += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
            X = X / torch.sqrt(chi / 4.0)
            del chi
        if tensor_id == 0:
            ch = key_outlier_channels(w)
            for h in range(w.Hkv):
                cols = torch.as_tensor(ch[h], device=X.device)
                X[:, h, :, cols] *= KEY_CHANNEL_SCALE
                if w.key_channel_offset:
                    X[:, h, :, cols] += w.key_channel_offset
        for b in range(w.B):
            rows = torch.as_tensor(sinks[b], device=X.device)
            X[b, :, rows, :] *= SINK_ROW_SCALE
            if w.sink_kv_spike:                      # a suppressed row with two extreme entries
                X[b, :, rows, 17] = w.sink_kv_spike
                X[b, :, rows, 101] = -w.sink_kv_spike
        # fp16 inputs must be finite (a precondition of the library); the heavy tail could overflow.
        out.append(X.clamp_(-60000.0, 60000.0).to(torch.float16))
        del X
    return out[0], out[1]


def make_query(w: Workload, device="cpu", layer: int = 0) -> torch.Tensor:
    """One decode query per sequence and head, fp16 [B, Hq, D], N(0,1)."""
    g = _torch_gen(device, w.seed, 5000 + layer)
    return torch.randn((w.B, w.Hq, w.D), generator=g, device=device, dtype=torch.float32).to(torch.float16)
