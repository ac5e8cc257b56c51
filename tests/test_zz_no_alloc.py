"""kvs_decode_attn_noalloc (the decode call for callers that cannot allocate: no workspace argument,
the library's own scratch array) against kvs_decode_attn on the same cache, through the C ABI.

Two calls in a row on one GPU, the second on a smaller input, so that the second runs on scratch
that still holds the first call's contents.  Shapes are chosen so that the scratch is really used:
several workgroups per (sequence, KV head) leave their parts there and count themselves in on the
arrival counters at its head (the dense-and-sparse cache takes the same path with its outlier
corrections inside the stream kernel).
"""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16

pytestmark = pytest.mark.gpu

DEV = "cuda"
OUT_TOL = 2e-3


def _row_rel_err(got, ref):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    return float((np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max())


def _make(seed, B, H, Hq, n, bits, G, sparse):
    rng = np.random.default_rng(seed)
    K = random_fp16(rng, (B, H, n, 128))
    V = random_fp16(rng, (B, H, n, 128))
    q = random_fp16(rng, (B, Hq, 128))
    mask = np.zeros((B, n), np.uint8)
    mask[:, 0] = 1
    mask[:, 14] = 1
    mask[np.arange(B), rng.integers(16, n, B)] = 1
    frac, cap = (0.01, int(0.03 * B * H * n * 128)) if sparse else (0.0, 0)
    desc = kb.make_desc(B, n, Hq, H, bits, G, 4, sparse_frac=frac, sparse_cap=cap)
    cache = kb.alloc_cache(desc, DEV)
    ws = kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, torch.from_numpy(K).to(DEV), torch.from_numpy(V).to(DEV),
                       torch.from_numpy(mask).to(DEV), cache, ws)
    ref = O.quantize_kv(K, V, mask, bits, G, 4, sparse_frac=frac, sparse_cap=cap)
    ref_out = O.decode_attn(q, ref, Hq=Hq)[2]
    return desc, cache, ws, torch.from_numpy(q).to(DEV), ref_out


def _both(desc, cache, ws, q):
    out_ws = torch.zeros((desc.B, desc.Hq, 128), dtype=torch.float16, device=DEV)
    lse_ws = torch.zeros((desc.B, desc.Hq), dtype=torch.float32, device=DEV)
    out_na, lse_na = torch.zeros_like(out_ws), torch.zeros_like(lse_ws)
    kb.kvs_decode_attn(desc, q, cache, out_ws, lse_ws, ws)
    kb.kvs_decode_attn_noalloc(desc, q, cache, out_na, lse_na)
    torch.cuda.synchronize()
    return out_ws.cpu().numpy(), lse_ws.cpu().numpy(), out_na.cpu().numpy(), lse_na.cpu().numpy()


@pytest.mark.parametrize("sparse", [False, True])
def test_noalloc_decode_matches_the_workspace_call_on_two_calls_in_a_row(sparse):
    # first call: 2 x 2 (sequence, KV head) pairs of 2048 tokens -> 16 parts each; second call:
    # one pair of 512 tokens -> 4 parts, on the scratch the first call left behind.
    shapes = [(11, 2, 2, 8, 2048, 3, 64), (12, 1, 1, 1, 512, 3, 64)] if not sparse else \
             [(13, 2, 2, 2, 1024, 3, 128), (14, 1, 1, 1, 256, 3, 128)]
    for seed, B, H, Hq, n, bits, G in shapes:
        desc, cache, ws, q, ref_out = _make(seed, B, H, Hq, n, bits, G, sparse)
        assert kb.kvs_decode_splits(desc) > 1 or sparse            # the scratch is in use
        out_ws, lse_ws, out_na, lse_na = _both(desc, cache, ws, q)
        # same kernels on another buffer: equal up to the order in which a workgroup's waves
        # happened to take their chunks (fp32 sums), far inside the bar against the oracle
        assert _row_rel_err(out_na, out_ws) <= 1e-3
        assert np.allclose(lse_na, lse_ws, rtol=0, atol=1e-4)
        assert _row_rel_err(out_na, ref_out) <= OUT_TOL
        assert _row_rel_err(out_ws, ref_out) <= OUT_TOL


def test_noalloc_decode_rejects_a_descriptor_beyond_its_scratch():
    # 128 sequences x 64 heads: 8192 output rows of 520 bytes, one part each plus the residual part
    d = kb.make_desc(B=128, n=1024, Hq=64, Hkv=64, bits=4, group=128, keep_cap=8)
    assert 2 * 128 * 64 * 520 > kb.KVS_NOALLOC_SCRATCH_BYTES
    full = kb.KvsCache(**{name: 16 for name in kb.CACHE_FIELD_NAMES})
    st = kb.lib().kvs_decode_attn_noalloc(C.byref(d), 16, C.byref(full), 16, None, None)
    assert st == kb.KVS_ERR_SCRATCH
    assert "scratch" in kb.status_string(st)
