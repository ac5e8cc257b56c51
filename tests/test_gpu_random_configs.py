"""Seeded sweep over descriptor combinations the other parity tests do not enumerate one by one:
bit width x group size x heads per KV head x Key scheme x isolated outliers x shapes x keep
patterns.  Same bars as everywhere: cache bit-exact, attention outputs within 2e-3."""
import os

import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV, OUT_TOL, assert_cache_equal, assert_csr_equal, hip_decode, row_rel_err

pytestmark = pytest.mark.gpu


def _draw(rng):
    bits = int(rng.choice([2, 3, 4, 8]))
    G = int(rng.choice([32, 64, 128]))
    rep = int(rng.choice([1, 2, 4, 8]))
    kpt = bool(rng.integers(0, 2))
    sparse = (not kpt) and bits != 8 and rng.random() < 0.3
    B = int(rng.integers(1, 4))
    H = int(rng.integers(1, 4))
    n = 128 * int(rng.integers(1, 13))
    return bits, G, rep, kpt, sparse, B, H, n


@pytest.mark.parametrize("case", range(int(os.environ.get("KVS_RANDOM_CASES", "64"))))   # more seeds on request
def test_random_configuration(case):
    rng = np.random.default_rng(9000 + case)
    bits, G, rep, kpt, sparse, B, H, n = _draw(rng)
    kind = str(rng.choice(["normal", "wide", "tiny"])) if not sparse else "normal"
    # (heavy-tailed Keys would put scores in the thousands, where fp32 score arithmetic itself is
    # coarser than the 2e-3 bar; the tail goes to the Values only)
    K = random_fp16(rng, (B, H, n, 128), "tiny" if kind == "tiny" else "normal")
    V = random_fp16(rng, (B, H, n, 128), kind)
    if rng.random() < 0.5:                                                  # outlier channels (inputs stay finite)
        cols = rng.integers(0, 128, 3)
        K[:, :, :, cols] = np.clip(K[:, :, :, cols].astype(np.float32) * 8, -60000, 60000).astype(np.float16)
    mask = np.zeros((B, n), np.uint8)
    style = int(rng.integers(0, 4))
    if style == 1:
        mask[:, :int(rng.integers(1, min(n, 40)))] = 1                      # first-N
    elif style == 2:
        for b in range(B):
            mask[b, rng.choice(n, size=int(rng.integers(1, 9)), replace=False)] = 1
    elif style == 3:
        mask[0, :128] = 1                                                   # a whole Key group kept
    cap = int(mask.sum(1).max()) + int(rng.integers(0, 3))
    frac = 0.02 if sparse else 0.0
    scap = int(B * H * n * 128 * frac * 1.5) + 256 if sparse else 0
    q = random_fp16(rng, (B, H * rep, 128))
    desc = kb.make_desc(B, n, H * rep, H, bits, G, cap, sparse_frac=frac, sparse_cap=scap, key_per_token=kpt)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, torch.from_numpy(K).to(DEV), torch.from_numpy(V).to(DEV), torch.from_numpy(mask).to(DEV),
                       cache, ws)
    torch.cuda.synchronize()
    ref = O.quantize_kv(K, V, mask, bits, G, cap, sparse_frac=frac, sparse_cap=scap if sparse else None,
                        key_per_token=kpt)
    assert ref.status == O.STATUS_OK, (bits, G, rep, kpt, sparse, B, H, n)
    assert_cache_equal(cache, ref)
    if sparse:
        assert_csr_equal(cache, ref)
    out, lse = hip_decode(desc, cache, ws, q)
    _, ref_lse, ref64 = O.decode_attn(q, ref, Hq=H * rep)
    if kind == "tiny":
        assert np.abs(out.astype(np.float64) - ref64).max() <= 2e-7
    else:
        assert row_rel_err(out, ref64) <= OUT_TOL, (bits, G, rep, kpt, sparse, B, H, n)
    assert np.abs(lse - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())
