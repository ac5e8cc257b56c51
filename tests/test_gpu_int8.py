"""Parity of 8-bit caches with the oracle: every group size and heads-per-KV-head ratio, per-channel
and per-token Keys, and data far from zero, where the scale is widened so that the zero point fits
its int16 half.  Codes, parameter words and kept rows bit-exact, outputs within 2e-3."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV, OUT_TOL, assert_cache_equal, hip_decode, row_rel_err

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _run(K, V, mask, q, G, rep, cap, kpt):
    B, H, n, _ = K.shape
    desc = kb.make_desc(B, n, H * rep, H, 8, G, cap, key_per_token=kpt)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(mask), cache, ws)
    torch.cuda.synchronize()
    ref = O.quantize_kv(K, V, mask, 8, G, cap, key_per_token=kpt)
    assert_cache_equal(cache, ref)
    out, lse = hip_decode(desc, cache, ws, q)
    _, ref_lse, ref64 = O.decode_attn(q, ref, Hq=H * rep)
    return row_rel_err(out, ref64), np.abs(lse - ref_lse).max(), ref


@pytest.mark.parametrize("kpt", [False, True])
@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("rep", [1, 2, 4, 8])
def test_quantize_and_decode(G, rep, kpt):
    rng = np.random.default_rng(800 + G + rep + kpt)
    B, H, n = 2, 2, 1152                                  # 9 Value tiles: uneven splits
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128), "wide")
    K[:, :, :, [3, 77]] *= np.float16(10)
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 14, 500]] = 1
    mask[1, [0, 1, 2, 3, 1151]] = 1
    q = random_fp16(rng, (B, H * rep, 128))
    err, lse_err, _ = _run(K, V, mask, q, G, rep, 6, kpt)
    assert err <= OUT_TOL and lse_err <= 1e-3


@pytest.mark.parametrize("kpt", [False, True])
@pytest.mark.parametrize("G", [32, 128])
def test_groups_far_from_zero(G, kpt):
    """Channels (Keys) and rows (Values) that sit at a large offset with a spread of a few fp16
    steps: range / 255 would need a zero point beyond int16; the widened scale is what both
    sides must use, and such groups still come back to within the fp16 spacing."""
    rng = np.random.default_rng(88 + G + kpt)
    B, H, n = 1, 2, 512
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    step = lambda base: np.spacing(np.float16(abs(base)))
    for c, base in ((5, 1000.0), (64, -812.0), (127, 30000.0), (31, 2.5)):
        K[:, :, :, c] = (np.float16(base) + rng.integers(0, 4, (B, H, n)) * step(base)).astype(np.float16)
    for t, base in ((7, 1000.0), (300, -44.0), (511, 6000.0)):
        V[:, :, t, :] = (np.float16(base) + rng.integers(0, 3, (B, H, 128)) * step(base)).astype(np.float16)
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 200]] = 1
    q = (random_fp16(rng, (B, H, 128)).astype(np.float32) * 0.01).astype(np.float16)   # (scores stay moderate)
    err, lse_err, ref = _run(K, V, mask, q, G, 1, 2, kpt)
    assert err <= OUT_TOL and lse_err <= 2e-3
    zk = (ref.k_params >> np.uint32(16)).astype(np.uint16).view(np.int16).astype(np.int64)
    zv = (ref.v_params >> np.uint32(16)).astype(np.uint16).view(np.int16).astype(np.int64)
    assert np.abs(zk).max() > 20000 or kpt                # the bound binds for the planted Key channels
    assert np.abs(zv).max() > 20000 and max(np.abs(zk).max(), np.abs(zv).max()) <= 32766
