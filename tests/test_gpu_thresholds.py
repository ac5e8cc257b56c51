"""Outlier thresholds kept apart from the quantise call: kvs_outlier_thresholds is the search of
kvs_quantize_kv alone, kvs_quantize_kv_thresholds the quantise call with thresholds given.  The
oracle takes given thresholds through `taus` (15-bit fp16 magnitude patterns; 32768 isolates
nothing)."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV, OUT_TOL, assert_cache_equal, assert_csr_equal, hip_decode, row_rel_err

pytestmark = pytest.mark.gpu


def _to_dev(*arrays):
    return [torch.from_numpy(a).to(DEV) for a in arrays]


def _quantize_with(desc, K, V, mask, tau):
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv_thresholds(desc, *_to_dev(K, V, mask), tau, cache, ws)
    torch.cuda.synchronize()
    return cache, ws


@pytest.mark.parametrize("bits,G,rep", [(3, 128, 1), (4, 64, 4), (2, 32, 2)])
def test_thresholds_found_once_and_given_to_later_calls(bits, G, rep):
    rng = np.random.default_rng(100 * bits + rep)
    B, H, n, frac, keep_cap = 2, 2, 640, 0.01, 4
    K1, V1 = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    K2 = (random_fp16(rng, (B, H, n, 128)).astype(np.float32) * 1.3).astype(np.float16)     # wider: more than 1 % reach the thresholds
    V2 = (random_fp16(rng, (B, H, n, 128)).astype(np.float32) * 0.8).astype(np.float16)     # narrower: fewer do
    mask = np.zeros((B, n), np.uint8)
    mask[:, [0, 14]] = 1
    mask[1, 300] = 1
    desc = kb.make_desc(B, n, H * rep, H, bits, G, keep_cap, sparse_frac=frac, sparse_cap=24000)
    ws = kb.alloc_workspace(desc, DEV)
    tau = torch.full((2,), -1, dtype=torch.int32, device=DEV)
    kb.kvs_outlier_thresholds(desc, *_to_dev(K1, V1, mask), tau, ws)
    torch.cuda.synchronize()
    ref_tau = (O.sparse_threshold(K1, mask, frac), O.sparse_threshold(V1, mask, frac))
    assert tuple(tau.cpu().tolist()) == ref_tau

    # on the data they were found on: the dynamic call, bit for bit
    dyn, dyn_ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, *_to_dev(K1, V1, mask), dyn, dyn_ws)
    given, _ = _quantize_with(desc, K1, V1, mask, tau)
    ref1 = O.quantize_kv(K1, V1, mask, bits, G, keep_cap, sparse_frac=frac)
    for cache in (dyn, given):
        assert_cache_equal(cache, ref1)
        assert_csr_equal(cache, ref1)

    # on other data: whatever reaches the thresholds is isolated, more or fewer than the fraction
    cache2, ws2 = _quantize_with(desc, K2, V2, mask, tau)
    ref2 = O.quantize_kv(K2, V2, mask, bits, G, keep_cap, sparse_frac=frac, taus=ref_tau)
    count = (mask == 0).sum() * H * 128
    assert len(ref2.k_col) > 1.5 * frac * count and len(ref2.v_col) < 0.7 * frac * count
    assert_cache_equal(cache2, ref2)
    assert_csr_equal(cache2, ref2)
    q = random_fp16(rng, (B, H * rep, 128))
    out, lse = hip_decode(desc, cache2, ws2, q)
    _, ref_lse, ref64 = O.decode_attn(q, ref2, Hq=H * rep)
    assert row_rel_err(out, ref64) <= OUT_TOL
    assert np.abs(lse - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_threshold_words_at_their_limits():
    rng = np.random.default_rng(5)
    B, H, n, bits, G, keep_cap = 1, 2, 256, 3, 128, 2
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    mask = np.zeros((B, n), np.uint8)
    mask[0, 0] = 1
    desc = kb.make_desc(B, n, H, H, bits, G, keep_cap, sparse_frac=0.01, sparse_cap=1000)
    # 0x8000 and anything above it: nothing is isolated, the cache is the dense one plus empty CSR rows
    for word in (0x8000, 0x7FFFFFFF, -1):
        tau = torch.tensor([word, word], dtype=torch.int32, device=DEV)
        cache, _ = _quantize_with(desc, K, V, mask, tau)
        ref = O.quantize_kv(K, V, mask, bits, G, keep_cap, sparse_frac=0.01, taus=(32768, 32768))
        assert len(ref.k_col) == 0
        assert_cache_equal(cache, ref)
        assert_csr_equal(cache, ref)
    # a threshold that most of the tensor reaches: reported through the status word, never overrun
    tau = torch.tensor([1, 1], dtype=torch.int32, device=DEV)
    cache, ws = _quantize_with(desc, K, V, mask, tau)
    assert int(cache.status.cpu()[0]) == kb.KVS_ERR_CAPACITY
    out, _ = hip_decode(desc, cache, ws, random_fp16(rng, (B, H, 128)))
    assert np.all(np.isfinite(out))
