"""Pins for the oracle's growing cache (Section 2, "KV cache": the decoding phase appends the new
token's K and V; Appendix A: quantisation after accumulating a number of local tokens)."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16


def _fields(c: O.Cache):
    return dict(k_codes=c.k_codes, v_codes=c.v_codes, k_params=c.k_params, v_params=c.v_params, keep_k=c.keep_k,
                keep_v=c.keep_v, keep_idx=c.keep_idx, keep_cnt=c.keep_cnt, keep_mask=c.keep_mask)


def assert_same_growing(a: O.GrowingCache, b: O.GrowingCache):
    assert a.n_tokens == b.n_tokens and a.n_quant == b.n_quant
    assert np.array_equal(a.res_k.view(np.uint16), b.res_k.view(np.uint16))
    assert np.array_equal(a.res_v.view(np.uint16), b.res_v.view(np.uint16))
    assert np.array_equal(a.res_mask, b.res_mask)
    if a.quant is None:
        assert b.quant is None
        return
    fa, fb = _fields(a.quant), _fields(b.quant)
    for name in fa:
        x, y = fa[name], fb[name]
        assert np.array_equal(x.view(np.uint16) if x.dtype == np.float16 else x,
                              y.view(np.uint16) if y.dtype == np.float16 else y), name


def sdpa64(q, K, V):
    qt = torch.from_numpy(q.astype(np.float64))[None, None, None, :]
    Kt = torch.from_numpy(K.astype(np.float64))[None, None]
    Vt = torch.from_numpy(V.astype(np.float64))[None, None]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)[0, 0, 0].numpy()


@pytest.mark.parametrize("bits,G", [(4, 128), (3, 64), (2, 32), (8, 64)])
def test_blockwise_quantisation_is_the_whole_quantisation(bits, G):
    """Groups are positional and never straddle a 128-token block, so quantising block by block
    and concatenating is quantising the whole: what lets a cache grow one block at a time."""
    rng = np.random.default_rng(bits)
    K, V = random_fp16(rng, (2, 2, 384, 128)), random_fp16(rng, (2, 2, 384, 128))
    mask = np.zeros((2, 384), np.uint8)
    mask[0, [0, 14, 130, 383]] = 1
    mask[1, [127, 128]] = 1
    whole = O.quantize_kv(K, V, mask, bits, G, keep_cap=6)
    pieces = None
    for t0 in range(0, 384, 128):
        blk = O.quantize_kv(K[:, :, t0:t0 + 128], V[:, :, t0:t0 + 128], mask[:, t0:t0 + 128], bits, G, keep_cap=6)
        pieces = O._concat_caches(pieces, blk)
    fa, fb = _fields(whole), _fields(pieces)
    for name in fa:
        x, y = fa[name], fb[name]
        assert np.array_equal(x.view(np.uint16) if x.dtype == np.float16 else x,
                              y.view(np.uint16) if y.dtype == np.float16 else y), name


def test_kept_rows_beyond_the_capacity_are_reported_however_the_blocks_split_them():
    rng = np.random.default_rng(17)
    K, V = random_fp16(rng, (1, 1, 256, 128)), random_fp16(rng, (1, 1, 256, 128))
    blocks = lambda mask: [O.quantize_kv(K[:, :, t:t + 128], V[:, :, t:t + 128], mask[:, t:t + 128], 4, 128, keep_cap=3)
                           for t in (0, 128)]
    # two kept tokens in each block: neither block overflows on its own, together they do
    mask = np.zeros((1, 256), np.uint8)
    mask[0, [4, 9, 130, 200]] = 1
    a, b = blocks(mask)
    assert a.status == b.status == O.STATUS_OK
    both = O._concat_caches(a, b)
    assert both.status == O.STATUS_CAPACITY and both.keep_cnt.tolist() == [4]
    assert both.keep_idx[0].tolist() == [4, 9, 130]
    whole = O.quantize_kv(K, V, mask, 4, 128, keep_cap=3)
    assert whole.status == O.STATUS_CAPACITY and np.array_equal(whole.keep_idx, both.keep_idx)
    assert np.array_equal(whole.keep_k.view(np.uint16), both.keep_k.view(np.uint16))
    # the second block overflows by itself, the first holds none
    mask = np.zeros((1, 256), np.uint8)
    mask[0, [130, 140, 150, 160, 170]] = 1
    a, b = blocks(mask)
    assert (a.status, b.status) == (O.STATUS_OK, O.STATUS_CAPACITY)
    assert O._concat_caches(a, b).status == O.STATUS_CAPACITY
    # decoding such a cache still works on the rows it has (the count is clamped to the capacity)
    q = random_fp16(rng, (1, 1, 128))
    Kd, _ = O.effective_kv(both, 0, 0)
    assert np.array_equal(Kd[[4, 9, 130]], K[0, 0, [4, 9, 130]].astype(np.float64))
    assert np.all(np.isfinite(O.decode_attn(q, both, Hq=1)[2]))


@pytest.mark.parametrize("n0,n1", [(0, 130), (44, 300), (128, 257), (300, 300), (255, 256)])
def test_appending_reaches_the_state_of_a_prefill(n0, n1):
    rng = np.random.default_rng(n0 + n1)
    bits, G, cap = 4, 64, 5
    K, V = random_fp16(rng, (2, 2, n1, 128)), random_fp16(rng, (2, 2, n1, 128))
    mask = np.zeros((2, n1), np.uint8)
    for t in (0, 14, 40, 129):                                  # kept tokens only inside the prompt
        if t < n0:
            mask[0, t] = 1
    if n0 > 2:
        mask[1, n0 - 1] = 1                                      # a kept token in the fp16 tail of the prompt
    gc = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], bits, G, cap)
    assert gc.n_quant == (n0 // 128) * 128 and gc.res_k.shape[2] == n0 % 128
    for t in range(n0, n1):
        gc = O.append_token(gc, K[:, :, t], V[:, :, t])
        assert gc.n_tokens == t + 1 and gc.res_k.shape[2] == (t + 1) % 128
    assert_same_growing(gc, O.prefill_cache(K, V, mask, bits, G, cap))


def test_a_token_appended_with_its_keep_flag_is_kept_when_its_block_is_quantised():
    rng = np.random.default_rng(21)
    bits, G, cap, n0, n1 = 4, 128, 4, 100, 256
    K, V = random_fp16(rng, (2, 1, n1, 128)), random_fp16(rng, (2, 1, n1, 128))
    mask = np.zeros((2, n1), np.uint8)
    mask[0, 3], mask[0, 110], mask[1, 200] = 1, 1, 1              # 110 and 200 arrive by append
    K[0, 0, 110] *= 50                                             # a kept row this wild would wreck its groups' ranges
    gc = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], bits, G, cap)
    for t in range(n0, n1):
        gc = O.append_token(gc, K[:, :, t], V[:, :, t], keep_new=mask[:, t])
    want = O.prefill_cache(K, V, mask, bits, G, cap)
    assert_same_growing(gc, want)
    assert gc.quant.keep_idx[0].tolist() == [3, 110, -1, -1] and gc.quant.keep_idx[1].tolist() == [200, -1, -1, -1]
    assert np.array_equal(gc.quant.keep_k[0, 0, 1].view(np.uint16), K[0, 0, 110].view(np.uint16))
    # without the flag the wild row is quantised and stretches the range of every channel's group
    plain = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], bits, G, cap)
    for t in range(n0, n1):
        plain = O.append_token(plain, K[:, :, t], V[:, :, t])
    assert plain.quant.keep_cnt.tolist() == [1, 0]
    assert not np.array_equal(plain.quant.k_params[0, 0, 0], gc.quant.k_params[0, 0, 0])


def test_residual_rows_are_exact_and_short_caches_are_plain_attention():
    rng = np.random.default_rng(3)
    K, V = random_fp16(rng, (1, 2, 100, 128)), random_fp16(rng, (1, 2, 100, 128))
    q = random_fp16(rng, (1, 4, 128))
    gc = O.prefill_cache(K, V, np.zeros((1, 100), np.uint8), 4, 128, 2)
    assert gc.quant is None
    assert np.array_equal(gc.res_k.view(np.uint16), K.view(np.uint16))
    _, lse, o64 = O.decode_attn_growing(q, gc, Hq=4)
    for hq in range(4):
        ref = sdpa64(q[0, hq], K[0, hq // 2], V[0, hq // 2])
        assert np.abs(o64[0, hq] - ref).max() <= 1e-12


def test_growing_decode_is_attention_over_prefix_and_residual():
    """Lossless integer grid (scale 1): the quantised prefix reproduces K, V exactly, so the whole
    result must equal plain attention over the raw tokens - prefix, kept rows and residual alike."""
    rng = np.random.default_rng(4)
    n = 128 * 2 + 37
    K = rng.integers(-7, 8, (1, 1, n, 128)).astype(np.float16)
    V = rng.integers(-7, 8, (1, 1, n, 128)).astype(np.float16)
    K[0, 0, ::128] = -7; K[0, 0, 1::128] = 8          # every group spans exactly [-7, 8]: scale 1, zero 7
    V[0, 0, :, 0] = -7; V[0, 0, :, 1] = 8
    mask = np.zeros((1, n), np.uint8)
    mask[0, [5, 200, 270]] = 1                         # 270 sits in the fp16 tail
    K[0, 0, 5] *= 3; V[0, 0, 200] *= 0.5               # kept rows may hold anything
    q = (random_fp16(rng, (1, 1, 128)).astype(np.float32) * 0.05).astype(np.float16)
    gc = O.prefill_cache(K, V, mask, 4, 128, 4)
    _, _, o64 = O.decode_attn_growing(q, gc, Hq=1)
    assert np.abs(o64[0, 0] - sdpa64(q[0, 0], K[0, 0], V[0, 0])).max() <= 1e-10
    # and with no residual it is decode_attn itself
    gc2 = O.prefill_cache(K[:, :, :256], V[:, :, :256], mask[:, :256], 4, 128, 4)
    a = O.decode_attn_growing(q, gc2, Hq=1)[2]
    b = O.decode_attn(q, gc2.quant, Hq=1)[2]
    assert np.array_equal(a, b)
