"""Parity of the growing-cache calls (kvs_quantize_prefix, kvs_append_kv, kvs_decode_attn_n) with the
oracle's GrowingCache on the same seeded inputs.  Bars as in test_gpu_parity.py: codes, parameter
words, kept rows, residual rows and masks bit-exact; attention outputs within 2e-3."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV, OUT_TOL, row_rel_err, u32

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def assert_growing_equal(desc, cache, gc: O.GrowingCache):
    """The device buffers are laid out for the capacity desc.n; the oracle's for the tokens held."""
    B, H, n_cap, cap = desc.B, desc.Hkv, desc.n, desc.keep_cap
    W, G = O.words_per_128(gc.bits), gc.group
    nq, r = gc.n_quant, gc.n_tokens - gc.n_quant
    if nq:
        ref = gc.quant
        kc = u32(cache.k_codes)[:B * H * (n_cap // 64) * W * 64].reshape(B, H, n_cap // 64, W, 64)
        vc = u32(cache.v_codes)[:B * H * (n_cap // 128) * W * 128].reshape(B, H, n_cap // 128, W, 128)
        kp = u32(cache.k_params)[:B * H * (n_cap // G) * 128]
        kp = kp.reshape(B, H, n_cap, 128 // G) if gc.key_per_token else kp.reshape(B, H, n_cap // G, 128)
        vp = u32(cache.v_params)[:B * H * n_cap * (128 // G)].reshape(B, H, n_cap, 128 // G)
        assert np.array_equal(kc[:, :, :nq // 64], ref.k_codes)
        assert np.array_equal(vc[:, :, :nq // 128], ref.v_codes)
        assert np.array_equal(kp[:, :, :(nq if gc.key_per_token else nq // G)], ref.k_params)
        assert np.array_equal(vp[:, :, :nq], ref.v_params)
        assert np.array_equal(cache.keep_cnt.cpu().numpy()[:B], ref.keep_cnt)
        assert int(cache.status.cpu()[0]) == ref.status
        if ref.status == O.STATUS_OK:
            assert np.array_equal(cache.keep_idx.cpu().numpy()[:B * cap].reshape(B, cap), ref.keep_idx)
            kk = cache.keep_k.cpu().numpy().view(np.uint16)[:B * H * cap * 128].reshape(B, H, cap, 128)
            kv = cache.keep_v.cpu().numpy().view(np.uint16)[:B * H * cap * 128].reshape(B, H, cap, 128)
            assert np.array_equal(kk, ref.keep_k.view(np.uint16))
            assert np.array_equal(kv, ref.keep_v.view(np.uint16))
    else:
        assert not cache.keep_cnt.cpu().numpy()[:B].any()
    mask = cache.keep_mask.cpu().numpy()[:B * n_cap].reshape(B, n_cap)
    if nq:
        assert np.array_equal(mask[:, :nq], gc.quant.keep_mask)
    assert np.array_equal(mask[:, nq:nq + r], gc.res_mask)
    rk = cache.res_k.cpu().numpy().view(np.uint16)[:B * H * 128 * 128].reshape(B, H, 128, 128)
    rv = cache.res_v.cpu().numpy().view(np.uint16)[:B * H * 128 * 128].reshape(B, H, 128, 128)
    assert np.array_equal(rk[:, :, :r], gc.res_k.view(np.uint16))
    assert np.array_equal(rv[:, :, :r], gc.res_v.view(np.uint16))


def hip_decode_n(desc, cache, ws, q, n_tokens):
    out = torch.empty((desc.B, desc.Hq, 128), dtype=torch.float16, device=DEV)
    lse = torch.empty((desc.B, desc.Hq), dtype=torch.float32, device=DEV)
    kb.kvs_decode_attn_n(desc, dev(q), cache, n_tokens, out, lse, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def check_decode(desc, cache, ws, q, gc, Hq):
    out, lse = hip_decode_n(desc, cache, ws, q, gc.n_tokens)
    _, ref_lse, ref64 = O.decode_attn_growing(q, gc, Hq)
    assert np.all(np.isfinite(out))
    assert row_rel_err(out, ref64) <= OUT_TOL
    assert np.abs(lse - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("bits,G,rep,n0", [
    (4, 128, 1, 300), (3, 64, 4, 300), (2, 32, 1, 300), (4, 64, 2, 300), (3, 128, 8, 257),
    (4, 128, 1, 100),      # shorter than one block: residual rows only
    (2, 128, 4, 384),      # whole blocks only
    (4, 32, 1, 0),         # an empty prompt
    (8, 64, 4, 300), (8, 128, 1, 257),
    (8, 128, 8, 300),      # four-wave workgroups: a wave merges two heads and takes two residual states
    (3, 32, 4, 300),       # four-wave workgroups at 3 bit
])
def test_prefix_then_appends_match_the_oracle(bits, G, rep, n0):
    rng = np.random.default_rng(bits * 1000 + G + n0)
    B, H, n_cap, cap, n1 = 2, 2, 640, 6, max(n0, 1) + 140
    K, V = random_fp16(rng, (B, H, n1, 128)), random_fp16(rng, (B, H, n1, 128))
    K[:, :, :, [7, 90]] *= np.float16(8)
    mask = np.zeros((B, n1), np.uint8)
    for t in (0, 14, 130):
        if t < n0:
            mask[0, t] = 1
    if n0 > 3:
        mask[1, n0 - 2] = 1                                   # kept token in the prompt's fp16 tail (when there is one)
    desc = kb.make_desc(B, n_cap, H * rep, H, bits, G, cap)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_prefix(desc, dev(K[:, :, :n0]), dev(V[:, :, :n0]), dev(mask[:, :n0]), n0, cache, ws)
    torch.cuda.synchronize()
    gc = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], bits, G, cap)
    assert_growing_equal(desc, cache, gc)
    q = random_fp16(rng, (B, H * rep, 128))
    if n0:
        check_decode(desc, cache, ws, q, gc, H * rep)
    checkpoints = {n0 + 1, (n0 // 128 + 1) * 128 - 1, (n0 // 128 + 1) * 128, (n0 // 128 + 1) * 128 + 1, n1}
    for t in range(n0, n1):
        kb.kvs_append_kv(desc, dev(K[:, :, t]), dev(V[:, :, t]), t, cache, ws)
        gc = O.append_token(gc, K[:, :, t], V[:, :, t])
        if t + 1 in checkpoints:
            torch.cuda.synchronize()
            assert_growing_equal(desc, cache, gc)
            check_decode(desc, cache, ws, q, gc, H * rep)
    # the state reached by appending is the state of a prefill of the same tokens
    cache2 = kb.alloc_cache(desc, DEV)
    kb.kvs_quantize_prefix(desc, dev(K), dev(V), dev(mask), n1, cache2, ws)
    torch.cuda.synchronize()
    assert_growing_equal(desc, cache2, gc)


def test_growing_cache_filled_to_capacity_equals_the_plain_calls():
    """n_tokens == capacity: kvs_quantize_prefix is kvs_quantize_kv and kvs_decode_attn_n is kvs_decode_attn."""
    rng = np.random.default_rng(11)
    B, H, n, bits, G, cap = 2, 3, 512, 4, 128, 4
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 14]] = 1
    mask[1, [511]] = 1
    q = random_fp16(rng, (B, H, 128))
    desc = kb.make_desc(B, n, H, H, bits, G, cap)
    ws = kb.alloc_workspace(desc, DEV)
    a, b = kb.alloc_cache(desc, DEV), kb.alloc_cache(desc, DEV)
    kb.kvs_quantize_prefix(desc, dev(K), dev(V), dev(mask), n, a, ws)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(mask), b, ws)
    torch.cuda.synchronize()
    used = dict(keep_idx=B * cap, keep_cnt=B)               # buffers are rounded up to 16 bytes
    for name in ("k_codes", "v_codes", "k_params", "v_params", "keep_k", "keep_v", "keep_idx", "keep_cnt", "keep_mask"):
        x, y = getattr(a, name), getattr(b, name)
        m = used.get(name, x.numel())
        assert torch.equal(x[:m], y[:m]), name
    o1, _ = hip_decode_n(desc, a, ws, q, n)
    out = torch.empty((B, H, 128), dtype=torch.float16, device=DEV)
    kb.kvs_decode_attn(desc, dev(q), b, out, None, ws)
    torch.cuda.synchronize()
    ref = O.decode_attn(q, O.quantize_kv(K, V, mask, bits, G, cap), Hq=H)[2]
    assert row_rel_err(o1, ref) <= OUT_TOL and row_rel_err(out.cpu().numpy(), ref) <= OUT_TOL
