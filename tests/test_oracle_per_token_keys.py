"""Pins for the oracle's per-token Key scheme (Section 5.1: the comparison runs on per-token Key
and Value quantisation, static and dynamic, beside per-channel Keys; Appendix C equations).  A Key
row is quantised like a Value row: groups of G consecutive channels of one token."""
import math

import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16


def _brute_force_row(x16, bits, G):
    """Scale / zero / codes of one row by the Appendix C equations, one group at a time, with
    Python scalars rounded to fp32 where the quantiser's arithmetic is fp32."""
    f32 = np.float32
    qmax = 2 ** bits - 1
    codes, scales, zeros = [], [], []
    for g in range(len(x16) // G):
        xs = [f32(v) for v in x16[g * G:(g + 1) * G]]
        mn, mx = min(xs), max(xs)
        s32 = f32(f32(mx - mn) / f32(qmax))
        s16 = np.float16(s32)
        if f32(s16) < s32:
            s16 = np.nextafter(s16, np.float16(np.inf))
        if mx == mn:
            s16 = np.float16(abs(mn)) if mn != 0 else np.float16(1)
        inv = f32(f32(1) / f32(s16))
        zero = -int(np.rint(f32(mn * inv)))
        scales.append(s16)
        zeros.append(zero)
        codes += [min(max(int(np.rint(f32(x * inv))) + zero, 0), qmax) for x in xs]
    return np.array(codes, np.uint8), np.array(scales, np.float16), np.array(zeros, np.int16)


@pytest.mark.parametrize("bits,G", [(4, 128), (3, 64), (2, 32), (8, 32)])
def test_rows_match_a_scalar_brute_force(bits, G):
    rng = np.random.default_rng(10 + bits)
    B, H, n = 1, 2, 128
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    K[0, 1, 5, 40:44] = [np.float16(30), np.float16(-25), np.float16(0.5), np.float16(0)]     # a row with a wide group
    mask = np.zeros((B, n), np.uint8)
    mask[0, 9] = 1
    c = O.quantize_kv(K, V, mask, bits, G, 2, key_per_token=True)
    assert c.k_params.shape == (B, H, n, 128 // G) and c.key_per_token
    s, z = O.decode_params(c.k_params)
    for h in range(H):
        for t in (0, 5, 9, 127):
            if mask[0, t]:
                assert not c.k_codes_logical[0, h, t].any()                    # kept row: code 0
                assert np.all(s[0, h, t] == np.float16(1)) and not z[0, h, t].any()   # and an empty group's parameters
                continue
            codes, sc, zr = _brute_force_row(K[0, h, t], bits, G)
            assert np.array_equal(c.k_codes_logical[0, h, t], codes)
            assert np.array_equal(s[0, h, t], sc) and np.array_equal(z[0, h, t], zr)
    # the packed words are the same function of the logical codes as in the per-channel scheme
    assert np.array_equal(O.unpack_k(c.k_codes[0, 0], bits), c.k_codes_logical[0, 0])


def test_values_and_keep_rows_do_not_depend_on_the_key_scheme():
    rng = np.random.default_rng(3)
    K, V = random_fp16(rng, (2, 2, 256, 128)), random_fp16(rng, (2, 2, 256, 128))
    mask = np.zeros((2, 256), np.uint8); mask[0, [0, 77]] = 1; mask[1, 200] = 1
    a = O.quantize_kv(K, V, mask, 4, 64, 3)
    b = O.quantize_kv(K, V, mask, 4, 64, 3, key_per_token=True)
    for f in ("v_codes", "v_params", "keep_k", "keep_v", "keep_idx", "keep_cnt", "keep_mask"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert not np.array_equal(a.k_codes, b.k_codes)


def test_symmetric_tile_transposes_between_the_two_key_schemes():
    """For a symmetric 128 x 128 Key tile with G = 128 the tokens-of-a-channel group of the
    per-channel scheme and the channels-of-a-token group of the per-token scheme hold the same
    numbers, so codes and parameters are each other's transpose."""
    rng = np.random.default_rng(4)
    A = random_fp16(rng, (128, 128)).astype(np.float32)
    S = np.triu(A) + np.triu(A, 1).T
    K = S.astype(np.float16)[None, None]
    assert np.array_equal(K[0, 0], K[0, 0].T)
    V = random_fp16(rng, (1, 1, 128, 128))
    mask = np.zeros((1, 128), np.uint8)
    for bits in (2, 3, 4, 8):
        pc = O.quantize_kv(K, V, mask, bits, 128, 0)
        pt = O.quantize_kv(K, V, mask, bits, 128, 0, key_per_token=True)
        assert np.array_equal(pc.k_codes_logical[0, 0], pt.k_codes_logical[0, 0].T)
        assert np.array_equal(pc.k_params[0, 0, 0], pt.k_params[0, 0, :, 0])


@pytest.mark.parametrize("bits,G", [(4, 128), (4, 32), (2, 64)])
def test_round_trip_bound_and_a_channel_outlier_stays_in_its_token_group(bits, G):
    rng = np.random.default_rng(5)
    K, V = random_fp16(rng, (1, 1, 128, 128)), random_fp16(rng, (1, 1, 128, 128))
    K[0, 0, :, 7] *= 40                                     # an outlier channel, as Keys have
    mask = np.zeros((1, 128), np.uint8)
    c = O.quantize_kv(K, V, mask, bits, G, 0, key_per_token=True)
    Kd, _ = O.effective_kv(c, 0, 0)
    s, _ = O.decode_params(c.k_params[0, 0])                                    # [n, D/G]
    bound = np.repeat(s.astype(np.float64), G, axis=1) / 2 * (1 + 2 ** -8)
    assert np.all(np.abs(Kd - K[0, 0].astype(np.float64)) <= bound)
    # the outlier channel widens only the channel group it is in
    qmax = 2 ** bits - 1
    rng_g = K[0, 0].astype(np.float32).reshape(128, 128 // G, G)
    want = (rng_g.max(axis=2) - rng_g.min(axis=2)) / qmax
    assert np.all(s.astype(np.float32) >= want) and np.all(s.astype(np.float32) <= want * (1 + 2 ** -10) + 1e-7)
    if G < 128:
        assert np.median(s[:, 0].astype(np.float32)) > 5 * np.median(s[:, 1].astype(np.float32))


def test_lossless_grid_attention_matches_a_library_routine():
    """Keys whose every (token, channel group) holds exactly the values offset + step * {0..qmax}
    survive the per-token scheme without error; decode attention over that cache must then equal
    a library softmax attention over the original tensors."""
    rng = np.random.default_rng(6)
    B, H, Hq, n, G, bits = 1, 2, 4, 256, 32, 4
    qmax = 2 ** bits - 1
    step = np.float16(0.125)
    codes = rng.integers(0, qmax + 1, (B, H, n, 128))
    codes.reshape(B, H, n, 128 // G, G)[..., 0] = 0
    codes.reshape(B, H, n, 128 // G, G)[..., 1] = qmax
    off = rng.integers(-8, 8, (B, H, n, 128 // G, 1)) * 0.125 * qmax
    K = (codes.reshape(B, H, n, 128 // G, G) * float(step) + off).reshape(B, H, n, 128).astype(np.float16)
    vcodes = rng.integers(0, qmax + 1, (B, H, n, 128))
    vcodes.reshape(B, H, n, 128 // G, G)[..., 0] = 0
    vcodes.reshape(B, H, n, 128 // G, G)[..., 1] = qmax
    V = (vcodes * 0.25 - 1.0).astype(np.float16)
    mask = np.zeros((B, n), np.uint8); mask[0, [0, 100]] = 1
    K[0, :, 100] = random_fp16(rng, (H, 128)); V[0, :, 100] = random_fp16(rng, (H, 128))
    c = O.quantize_kv(K, V, mask, bits, G, 2, key_per_token=True)
    Kd, Vd = O.effective_kv(c, 0, 1)
    assert np.array_equal(Kd, K[0, 1].astype(np.float64)) and np.array_equal(Vd, V[0, 1].astype(np.float64))
    q = (random_fp16(rng, (B, Hq, 128)).astype(np.float32) * 0.3).astype(np.float16)
    _, lse, out64 = O.decode_attn(q, c, Hq)
    Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(Hq // H, dim=1)
    Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(Hq // H, dim=1)
    qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)[:, :, 0].numpy()
    assert np.allclose(out64, ref, rtol=1e-10, atol=1e-12)
    s = torch.einsum("bhd,bhnd->bhn", qt[:, :, 0], Kt) / math.sqrt(128)
    assert np.allclose(lse, torch.logsumexp(s, dim=-1).numpy(), rtol=1e-6)


def test_static_parameters_per_key_channel_group():
    rng = np.random.default_rng(7)
    B, H, n, G, bits = 2, 2, 256, 64, 4
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    mask = np.zeros((B, n), np.uint8); mask[:, 3] = 1
    K[:, :, 3] *= 100                                       # kept row: must not widen anything
    cal = O.calibrate(O.new_calibration(H), K, V, mask)
    ks, vs = O.static_params(cal, bits, G, key_per_token=True)
    assert ks.shape == (H, 128 // G)
    free = K[:, :, np.arange(n) != 3].astype(np.float32)                        # [B, H, n-1, 128]
    s, z = O.decode_params(ks)
    for h in range(H):
        for g in range(128 // G):
            blk = free[:, h, :, g * G:(g + 1) * G]
            want = (blk.max() - blk.min()) / (2 ** bits - 1)
            assert float(s[h, g]) >= want and float(s[h, g]) <= want * (1 + 2 ** -10)
            assert int(z[h, g]) == -int(np.rint(np.float32(blk.min()) * (np.float32(1) / np.float32(s[h, g]))))
    c = O.quantize_kv_static(K, V, mask, bits, G, 2, ks, vs, key_per_token=True)
    assert np.all(c.k_params == ks[None, :, None, :])
    Kd, _ = O.effective_kv(c, 1, 0)
    bound = np.repeat(s[0].astype(np.float64), G)[None, :] / 2 * (1 + 2 ** -8)
    keep = mask[1] != 0
    assert np.all(np.abs(Kd[~keep] - K[1, 0][~keep].astype(np.float64)) <= bound)
    assert np.array_equal(Kd[keep], K[1, 0][keep].astype(np.float64))


def test_growing_cache_with_per_token_keys_equals_a_prefill():
    rng = np.random.default_rng(8)
    B, H, n0, steps = 1, 2, 200, 70
    K, V = random_fp16(rng, (B, H, n0 + steps, 128)), random_fp16(rng, (B, H, n0 + steps, 128))
    mask = np.zeros((B, n0 + steps), np.uint8); mask[0, [0, 130]] = 1
    gc = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], 4, 32, 4, key_per_token=True)
    for t in range(n0, n0 + steps):
        gc = O.append_token(gc, K[:, :, t], V[:, :, t])
    whole = O.prefill_cache(K, V, mask, 4, 32, 4, key_per_token=True)
    assert gc.n_quant == whole.n_quant == 256 and gc.quant.key_per_token
    for f in ("k_codes", "k_params", "v_codes", "v_params", "keep_idx"):
        assert np.array_equal(getattr(gc.quant, f), getattr(whole.quant, f)), f
    assert np.array_equal(gc.res_k, whole.res_k)
