"""Pins for the oracle's static (calibrated) quantisation (Appendix C, dynamic vs static; Table 1's
setting: global min-max, sink tokens excluded from calibration and quantisation)."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16


def _dequant_static(cache: O.Cache, b, h):
    return O.effective_kv(cache, b, h)


@pytest.mark.parametrize("bits,G", [(4, 128), (3, 64), (2, 32), (8, 128)])
def test_in_range_error_bound_and_clamping(bits, G):
    rng = np.random.default_rng(bits)
    B, H, n = 2, 2, 256
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 14]] = 1
    K[0, :, 0] *= 50; V[0, :, 14] *= 50                          # kept rows are wild: they must not matter
    cal = O.calibrate(O.new_calibration(H), K, V, mask)
    ks, vs = O.static_params(cal, bits, G)
    c = O.quantize_kv_static(K, V, mask, bits, G, 4, ks, vs)
    sk, _ = O.decode_params(ks)
    sv, _ = O.decode_params(vs)
    for b in range(B):
        for h in range(H):
            Kd, Vd = _dequant_static(c, b, h)
            free = mask[b] == 0
            # calibrated on the very data: every free entry is in range, so the round-trip bound holds
            assert np.all(np.abs(Kd[free] - K[b, h][free].astype(np.float64)) <= sk[h].astype(np.float64)[None, :] / 2 * (1 + 2 ** -8))
            bound_v = np.repeat(sv[h].astype(np.float64), G)[None, :] / 2 * (1 + 2 ** -8)
            assert np.all(np.abs(Vd[free] - V[b, h][free].astype(np.float64)) <= bound_v)
            assert np.array_equal(Kd[~free], K[b, h][~free].astype(np.float64))       # kept rows exact
    # values outside the calibrated range clamp to the ends of the code range
    K2 = K.copy(); K2[1, 0, 5, 3] = np.float16(1000); K2[1, 0, 6, 3] = np.float16(-1000)
    c2 = O.quantize_kv_static(K2, V, mask, bits, G, 4, ks, vs)
    assert c2.k_codes_logical[1, 0, 5, 3] == 2 ** bits - 1 and c2.k_codes_logical[1, 0, 6, 3] == 0
    # every group's stored parameter word is the static word
    assert np.all(c.k_params == ks[None, :, None, :]) and np.all(c.v_params == vs[None, :, None, :])


def test_kept_tokens_do_not_move_the_calibration_and_batches_accumulate():
    rng = np.random.default_rng(1)
    K, V = random_fp16(rng, (2, 2, 128, 128)), random_fp16(rng, (2, 2, 128, 128))
    mask = np.zeros((2, 128), np.uint8); mask[:, 7] = 1
    a = O.calibrate(O.new_calibration(2), K, V, mask)
    K2 = K.copy(); K2[:, :, 7] = 999
    b = O.calibrate(O.new_calibration(2), K2, V, mask)
    assert np.array_equal(a.k_min, b.k_min) and np.array_equal(a.k_max, b.k_max)
    free = K[:, :, np.arange(128) != 7].astype(np.float32)
    assert np.array_equal(a.k_min, free.min(axis=(0, 2))) and np.array_equal(a.k_max, free.max(axis=(0, 2)))
    # two batches one after the other = both at once
    two = O.calibrate(O.calibrate(O.new_calibration(2), K[:1], V[:1], mask[:1]), K[1:], V[1:], mask[1:])
    for f in ("k_min", "k_max", "v_min", "v_max"):
        assert np.array_equal(getattr(two, f), getattr(a, f))
    # nothing seen: parameters of an empty group
    ks, vs = O.static_params(O.new_calibration(2), 4, 64)
    s, z = O.decode_params(ks)
    assert np.all(s == np.float16(1)) and not z.any()


def test_one_group_per_channel_static_equals_dynamic():
    """With a single sequence, one head and n == G the dynamic per-channel Key groups ARE the global
    per-channel ranges, so static Keys calibrated on the tensor equal the dynamic ones bit for bit."""
    rng = np.random.default_rng(2)
    K, V = random_fp16(rng, (1, 1, 128, 128)), random_fp16(rng, (1, 1, 128, 128))
    mask = np.zeros((1, 128), np.uint8); mask[0, 3] = 1
    ks, vs = O.static_params(O.calibrate(O.new_calibration(1), K, V, mask), 4, 128)
    st = O.quantize_kv_static(K, V, mask, 4, 128, 2, ks, vs)
    dy = O.quantize_kv(K, V, mask, 4, 128, 2)
    assert np.array_equal(st.k_codes, dy.k_codes) and np.array_equal(st.k_params, dy.k_params)
    # and a Value row whose own range equals the calibrated one gets the dynamic codes
    V2 = V.copy()
    V2[0, 0, 9, 0], V2[0, 0, 9, 1] = V[0, 0][mask[0] == 0].min(), V[0, 0][mask[0] == 0].max()
    st2 = O.quantize_kv_static(K, V2, mask, 4, 128, 2, ks, vs)
    dy2 = O.quantize_kv(K, V2, mask, 4, 128, 2)
    assert np.array_equal(st2.v_codes_logical[0, 0, 9], dy2.v_codes_logical[0, 0, 9])


def test_static_cache_decodes_like_any_other():
    rng = np.random.default_rng(3)
    K = rng.integers(-7, 8, (1, 1, 256, 128)).astype(np.float16)
    V = rng.integers(-7, 8, (1, 1, 256, 128)).astype(np.float16)
    K[0, 0, 0], K[0, 0, 1] = -7, 8
    V[0, 0, 0], V[0, 0, 1] = -7, 8
    mask = np.zeros((1, 256), np.uint8)
    ks, vs = O.static_params(O.calibrate(O.new_calibration(1), K, V, mask), 4, 128)   # range [-7, 8]: scale 1
    c = O.quantize_kv_static(K, V, mask, 4, 128, 1, ks, vs)
    q = (random_fp16(rng, (1, 1, 128)).astype(np.float32) * 0.05).astype(np.float16)
    o = O.decode_attn(q, c, Hq=1)[2][0, 0]
    qt = torch.from_numpy(q[0, 0].astype(np.float64))[None, None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, torch.from_numpy(K.astype(np.float64)),
                                                           torch.from_numpy(V.astype(np.float64)))[0, 0, 0].numpy()
    assert np.abs(o - ref).max() <= 1e-10
