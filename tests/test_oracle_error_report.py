"""Pins for the oracle's quantisation-error report (Section 4.1, Table 1: MSE overall, over the
groups without sink tokens and over the groups that contain one; per-token Keys, per-token Values,
per-channel Keys; dynamic and static)."""
import numpy as np
import pytest

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16


def _loop_report(K, V, cache, sink_mask):
    """The same sums entry by entry with Python scalars, straight from codes and parameter words."""
    B, H, n, D = K.shape
    G, bits = cache.group, cache.bits
    res = {"k": [0.0, 0, 0.0, 0], "v": [0.0, 0, 0.0, 0]}
    for b in range(B):
        for h in range(H):
            ck, cv = O.unpack_k(cache.k_codes[b, h], bits), O.unpack_v(cache.v_codes[b, h], bits)
            sk, zk = O.decode_params(cache.k_params[b, h])
            sv, zv = O.decode_params(cache.v_params[b, h])
            for t in range(n):
                if cache.keep_mask[b, t]:
                    continue
                g0 = (t // G) * G
                k_cls = int(sink_mask[b, t] != 0) if cache.key_per_token else int(sink_mask[b, g0:g0 + G].any())
                v_cls = int(sink_mask[b, t] != 0)
                for c in range(D):
                    if cache.key_per_token:
                        s, z = float(sk[t, c // G]), int(zk[t, c // G])
                    else:
                        s, z = float(sk[t // G, c]), int(zk[t // G, c])
                    e = float(K[b, h, t, c]) - float(np.float32(s) * np.float32(int(ck[t, c]) - z))
                    res["k"][2 * k_cls] += e * e
                    res["k"][2 * k_cls + 1] += 1
                    s, z = float(sv[t, c // G]), int(zv[t, c // G])
                    e = float(V[b, h, t, c]) - float(np.float32(s) * np.float32(int(cv[t, c]) - z))
                    res["v"][2 * v_cls] += e * e
                    res["v"][2 * v_cls + 1] += 1
    return res


@pytest.mark.parametrize("bits,G,kpt", [(4, 32, False), (3, 64, True), (2, 128, False), (8, 64, False)])
def test_against_an_entry_by_entry_loop(bits, G, kpt):
    rng = np.random.default_rng(bits)
    B, H, n = 2, 1, 128
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    keep = np.zeros((B, n), np.uint8); keep[0, 3] = 1
    sinks = np.zeros((B, n), np.uint8); sinks[0, [3, 70]] = 1; sinks[1, 127] = 1
    c = O.quantize_kv(K, V, keep, bits, G, 2, key_per_token=kpt)
    got, ref = O.quant_error(K, V, c, sinks), _loop_report(K, V, c, sinks)
    for name in ("k", "v"):
        assert got[name][1] == ref[name][1] and got[name][3] == ref[name][3]
        assert got[name][0] == pytest.approx(ref[name][0], rel=1e-12)
        assert got[name][2] == pytest.approx(ref[name][2], rel=1e-12)
        assert got[name][1] + got[name][3] == (B * n - 1) * H * 128             # every non-kept entry once


def test_lossless_grid_has_no_error_and_uniform_data_has_the_textbook_noise():
    rng = np.random.default_rng(1)
    n, G, bits = 256, 128, 4
    grid = rng.integers(0, 16, (1, 1, n, 128))
    grid[0, 0, 0::G, :] = 0; grid[0, 0, 1::G, :] = 15        # every Key group spans the grid
    grid[0, 0, :, 0] = 0; grid[0, 0, :, 1] = 15              # every Value group too
    X = (grid * 0.5 - 2.0).astype(np.float16)
    none = np.zeros((1, n), np.uint8)
    r = O.quant_error(X, X, O.quantize_kv(X, X, none, bits, G, 0), none)
    assert r["k"][0] == 0.0 and r["v"][0] == 0.0 and r["k"][1] == r["v"][1] == n * 128
    # uniform data: the rounding error is uniform in [-scale/2, scale/2], variance scale^2 / 12
    U = rng.uniform(-1, 1, (1, 4, 1024, 128)).astype(np.float16)
    none = np.zeros((1, 1024), np.uint8)
    c = O.quantize_kv(U, U, none, bits, G, 0)
    r = O.quant_error(U, U, c, none)
    for name, params in (("k", c.k_params), ("v", c.v_params)):
        s, _ = O.decode_params(params)
        want = float((s.astype(np.float64) ** 2).mean()) / 12
        assert r[name][0] / r[name][1] == pytest.approx(want, rel=0.03)


def test_the_two_classes_follow_the_group_geometry_of_each_scheme():
    """A sink token with an expanded range (quantised, not kept) hurts the 63 other tokens of its
    per-channel Key group and nobody else; per token it only hurts itself."""
    rng = np.random.default_rng(2)
    n, G = 256, 64
    K, V = random_fp16(rng, (1, 2, n, 128)), random_fp16(rng, (1, 2, n, 128))
    K[0, :, 70] *= np.float16(30); V[0, :, 70] *= np.float16(30)
    none = np.zeros((1, n), np.uint8)
    sinks = none.copy(); sinks[0, 70] = 1
    pc = O.quant_error(K, V, O.quantize_kv(K, V, none, 4, G, 0), sinks)
    pt = O.quant_error(K, V, O.quantize_kv(K, V, none, 4, G, 0, key_per_token=True), sinks)
    assert pc["k"][3] == 2 * G * 128 and pc["k"][1] == 2 * (n - G) * 128          # one token group of each head
    assert pt["k"][3] == 2 * 128 and pc["v"][3] == 2 * 128                        # one row of each head
    mse = lambda r, i: r[i] / r[i + 1]
    assert mse(pc["k"], 2) > 10 * mse(pc["k"], 0)            # the shared range costs the whole group
    # per token the damage stays in the sink's own rows: the other rows are as good as without it
    clean = O.quant_error(K, V, O.quantize_kv(K, V, sinks, 4, G, 1, key_per_token=True), sinks)
    assert mse(pt["k"], 0) == pytest.approx(mse(clean["k"], 0), rel=1e-12) and clean["k"][3] == 0
    # keeping the sink (Algorithm 1) brings the per-channel groups back to the level of the others
    kept = O.quant_error(K, V, O.quantize_kv(K, V, sinks, 4, G, 1), sinks)
    assert kept["k"][3] == 2 * (G - 1) * 128
    assert mse(kept["k"], 2) < 1.3 * mse(kept["k"], 0)


def test_static_range_excluding_the_sinks_lowers_the_error_of_everyone_else():
    """Table 1's static rows: with the sinks in the calibration the one global range is wide for
    every token; excluding them from calibration and quantisation shrinks it."""
    rng = np.random.default_rng(3)
    n, G = 256, 128
    K, V = random_fp16(rng, (1, 2, n, 128)), random_fp16(rng, (1, 2, n, 128))
    K[0, :, 0] *= np.float16(30); V[0, :, 0] *= np.float16(30)
    none = np.zeros((1, n), np.uint8)
    sinks = none.copy(); sinks[0, 0] = 1
    ks, vs = O.static_params(O.calibrate(O.new_calibration(2), K, V, none), 4, G)
    with_sinks = O.quant_error(K, V, O.quantize_kv_static(K, V, none, 4, G, 1, ks, vs), sinks)
    ks2, vs2 = O.static_params(O.calibrate(O.new_calibration(2), K, V, sinks), 4, G)
    without = O.quant_error(K, V, O.quantize_kv_static(K, V, sinks, 4, G, 1, ks2, vs2), sinks)
    for name in ("k", "v"):
        overall = (with_sinks[name][0] + with_sinks[name][2]) / (with_sinks[name][1] + with_sinks[name][3])
        assert without[name][0] / without[name][1] < overall / 20
