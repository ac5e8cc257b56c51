"""Parity of kvs_quant_error with the oracle's report: counts exact, sums of squared errors to
1e-10 relative (both sides form every squared difference in fp64 from the same fp32 dequantised
value; only the order of the fp64 additions differs)."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _close(got, ref):
    for name in ("k", "v"):
        assert got[name][1] == ref[name][1] and got[name][3] == ref[name][3], name
        for i in (0, 2):
            assert got[name][i] == pytest.approx(ref[name][i], rel=1e-10, abs=1e-300), (name, i)


@pytest.mark.parametrize("bits,G,kpt", [(4, 128, False), (3, 64, False), (2, 32, False), (4, 64, True), (3, 32, True),
                                        (2, 128, True), (8, 64, False), (8, 32, True)])
def test_report_matches_the_oracle(bits, G, kpt):
    rng = np.random.default_rng(bits * 10 + G + kpt)
    B, H, n, cap = 2, 3, 640, 3
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    V *= np.exp(rng.uniform(-3, 3, (B, H, n, 1))).astype(np.float16)     # row norms over a wide range
    K[:, :, :, [5, 99]] *= np.float16(7)
    K[0, :, 14] *= np.float16(25); V[0, :, 14] *= np.float16(25)          # a quantised sink with a wide range
    keep = np.zeros((B, n), np.uint8); keep[0, 0] = 1; keep[1, [200, 639]] = 1
    sinks = np.zeros((B, n), np.uint8); sinks[0, [0, 14]] = 1; sinks[1, [200, 333]] = 1
    desc = kb.make_desc(B, n, H, H, bits, G, cap, key_per_token=kpt)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(keep), cache, ws)
    got = kb.kvs_quant_error(desc, dev(K), dev(V), cache, dev(sinks))
    ref = O.quant_error(K, V, O.quantize_kv(K, V, keep, bits, G, cap, key_per_token=kpt), sinks)
    _close(got, ref)
    # a second call overwrites the report (nothing accumulates across calls)
    _close(kb.kvs_quant_error(desc, dev(K), dev(V), cache, dev(sinks)), ref)
    # no flagged token: everything is in the first class
    none = kb.kvs_quant_error(desc, dev(K), dev(V), cache, dev(np.zeros_like(sinks)))
    assert none["k"][3] == 0 and none["v"][3] == 0 and none["k"][2] == 0.0
    assert none["k"][0] == pytest.approx(ref["k"][0] + ref["k"][2], rel=1e-10)


def test_report_on_a_static_cache_and_on_an_all_kept_sequence():
    rng = np.random.default_rng(4)
    B, H, n, bits, G, cap = 2, 2, 256, 4, 128, 256
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    keep = np.zeros((B, n), np.uint8); keep[1] = 1                         # sequence 1 entirely in fp16
    sinks = np.zeros((B, n), np.uint8); sinks[0, 7] = 1
    desc = kb.make_desc(B, n, H, H, bits, G, cap)
    calib = kb.alloc_calibration(desc, DEV)
    kb.kvs_calibrate(desc, dev(K), dev(V), dev(keep), calib)
    ks, vs = kb.kvs_static_params(desc, calib)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv_static(desc, dev(K), dev(V), dev(keep), ks, vs, cache, ws)
    got = kb.kvs_quant_error(desc, dev(K), dev(V), cache, dev(sinks))
    rks, rvs = O.static_params(O.calibrate(O.new_calibration(H), K, V, keep), bits, G)
    ref = O.quant_error(K, V, O.quantize_kv_static(K, V, keep, bits, G, cap, rks, rvs), sinks)
    _close(got, ref)
    assert got["k"][1] + got["k"][3] == n * H * 128                        # only sequence 0 is counted
