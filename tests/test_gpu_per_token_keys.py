"""Parity of the per-token Key scheme (desc.key_per_token; Section 5.1) with the oracle: codes,
parameter words and kept rows bit-exact, attention outputs within 2e-3 - dynamic, static and in a
growing cache, over every shape the descriptor check lets through."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_growing import assert_growing_equal, check_decode
from tests.test_gpu_parity import DEV, OUT_TOL, assert_cache_equal, hip_decode, row_rel_err, u32

pytestmark = pytest.mark.gpu

# the last three (heads x channel groups > 8) have no room in the matrix-core score tile: stream kernel
SHAPES = [(128, 1), (128, 2), (128, 4), (128, 8), (64, 1), (64, 2), (64, 4), (32, 1), (32, 2), (64, 8), (32, 4),
          (32, 8)]


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _inputs(rng, B, H, n, Hq, v_kind="wide"):
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128), v_kind)
    K[:, :, :, [3, 77]] *= np.float16(10)                 # outlier channels, as Keys have
    K += np.float16(0.75)                                 # and an offset: zero points far from the middle
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 14, min(500, n - 2)]] = 1
    if B > 1:
        mask[1, [0, 1, 2, 3, n - 1]] = 1
    return K, V, mask, random_fp16(rng, (B, Hq, 128))


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("G,rep", SHAPES)
def test_quantize_and_decode(bits, G, rep):
    rng = np.random.default_rng(1000 * bits + G + rep)
    B, H, n, cap = 2, 2, 1152, 6                          # 9 Value tiles: uneven splits
    K, V, mask, q = _inputs(rng, B, H, n, H * rep)
    desc = kb.make_desc(B, n, H * rep, H, bits, G, cap, key_per_token=True)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(mask), cache, ws)
    torch.cuda.synchronize()
    ref = O.quantize_kv(K, V, mask, bits, G, cap, key_per_token=True)
    assert_cache_equal(cache, ref)
    out, lse = hip_decode(desc, cache, ws, q)
    _, ref_lse, ref64 = O.decode_attn(q, ref, Hq=H * rep)
    assert row_rel_err(out, ref64) <= OUT_TOL
    assert np.abs(lse - ref_lse).max() <= 1e-3


@pytest.mark.parametrize("bits,G,rep,B,H,n", [
    (4, 128, 1, 8, 32, 512),      # one workgroup per (sequence, head): finished in one kernel
    (4, 64, 4, 1, 1, 4096),       # one (sequence, head): many parts, the combine kernel finishes
    (2, 32, 2, 1, 2, 2048),
    (3, 128, 8, 1, 1, 1280),
    (4, 32, 8, 1, 1, 4096),       # stream kernel, two groups of four heads, many parts
])
def test_single_part_and_many_parts(bits, G, rep, B, H, n):
    rng = np.random.default_rng(bits + G + n)
    K, V, mask, q = _inputs(rng, B, H, n, H * rep)
    desc = kb.make_desc(B, n, H * rep, H, bits, G, 5, key_per_token=True)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(mask), cache, ws)
    out, lse = hip_decode(desc, cache, ws, q)
    pairs = [(b, hq) for b in range(min(B, 2)) for hq in sorted({0, H * rep - 1})]
    ref = O.quantize_kv(K[:2], V[:2], mask[:2], bits, G, 5, key_per_token=True)
    _, ref_lse, ref64 = O.decode_attn(q[:2], ref, Hq=H * rep, pairs=pairs)
    for b, hq in pairs:
        assert row_rel_err(out[b:b + 1, hq:hq + 1], ref64[b:b + 1, hq:hq + 1]) <= OUT_TOL
        assert abs(lse[b, hq] - ref_lse[b, hq]) <= 1e-3


def test_degenerate_rows_and_everything_kept():
    rng = np.random.default_rng(3)
    B, H, n = 2, 2, 256
    K, V = random_fp16(rng, (B, H, n, 128)), random_fp16(rng, (B, H, n, 128))
    K[0, 0, 5] = np.float16(2.5)                          # a constant row
    K[0, 1, 6] = 0                                        # a zero row
    K[1, 0, 7, :64] = np.float16(-3)                      # one constant channel group
    mask = np.zeros((B, n), np.uint8)
    mask[1] = 1                                           # sequence 1: every token kept (capacity exceeded)
    mask[0, 9] = 1
    q = random_fp16(rng, (B, H, 128))
    desc = kb.make_desc(B, n, H, H, 4, 64, 4, key_per_token=True)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv(desc, dev(K), dev(V), dev(mask), cache, ws)
    torch.cuda.synchronize()
    ref = O.quantize_kv(K, V, mask, 4, 64, 4, key_per_token=True)
    assert ref.status == O.STATUS_CAPACITY
    assert_cache_equal(cache, ref)
    out, _ = hip_decode(desc, cache, ws, q)
    ref64 = O.decode_attn(q, ref, Hq=H)[2]
    assert row_rel_err(out[:1], ref64[:1]) <= OUT_TOL     # sequence 0 is an ordinary one


@pytest.mark.parametrize("bits,G,rep", [(4, 128, 1), (3, 64, 4), (2, 32, 2), (4, 32, 4), (8, 64, 2)])
def test_static_parameters(bits, G, rep):
    rng = np.random.default_rng(50 + bits)
    B, H, n, cap = 2, 3, 1152, 6
    # (one global Value range: a heavy-tailed V would round almost every entry to zero, and an
    # output row far below the quantisation step is not what the 2e-3 bar is about)
    K, V, mask, q = _inputs(rng, B, H, n, H * rep, "normal")
    K[0, :, 0] *= np.float16(40)                          # a wild kept row: must not count
    desc = kb.make_desc(B, n, H * rep, H, bits, G, cap, key_per_token=True)
    calib = kb.alloc_calibration(desc, DEV)
    kb.kvs_calibrate(desc, dev(K), dev(V), dev(mask), calib)
    ks, vs = kb.kvs_static_params(desc, calib)
    torch.cuda.synchronize()
    ref_ks, ref_vs = O.static_params(O.calibrate(O.new_calibration(H), K, V, mask), bits, G, key_per_token=True)
    assert ks.shape == (H, 128 // G)
    assert np.array_equal(u32(ks), ref_ks) and np.array_equal(u32(vs), ref_vs)
    Kt, Vt, _, _ = _inputs(rng, B, H, n, H * rep, "normal")
    Kt[1, 2, 100, 5] = np.float16(3000)                   # outside the calibrated range
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_kv_static(desc, dev(Kt), dev(Vt), dev(mask), ks, vs, cache, ws)
    torch.cuda.synchronize()
    ref = O.quantize_kv_static(Kt, Vt, mask, bits, G, cap, ref_ks, ref_vs, key_per_token=True)
    assert_cache_equal(cache, ref)
    out, lse = hip_decode(desc, cache, ws, q)
    _, ref_lse, ref64 = O.decode_attn(q, ref, Hq=H * rep)
    assert row_rel_err(out, ref64) <= OUT_TOL
    assert np.abs(lse - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("bits,G,rep,n0", [(4, 128, 1, 300), (3, 64, 2, 257), (2, 32, 1, 100), (3, 64, 8, 200), (8, 32, 2, 300)])
def test_growing_cache(bits, G, rep, n0):
    rng = np.random.default_rng(bits * 7 + n0)
    B, H, n_cap, cap, n1 = 2, 2, 640, 6, n0 + 140
    K, V = random_fp16(rng, (B, H, n1, 128)), random_fp16(rng, (B, H, n1, 128))
    K[:, :, :, [7, 90]] *= np.float16(8)
    mask = np.zeros((B, n1), np.uint8)
    mask[0, [0, 14]] = 1
    mask[1, n0 - 2] = 1
    desc = kb.make_desc(B, n_cap, H * rep, H, bits, G, cap, key_per_token=True)
    cache, ws = kb.alloc_cache(desc, DEV), kb.alloc_workspace(desc, DEV)
    kb.kvs_quantize_prefix(desc, dev(K[:, :, :n0]), dev(V[:, :, :n0]), dev(mask[:, :n0]), n0, cache, ws)
    torch.cuda.synchronize()
    gc = O.prefill_cache(K[:, :, :n0], V[:, :, :n0], mask[:, :n0], bits, G, cap, key_per_token=True)
    assert_growing_equal(desc, cache, gc)
    q = random_fp16(rng, (B, H * rep, 128))
    check_decode(desc, cache, ws, q, gc, H * rep)
    block_end = (n0 // 128 + 1) * 128
    checkpoints = {block_end - 1, block_end, block_end + 1, n1}
    for t in range(n0, n1):
        kb.kvs_append_kv(desc, dev(K[:, :, t]), dev(V[:, :, t]), t, cache, ws)
        gc = O.append_token(gc, K[:, :, t], V[:, :, t])
        if t + 1 in checkpoints:
            torch.cuda.synchronize()
            assert_growing_equal(desc, cache, gc)
            check_decode(desc, cache, ws, q, gc, H * rep)
