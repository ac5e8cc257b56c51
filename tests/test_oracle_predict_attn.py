"""Pins for the oracle's sink prediction, decode attention and memory accounting."""
import math

import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import constants, synth
from tests.helpers import golden_rows, random_fp16


# ------------------------------------------------------------------------------ prediction
def test_worked_example_positions_are_recovered():
    (name, positions), = golden_rows("worked_example_sinks.txt")
    expected = [int(p) for p in positions.split(",")]
    w = synth.WORKLOADS["cfg0_kvsink"]
    assert synth.sink_positions(w)[0].tolist() == expected
    H = synth.make_hidden(w).numpy()
    for channels in (w.channels, w.channels[:1], w.channels[1:]):      # one channel is enough
        idx, mask = O.predict_sinks(H, channels, 2, 0)
        assert idx.tolist() == [expected]
        assert np.nonzero(mask[0])[0].tolist() == expected
    # Preserve-First-N alone: k = 0 keeps exactly the first N tokens
    idx, mask = O.predict_sinks(H, w.channels, 0, 4)
    assert idx.shape == (1, 0) and np.nonzero(mask[0])[0].tolist() == [0, 1, 2, 3]
    # union of both policies
    idx, mask = O.predict_sinks(H, w.channels, 2, 4)
    assert np.nonzero(mask[0])[0].tolist() == [0, 1, 2, 3, 14]


def test_topk_against_python_sort_with_ties_and_permutation():
    rng = np.random.default_rng(0)
    B, n, d = 3, 97, 16
    H = random_fp16(rng, (B, n, d))
    H[:, :, 5] = np.round(H[:, :, 5] * 2) / 2                          # many equal magnitudes
    H[1, 40, 5], H[1, 41, 5] = 7.0, -7.0                               # an exact tie at the top
    for k in (1, 2, 5, 20):
        idx, mask = O.predict_sinks(H, [5], k, 0)
        for b in range(B):
            ranked = sorted(range(n), key=lambda i: (-abs(float(H[b, i, 5])), i))
            assert idx[b].tolist() == sorted(ranked[:k])
            assert mask[b].sum() == k
    assert 40 in O.predict_sinks(H, [5], 1, 0)[0][1]                   # tie -> lower token index
    # moving tokens moves the prediction identically (unique magnitudes here)
    Hu = random_fp16(rng, (1, n, d))
    Hu[0, :, 3] = (rng.permutation(n) + 1).astype(np.float16) * np.where(rng.random(n) < 0.5, -1, 1)
    perm = rng.permutation(n)
    idx0 = O.predict_sinks(Hu, [3], 6, 0)[0][0]
    idx1 = O.predict_sinks(Hu[:, perm], [3], 6, 0)[0][0]
    assert sorted(perm[idx1].tolist()) == idx0.tolist()
    # several channels: the score of a token is its largest listed magnitude
    Hm = np.zeros((1, 8, 4), np.float16)
    Hm[0, 2, 0], Hm[0, 6, 1], Hm[0, 4, 2] = 5, -9, 100                 # channel 2 is not listed
    Hm[0, 3, 0], Hm[0, 3, 1] = 4, -4                                   # largest, not summed: 4 < 5 although 4 + 4 > 5
    assert O.predict_sinks(Hm, [0, 1], 2, 0)[0].tolist() == [[2, 6]]
    assert O.predict_sinks(Hm, [0, 1], 3, 0)[0].tolist() == [[2, 3, 6]]


def test_model_constant_table_matches_the_paper():
    rows = golden_rows("stable_outlier_table.txt")
    assert len(rows) == len(constants.MODEL_TABLE) == 7
    for name, layers, l_e, hidden, channels in rows:
        assert constants.MODEL_TABLE[name] == (int(layers), int(l_e), int(hidden),
                                               tuple(int(c) for c in channels.split(",")))
    assert set(synth.LLAMA2_7B_OUTLIER_CHANNELS) == set(constants.MODEL_TABLE["LLaMA2-7B"][3])


# ------------------------------------------------------------------------------ attention
def _sdpa64(q, K, V):
    """Library attention in fp64: q [D], K/V [n, D]."""
    qt = torch.from_numpy(q.astype(np.float64))[None, None, None, :]
    Kt = torch.from_numpy(K.astype(np.float64))[None, None]
    Vt = torch.from_numpy(V.astype(np.float64))[None, None]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)[0, 0, 0].numpy()


def _small_case(seed=0, B=2, H=2, n=256, bits=4, G=128, kind="normal", keep=((0, 14), (0, 5, 100))):
    rng = np.random.default_rng(seed)
    K, V = random_fp16(rng, (B, H, n, 128), kind), random_fp16(rng, (B, H, n, 128), kind)
    mask = np.zeros((B, n), np.uint8)
    for b in range(B):
        mask[b, list(keep[b % len(keep)])] = 1
    q = random_fp16(rng, (B, H, 128))
    return K, V, mask, q


def test_attention_row_properties():
    rng = np.random.default_rng(1)
    Kp, Vp = rng.standard_normal((300, 128)), rng.standard_normal((300, 128))
    q = random_fp16(rng, (128,))
    o, lse, p = O.attention_row(q, Kp, Vp)
    assert abs(p.sum() - 1) < 1e-12 and np.all(p > 0)
    assert np.allclose(o, _sdpa64(q, Kp, Vp), rtol=0, atol=1e-12)
    s = Kp @ q.astype(np.float64) / math.sqrt(128)
    assert abs(lse - math.log(np.exp(s).sum())) < 1e-10
    # identical value rows: the output is that row whatever the query
    row = rng.standard_normal(128)
    assert np.allclose(O.attention_row(q, Kp, np.tile(row, (300, 1)))[0], row, atol=1e-12)
    # zero query: uniform weights, the output is the mean value row
    assert np.allclose(O.attention_row(np.zeros(128, np.float16), Kp, Vp)[0], Vp.mean(0), atol=1e-12)
    # the sum over tokens splits into a sink part and a non-sink part
    S = np.zeros(300, bool)
    S[[0, 14, 77]] = True
    assert np.allclose(p[S] @ Vp[S] + p[~S] @ Vp[~S], o, atol=1e-12)
    # a streaming (online-softmax) evaluation in chunks agrees with the two-pass one
    m, l, acc = -np.inf, 0.0, np.zeros(128)
    for lo in range(0, 300, 64):
        sc = s[lo:lo + 64]
        m2 = max(m, sc.max())
        acc = acc * math.exp(m - m2) + np.exp(sc - m2) @ Vp[lo:lo + 64]
        l = l * math.exp(m - m2) + np.exp(sc - m2).sum()
        m = m2
    assert np.allclose(acc / l, o, atol=1e-12)


def test_all_tokens_kept_equals_textbook_attention_on_the_fp16_inputs():
    K, V, _, q = _small_case(n=128)
    mask = np.ones((2, 128), np.uint8)
    cache = O.quantize_kv(K, V, mask, 2, 32, keep_cap=128)
    out16, lse, out64 = O.decode_attn(q, cache, Hq=2)
    for b in range(2):
        for h in range(2):
            assert np.allclose(out64[b, h], _sdpa64(q[b, h], K[b, h], V[b, h]), atol=1e-12)
    assert np.array_equal(out16, out64.astype(np.float16))


@pytest.mark.parametrize("G", [32, 128])
def test_lossless_grid_cache_equals_textbook_attention(G):
    """K and V on the 4-bit integer grid quantise without loss, so the whole chain
    quantise -> pack -> unpack -> dequantise -> attend must give exact attention."""
    rng = np.random.default_rng(2)
    B, H, n = 1, 2, 256
    K = rng.integers(-6, 10, (B, H, n, 128)).astype(np.float16)
    V = rng.integers(0, 16, (B, H, n, 128)).astype(np.float16)
    K[:, :, 0::G], K[:, :, 1::G] = -6, 9                              # every K group spans the grid
    V[..., 0::G], V[..., 1::G] = 0, 15                                # every V group too
    mask = np.zeros((B, n), np.uint8)
    mask[0, [2, 14]] = 1
    K[0, :, [2, 14]] = 0.37                                           # kept rows are off the grid
    q = (random_fp16(rng, (B, H, 128)) * np.float16(0.1)).astype(np.float16)
    cache = O.quantize_kv(K, V, mask, 4, G, keep_cap=2)
    _, _, out64 = O.decode_attn(q, cache, Hq=H)
    for h in range(H):
        assert np.allclose(out64[0, h], _sdpa64(q[0, h], K[0, h], V[0, h]), atol=1e-12)


def test_lossless_grid_with_isolated_outliers_equals_textbook_attention():
    rng = np.random.default_rng(3)
    B, H, n = 2, 2, 256
    K = rng.integers(0, 8, (B, H, n, 128)).astype(np.float16)
    V = rng.integers(0, 8, (B, H, n, 128)).astype(np.float16)
    K[:, :, 0::128], K[:, :, 1::128] = 0, 7
    V[..., 0], V[..., 1] = 0, 7
    for X in (K, V):                                                  # ~1% huge entries, not on rows 0/1 or channels 0/1,
        for b in range(B):                                            # elsewhere in every (sequence, head)
            for h in range(H):
                t, c = rng.integers(2, 128, 300), rng.integers(2, 128, 300)
                X[b, h, t + 128 * rng.integers(0, 2, 300), c] = 500.0
    mask = np.zeros((B, n), np.uint8)
    mask[1, 77] = 1
    K[1, :, 77], V[1, :, 77] = 0.37, -1000.0                          # a kept row is off the grid and never isolated
    q = (random_fp16(rng, (B, H, 128)) * np.float16(0.01)).astype(np.float16)
    live = np.ones((B, 1, n, 1), bool)
    live[1, 0, 77] = False
    frac = min(int(((X == 500) & live).sum()) for X in (K, V)) / float(live.sum() * H * 128)
    cache = O.quantize_kv(K, V, mask, 3, 128, keep_cap=1, sparse_frac=frac)
    assert cache.k_tau == cache.v_tau == int(np.float16(500).view(np.uint16))
    assert len(cache.k_col) == int((K == 500).sum()) and len(cache.v_col) == int((V == 500).sum())
    _, _, out64 = O.decode_attn(q, cache, Hq=H)
    for b in range(B):
        for h in range(H):
            assert np.allclose(out64[b, h], _sdpa64(q[b, h], K[b, h], V[b, h]), atol=1e-12), (b, h)


def test_sparse_capacity_is_the_larger_of_the_two_counts_and_may_be_met_exactly():
    rng = np.random.default_rng(5)
    K, V = random_fp16(rng, (1, 1, 128, 128)), random_fp16(rng, (1, 1, 128, 128))
    K[0, 0, 3, :4] = 900.0                                            # 4 isolated Key entries ...
    V[0, 0, 5, :9] = 900.0                                            # ... and 9 isolated Value entries
    mask = np.zeros((1, 128), np.uint8)
    tau = int(np.float16(900).view(np.uint16))
    for cap, want in ((9, O.STATUS_OK), (8, O.STATUS_CAPACITY), (4, O.STATUS_CAPACITY), (100, O.STATUS_OK)):
        c = O.quantize_kv(K, V, mask, 4, 128, keep_cap=0, sparse_frac=0.01, sparse_cap=cap, taus=(tau, tau))
        assert (len(c.k_col), len(c.v_col)) == (4, 9)
        assert c.status == want, cap


def test_quantised_attention_error_shrinks_with_bit_width():
    K, V, mask, q = _small_case(seed=7)
    errs = {}
    for bits in (2, 3, 4, 8):
        cache = O.quantize_kv(K, V, mask, bits, 64, keep_cap=3)
        _, _, out64 = O.decode_attn(q, cache, Hq=2)
        err = 0.0
        for b in range(2):
            for h in range(2):
                ref = _sdpa64(q[b, h], K[b, h], V[b, h])
                err = max(err, np.abs(out64[b, h] - ref).max() / np.abs(ref).max())
        errs[bits] = err
    assert errs[8] < errs[4] < errs[3] < errs[2] and errs[4] < 0.3 and errs[8] < 0.02


def test_gqa_mapping():
    K, V, mask, _ = _small_case(H=2)
    rng = np.random.default_rng(5)
    q = random_fp16(rng, (2, 8, 128))                                 # 8 query heads over 2 KV heads
    cache = O.quantize_kv(K, V, mask, 4, 128, keep_cap=3)
    out_gqa = O.decode_attn(q, cache, Hq=8)[2]
    # duplicating each KV head 4 times and running plain multi-head attention is the same thing
    cache_dup = O.quantize_kv(np.repeat(K, 4, axis=1), np.repeat(V, 4, axis=1), mask, 4, 128, keep_cap=3)
    out_mha = O.decode_attn(q, cache_dup, Hq=8)[2]
    assert np.array_equal(out_gqa, out_mha)
    # restricting to a list of pairs computes just those rows
    sub = O.decode_attn(q, cache, Hq=8, pairs=[(1, 5)])[2]
    assert np.array_equal(sub[1, 5], out_gqa[1, 5]) and not sub[0].any()


# ------------------------------------------------------------------------------ accounting
def test_memory_table_of_appendix_f():
    MB = 2.0 ** 20
    for name, layers, width, base, k1, k5, k20 in golden_rows("appendix_f_memory.txt"):
        layers, width = int(layers), int(width)
        assert O.kv_cache_bytes(4096, layers, width, bits=2) / MB == float(base)
        for k, printed in ((1, k1), (5, k5), (20, k20)):
            assert abs(O.preserved_token_bytes(k, layers, width) / MB - float(printed)) <= 0.0051


def test_average_bits_column_of_table_2():
    rows = {float(r[0]): (float(r[1]), float(r[2])) for r in golden_rows("table2_avg_bits.txt")}
    base_low = rows[0.0][0]
    for frac, (low, high) in rows.items():
        assert abs(O.average_bits(2, frac) - base_low - (low - base_low)) <= 0.0081
        assert O.average_bits(2, frac) <= high
