"""Pins for the oracle's quantiser, packer and keep-row logic: closed forms, invariants,
special cases and brute force.  None of these re-types the oracle's formulas; each checks a
consequence that a wrong sign, index, rounding or transposition would break."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16

BITS = [2, 3, 4, 8]
GROUPS = [32, 64, 128]


def _all_fp16_sorted():
    v = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)   # +0 .. max finite
    return v


def test_round_up_to_fp16_matches_brute_force_search():
    rng = np.random.default_rng(1)
    table = _all_fp16_sorted()
    x = np.concatenate([
        np.exp(rng.uniform(np.log(1e-9), np.log(6e4), 20000)),
        table[rng.integers(0, len(table), 2000)],                        # exactly representable
        table[1:2001] * (1 + 1e-7), table[1:2001] * (1 - 1e-7),
    ]).astype(np.float32)
    got = O.fp32_to_fp16_round_up(x).astype(np.float64)
    idx = np.searchsorted(table, x.astype(np.float64), side="left")   # first fp16 >= x
    assert np.array_equal(got, table[idx])


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("kind", ["normal", "wide", "positive", "tiny"])
def test_scale_is_tight_upper_rounding_of_range_over_qmax(bits, kind):
    rng = np.random.default_rng(bits)
    x = random_fp16(rng, (500, 16), kind)
    mn, mx = x.min(1).astype(np.float32), x.max(1).astype(np.float32)
    scale_h, zero = O.group_params(mn, mx, np.full(500, 16), bits)
    qmax = 2 ** bits - 1
    for i in range(500):
        if mx[i] == mn[i]:
            continue
        exact = (Fraction(float(mx[i])) - Fraction(float(mn[i]))) / qmax
        exact = max(exact, abs(Fraction(float(mn[i]))) / 32766)          # the int16 bound on the zero point
        s = Fraction(float(scale_h[i]))
        below = Fraction(float(np.nextafter(scale_h[i], np.float16(0))))
        assert s >= exact * (1 - Fraction(1, 2 ** 23))
        assert below < exact * (1 + Fraction(1, 2 ** 23))
        # zero is the rounded position of the minimum, with the sign the zero equation gives it
        assert abs(Fraction(int(zero[i])) + Fraction(float(mn[i])) / s) <= Fraction(1, 2) + Fraction(1, 256)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("G", GROUPS)
@pytest.mark.parametrize("kind", ["normal", "wide", "positive"])
def test_round_trip_error_at_most_half_scale(bits, G, kind):
    rng = np.random.default_rng(10 * bits + G)
    n, D = 256, 128
    qmax = 2 ** bits - 1
    for which in ("k", "v"):
        X = random_fp16(rng, (n, D), kind)
        masked = np.zeros((n, D), bool)
        masked[rng.integers(0, n, 5)] = True                      # some kept rows
        masked |= rng.random((n, D)) < 0.01                       # some isolated entries
        if which == "k":
            codes, s, z = O.quantize_k_head(X, masked, bits, G)
            S = np.repeat(s, G, axis=0)
            Z = np.repeat(z, G, axis=0)
        else:
            codes, s, z = O.quantize_v_head(X, masked, bits, G)
            S = np.repeat(s, G, axis=1)
            Z = np.repeat(z, G, axis=1)
        assert codes.min() >= 0 and codes.max() <= qmax
        assert np.all(codes[masked] == 0)
        xd = O.dequantize_entries(codes, S, Z).astype(np.float64)
        err = np.abs(xd - X.astype(np.float64))
        bound = S.astype(np.float64) / 2 * (1 + 2.0 ** -8)
        assert np.all(err[~masked] <= bound[~masked])
        # exact zeros stay exact whenever 0 lies inside the group's range (it always does
        # for a sign-mixed group)
        zeros = (X == 0) & ~masked
        assert np.all(xd[zeros] == 0) or kind == "positive"


@pytest.mark.parametrize("bits", BITS)
def test_group_min_maps_to_code_zero_and_max_to_top_codes(bits):
    rng = np.random.default_rng(3)
    X = random_fp16(rng, (128, 128), "normal")
    qmax = 2 ** bits - 1
    codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), bits, 64)
    for g in range(2):
        blk, cb = X[64 * g:64 * g + 64], codes[64 * g:64 * g + 64]
        assert np.all(cb[blk.argmin(0), np.arange(128)] == 0)
        top = cb[blk.argmax(0), np.arange(128)]
        assert np.all((top == qmax) | (top == qmax - 1))
    # monotone: a larger value in a group never gets a smaller code
    order = np.argsort(X[:64, 7].astype(np.float32), kind="stable")
    assert np.all(np.diff(codes[:64, 7][order].astype(int)) >= 0)


def test_constant_group_is_reproduced_exactly():
    for value in (3.25, -0.0123, 0.0, 60000.0, -5.96e-8):
        X = np.full((64, 128), value, np.float16)
        for bits in BITS:
            for fn, G in ((O.quantize_k_head, 32), (O.quantize_v_head, 64)):
                codes, s, z = fn(X, np.zeros_like(X, bool), bits, G)
                rep = (G, 0) if fn is O.quantize_k_head else (G, 1)
                xd = O.dequantize_entries(codes, np.repeat(s, rep[0], rep[1]), np.repeat(z, rep[0], rep[1]))
                assert np.array_equal(xd.astype(np.float16).view(np.uint16) & 0x7FFF,
                                      X.view(np.uint16) & 0x7FFF)
                assert np.array_equal(xd, X.astype(np.float32))


def test_fully_masked_group_has_unit_params_and_zero_codes():
    rng = np.random.default_rng(4)
    X = random_fp16(rng, (128, 128))
    masked = np.zeros((128, 128), bool)
    masked[:64] = True                                             # the whole first token group kept
    codes, s, z = O.quantize_k_head(X, masked, 4, 64)
    assert np.all(codes[:64] == 0) and np.all(s[0] == np.float16(1)) and np.all(z[0] == 0)
    assert np.any(codes[64:] != 0)
    codes, s, z = O.quantize_v_head(X, masked, 4, 128)
    assert np.all(codes[:64] == 0) and np.all(s[:64] == np.float16(1)) and np.all(z[:64] == 0)


def test_integer_grid_is_lossless_at_4_bits():
    rng = np.random.default_rng(5)
    for fn, axis in ((O.quantize_k_head, 0), (O.quantize_v_head, 1)):
        X = rng.integers(0, 16, (128, 128)).astype(np.float16)
        if axis == 0:                                              # both ends present in each K group
            X[0], X[1], X[64], X[65] = 0, 15, 0, 15
        else:                                                      # ... or in each V row
            X[:, 0], X[:, 1] = 0, 15
        G = 64 if axis == 0 else 128
        codes, s, z = fn(X, np.zeros_like(X, bool), 4, G)
        assert np.all(s == np.float16(1)) and np.all(z == 0)
        assert np.array_equal(codes, X.astype(np.uint8))


def test_shifted_grid_gives_nonzero_zero_point_with_the_right_sign():
    # values {-6 .. 9}: scale 1, minimum -6 -> zero = +6 (the zero equation's leading minus)
    X = np.tile(np.arange(-6, 10, dtype=np.float16), (32, 8))
    codes, s, z = O.quantize_v_head(X, np.zeros_like(X, bool), 4, 128)
    assert np.all(s == np.float16(1)) and np.all(z == 6)
    assert np.array_equal(codes, (X + 6).astype(np.uint8))


# Hand-computed pins for the rounding rule of Appendix C's "round" (reading R1: ties go to the even
# integer).  Every group below has scale exactly 1, so x * (1 / scale) is x itself and each listed
# value sits exactly halfway between two codes; rounding halves away from zero (or up) would give
# the neighbouring code.
_TIE_VALUES = [0.5, 1.5, 2.5, 3.5, 4.5, 5.5, 6.5]
_TIE_CODES_EVEN = [0, 2, 2, 4, 4, 6, 6]          # what half-away would make 1, 2, 3, 4, 5, 6, 7


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("which", ["k", "v"])
def test_exact_halves_round_to_the_even_code(bits, which):
    qmax = 2 ** bits - 1
    ties = [(v, c) for v, c in zip(_TIE_VALUES, _TIE_CODES_EVEN) if v < qmax]
    group = np.zeros(128, np.float16)
    group[0], group[1] = 0, qmax                                   # range qmax -> scale 1, zero 0
    for i, (v, _) in enumerate(ties):
        group[2 + i] = v
    other = np.linspace(-3, 3, 128).astype(np.float16)             # the other groups: anything
    if which == "k":                                               # Key group = tokens 0..127 of channel 5
        X = np.tile(other[:, None], (1, 128))
        X[:, 5] = group
        codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), bits, 128)
        assert s[0, 5] == np.float16(1) and z[0, 5] == 0
        got = codes[2:2 + len(ties), 5]
    else:                                                          # Value group = channels 0..127 of token 9
        X = np.tile(other[None, :], (128, 1))
        X[9, :] = group
        codes, s, z = O.quantize_v_head(X, np.zeros_like(X, bool), bits, 128)
        assert s[9, 0] == np.float16(1) and z[9, 0] == 0
        got = codes[9, 2:2 + len(ties)]
    assert got.tolist() == [c for _, c in ties]


@pytest.mark.parametrize("which", ["k", "v"])
def test_negative_halves_round_to_the_even_code(which):
    # 4 bit, values in [-8, 7]: scale 1, zero 8.  -0.5 -> -0 -> code 8 (half-away: 7);
    # -1.5 -> -2 -> 6;  -2.5 -> -2 -> 6 (half-away: 5);  -3.5 -> -4 -> 4;  2.5 -> 2 -> 10 (half-away: 11).
    group = np.zeros(32, np.float16)
    group[:7] = [-8, 7, -0.5, -1.5, -2.5, -3.5, 2.5]
    want = [0, 15, 8, 6, 6, 4, 10]
    if which == "k":
        X = np.zeros((64, 128), np.float16)
        X[32:64, 17] = group                                       # token group 1 of channel 17
        codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), 4, 32)
        assert s[1, 17] == np.float16(1) and z[1, 17] == 8
        assert codes[32:39, 17].tolist() == want
    else:
        X = np.zeros((64, 128), np.float16)
        X[3, 96:128] = group                                       # channel group 3 of token 3
        codes, s, z = O.quantize_v_head(X, np.zeros_like(X, bool), 4, 32)
        assert s[3, 3] == np.float16(1) and z[3, 3] == 8
        assert codes[3, 96:103].tolist() == want


@pytest.mark.parametrize("bits", BITS)
def test_zero_point_of_a_minimum_at_an_exact_half_is_the_even_integer(bits):
    # range exactly qmax -> scale 1; min / scale = -2.5 must give zero = 2 and -3.5 must give 4
    # (half-away: 3 and 4; half-up: 2 and 3 - only ties-to-even gives 2 and 4).  Positive minima:
    # +2.5 -> zero = -2, +3.5 -> -4.
    qmax = 2 ** bits - 1
    mins = np.array([-2.5, -3.5, 2.5, 3.5, -0.5, -1.5], np.float32)
    want = [2, 4, -2, -4, 0, 2]
    scale_h, zero = O.group_params(mins, mins + np.float32(qmax), np.full(len(mins), 8), bits)
    assert np.all(scale_h == np.float16(1))
    assert zero.tolist() == want
    # ... and through a whole head on both axes: the group's minimum itself is a tie
    # (-2.5 -> -2, plus zero 2 -> code 0) and so is its maximum (qmax - 2.5 rounds to the even
    # neighbour; 4 bit: 12.5 -> 12 -> code 14).
    top = qmax - 2.5
    top_code = {2: 0 + 2, 3: 4 + 2, 4: 12 + 2, 8: 252 + 2}[bits]     # 0.5 -> 0, 4.5 -> 4, 12.5 -> 12, 252.5 -> 252
    X = np.full((128, 128), -1.0, np.float16)
    X[0, :], X[1, :] = -2.5, top                                   # Key groups: tokens of each channel
    codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), bits, 64)
    assert np.all(s[0] == np.float16(1)) and np.all(z[0] == 2)
    assert np.all(codes[0] == 0) and np.all(codes[1] == top_code) and np.all(codes[2:64] == 1)
    Xv = np.ascontiguousarray(X.T)                                 # Value groups: channels of each token
    codes, s, z = O.quantize_v_head(Xv, np.zeros_like(Xv, bool), bits, 128)
    assert np.all(s[:, 0] == np.float16(1)) and np.all(z[:, 0] == 2)
    assert np.all(codes[:, 0] == 0) and np.all(codes[:, 1] == top_code)


# Hand-computed pins for the order of operations (reading R1: x / scale is evaluated as the fp32
# product x * fl32(1 / scale)).  Exact arithmetic, fp32 spacing 2^-23 in [1, 2), 2^-22 in [2, 4),
# 2^-21 in [4, 8):
#   scale 7/8:  1 / scale = 8/7 = 9586980.57.. * 2^-23 -> fl32 = 9586981 * 2^-23 (a little above 8/7);
#     x = 5.6875 = 91/16:  x * fl32(1 / scale) = 13631488.609.. * 2^-21 -> fl32 = 13631489 * 2^-21
#     = 6.5000005 -> 7, where the exact quotient 6.5 (and a true division) would round to the even 6.
#   scale 65/128:  1 / scale = 128/65 = 16519104.98.. * 2^-23 -> fl32 = 16519105 * 2^-23;
#     x = 325/256 = 1.26953125:  the product is 10485760.0098 * 2^-22 -> fl32 = 10485760 * 2^-22 = 2.5
#     exactly -> 2; left in double precision the product 2.5000000023 would round to 3.
def test_codes_come_from_an_fp32_product_with_the_fp32_reciprocal():
    a = np.zeros(32, np.float16)
    a[:3] = [0, 13.125, 5.6875]                         # range 15 * 7/8: scale 7/8, zero 0
    b = np.zeros(32, np.float16)
    b[:3] = [0, 7.6171875, 1.26953125]                  # range 15 * 65/128: scale 65/128, zero 0
    X = np.zeros((64, 128), np.float16)
    X[0:32, 9], X[32:64, 9] = a, b                      # Key groups 0 and 1 of channel 9
    codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), 4, 32)
    assert (float(s[0, 9]), float(s[1, 9]), int(z[0, 9]), int(z[1, 9])) == (0.875, 0.5078125, 0, 0)
    assert codes[0:3, 9].tolist() == [0, 15, 7] and codes[32:35, 9].tolist() == [0, 15, 2]
    Xv = np.zeros((64, 128), np.float16)
    Xv[5, 32:64], Xv[6, 96:128] = a, b                  # Value groups (token 5, group 1), (token 6, group 3)
    codes, s, z = O.quantize_v_head(Xv, np.zeros_like(Xv, bool), 4, 32)
    assert (float(s[5, 1]), float(s[6, 3]), int(z[5, 1]), int(z[6, 3])) == (0.875, 0.5078125, 0, 0)
    assert codes[5, 32:35].tolist() == [0, 15, 7] and codes[6, 96:99].tolist() == [0, 15, 2]


def test_zero_point_comes_from_the_same_product():
    # min -5.6875, max 7.4375: range 13.125 = 15 * 7/8 -> scale 7/8; min * fl32(8/7) = -6.5000005
    # -> zero = 7 (the exact quotient -6.5 would give the even 6).  Codes: min -> 0, max -> 15.
    scale_h, zero = O.group_params(np.float32([-5.6875]), np.float32([7.4375]), np.array([32]), 4)
    assert float(scale_h[0]) == 0.875 and int(zero[0]) == 7
    g = np.zeros(32, np.float16)
    g[:2] = [-5.6875, 7.4375]
    X = np.zeros((32, 128), np.float16)
    X[:, 0] = g
    codes, s, z = O.quantize_k_head(X, np.zeros_like(X, bool), 4, 32)
    assert int(z[0, 0]) == 7 and codes[:3, 0].tolist() == [0, 15, 7]      # 0 -> rne(0) + 7


@pytest.mark.parametrize("which", ["k", "v"])
def test_masked_entries_stay_out_of_both_ends_of_the_range(which):
    # group = 0 .. 15 plus two masked entries far below and far above: scale 1, zero 0 - either
    # entry taken into the minimum or the maximum would change both
    g = np.zeros(32, np.float16)
    g[:16] = np.arange(16)
    g[20], g[21] = -100, 300
    m = np.zeros(32, bool)
    m[20] = m[21] = True
    if which == "k":
        X, M = np.zeros((32, 128), np.float16), np.zeros((32, 128), bool)
        X[:, 40], M[:, 40] = g, m
        codes, s, z = O.quantize_k_head(X, M, 4, 32)
        assert float(s[0, 40]) == 1.0 and int(z[0, 40]) == 0
        assert codes[:, 40].tolist() == list(range(16)) + [0] * 16
    else:
        X, M = np.zeros((4, 128), np.float16), np.zeros((4, 128), bool)
        X[2, 64:96], M[2, 64:96] = g, m
        codes, s, z = O.quantize_v_head(X, M, 4, 32)
        assert float(s[2, 2]) == 1.0 and int(z[2, 2]) == 0
        assert codes[2, 64:96].tolist() == list(range(16)) + [0] * 16


def test_more_kept_tokens_than_rows_keeps_the_first_and_reports_the_count():
    rng = np.random.default_rng(12)
    K, V = random_fp16(rng, (1, 2, 128, 128)), random_fp16(rng, (1, 2, 128, 128))
    mask = np.zeros((1, 128), np.uint8)
    flagged = [2, 9, 40, 77, 100]
    mask[0, flagged] = 1
    c = O.quantize_kv(K, V, mask, 4, 128, keep_cap=3)
    assert c.status == O.STATUS_CAPACITY
    assert c.keep_cnt.tolist() == [5]                               # the number flagged, not the number stored
    assert c.keep_idx[0].tolist() == [2, 9, 40]                     # lowest token indices first
    for j, t in enumerate(flagged[:3]):
        assert np.array_equal(c.keep_k[0, :, j].view(np.uint16), K[0, :, t].view(np.uint16))
        assert np.array_equal(c.keep_v[0, :, j].view(np.uint16), V[0, :, t].view(np.uint16))
    # every flagged token, stored or not, is left out of the quantisation (code 0 everywhere)
    assert not c.k_codes_logical[0, :, flagged].any() and not c.v_codes_logical[0, :, flagged].any()


@pytest.mark.parametrize("bits", BITS)
def test_chosen_code_minimises_reconstruction_error_brute_force(bits):
    rng = np.random.default_rng(6 + bits)
    qmax = 2 ** bits - 1
    X = random_fp16(rng, (32, 128), "normal")
    codes, s, z = O.quantize_v_head(X, np.zeros_like(X, bool), bits, 32)
    for t in range(32):
        for c in range(128):
            sc, zc = float(s[t, c // 32]), int(z[t, c // 32])
            errs = [abs(float(X[t, c]) - sc * (q - zc)) for q in range(qmax + 1)]
            assert errs[codes[t, c]] <= min(errs) + sc * 2.0 ** -9


def test_key_groups_run_along_tokens_and_value_groups_along_channels():
    # One huge entry widens exactly the statistics of its own group and no other.
    base = np.tile(np.linspace(-1, 1, 128, dtype=np.float16), (128, 1))
    base = (base + base.T).astype(np.float16)
    ref_k = O.quantize_k_head(base, np.zeros_like(base, bool), 4, 32)[1]
    ref_v = O.quantize_v_head(base, np.zeros_like(base, bool), 4, 32)[1]
    X = base.copy()
    X[70, 5] = 1000
    sk = O.quantize_k_head(X, np.zeros_like(X, bool), 4, 32)[1]       # [n/G, D]
    sv = O.quantize_v_head(X, np.zeros_like(X, bool), 4, 32)[1]       # [n, D/G]
    changed_k = np.argwhere(sk != ref_k)
    changed_v = np.argwhere(sv != ref_v)
    assert changed_k.tolist() == [[70 // 32, 5]]
    assert changed_v.tolist() == [[70, 5 // 32]]
    # ... and masking that entry (a kept token / an isolated outlier) restores the statistics
    m = np.zeros_like(X, bool)
    m[70, 5] = True
    sk_m = O.quantize_k_head(X, m, 4, 32)[1]
    assert sk_m[70 // 32, 5] < sk[70 // 32, 5]
    others = np.ones_like(sk_m, bool)
    others[70 // 32, 5] = False
    assert np.array_equal(sk_m[others], ref_k[others])


# ------------------------------------------------------------------------------ packing
def test_hand_computed_words():
    c = np.zeros(128, np.uint8)
    c[:8] = [1, 2, 3, 4, 5, 6, 7, 8]
    assert O._pack_last_axis(c, 4)[0] == 0x87654321
    c = np.zeros(128, np.uint8)
    c[:10] = [1, 2, 3, 4, 5, 6, 7, 0, 1, 2]
    # five codes in the low half-word: 1 | 2<<3 | 3<<6 | 4<<9 | 5<<12 = 0x58D1;
    # five in the high half-word: 6 | 7<<3 | 0<<6 | 1<<9 | 2<<12 = 0x223E
    assert O._pack_last_axis(c, 3)[0] == 0x223E58D1
    c = np.zeros(128, np.uint8)
    c[:16] = [1, 2, 3, 0, 1, 2, 3, 0, 3, 3, 0, 0, 1, 1, 2, 2]
    assert O._pack_last_axis(c, 2)[0] == int("".join(f"{v:02b}" for v in reversed(c[:16].tolist())), 2)
    c = np.zeros(128, np.uint8)
    c[:8] = [0x11, 0x22, 0x33, 0xFF, 0x01, 0x80, 0x7F, 0xA5]
    words = O._pack_last_axis(c, 8)
    assert words[0] == 0xFF332211 and words[1] == 0xA57F8001 and not words[2:].any()
    assert O.words_per_128(2) == 8 and O.words_per_128(3) == 13 and O.words_per_128(4) == 16 and O.words_per_128(8) == 32


@pytest.mark.parametrize("bits", BITS)
def test_pack_unpack_identity_and_padding(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2 ** bits, (256, 128)).astype(np.uint8)
    wk, wv = O.pack_k(codes, bits), O.pack_v(codes, bits)
    assert wk.shape == (4, O.words_per_128(bits), 64) and wv.shape == (2, O.words_per_128(bits), 128)
    assert np.array_equal(O.unpack_k(wk, bits), codes)
    assert np.array_equal(O.unpack_v(wv, bits), codes)
    if bits == 3:
        assert np.all(wk & np.uint32(0x80008000) == 0) and np.all(wv & np.uint32(0x80008000) == 0)
        # the 13th word holds elements 120..127 only: slots 8 and 9 (bits 25..30) are empty
        assert np.all(wk[:, 12, :] >> np.uint32(25) == 0) and np.all(wv[:, 12, :] >> np.uint32(25) == 0)


@pytest.mark.parametrize("bits", BITS)
def test_single_code_lands_in_the_documented_word_and_bits(bits):
    cpw = O.codes_per_word(bits)
    rng = np.random.default_rng(17)
    for _ in range(20):
        t, c = int(rng.integers(0, 256)), int(rng.integers(0, 128))
        codes = np.zeros((256, 128), np.uint8)
        codes[t, c] = 2 ** bits - 1
        shift = lambda j: (3 * (j % 5) + 16 * (j // 5)) if bits == 3 else bits * j
        wk = O.pack_k(codes, bits)
        nz = np.argwhere(wk)
        assert nz.tolist() == [[t // 64, c // cpw, t % 64]]           # (tile, word = channel chunk, token)
        assert wk[tuple(nz[0])] == (2 ** bits - 1) << shift(c % cpw)
        wv = O.pack_v(codes, bits)
        nz = np.argwhere(wv)
        assert nz.tolist() == [[t // 128, (t % 128) // cpw, c]]       # (tile, word = token chunk, channel)
        assert wv[tuple(nz[0])] == (2 ** bits - 1) << shift((t % 128) % cpw)


def test_zero_point_bound_on_the_scale_cannot_bind_up_to_4_bits():
    """Exhaustive over fp16: the narrowest non-constant group at a given minimum is {x, next fp16
    above x}; even there (max - min) / 15 exceeds |min| / 32766 by a margin far above fp32 rounding,
    so for 2, 3 and 4 bit the scale is the plain range / qmax whatever the data."""
    bits16 = np.concatenate([np.arange(0x0000, 0x7BFF, dtype=np.uint16), np.arange(0x8001, 0xFC00, dtype=np.uint16)])
    x = bits16.view(np.float16)
    up = np.nextafter(x, np.float16(np.inf))
    ok = np.isfinite(up) & (up > x)
    mn, mx = x[ok].astype(np.float64), up[ok].astype(np.float64)
    assert np.all((mx - mn) / 15 > 1.05 * np.abs(mn) / 32766)
    for bits in (2, 3, 4):
        pick = np.random.default_rng(bits).integers(0, mn.size, 4000)
        scale_h, zero = O.group_params(mn[pick].astype(np.float32), mx[pick].astype(np.float32), np.full(4000, 2), bits)
        plain = O.fp32_to_fp16_round_up(((mx[pick] - mn[pick]).astype(np.float32) / np.float32(2 ** bits - 1)).astype(np.float32))
        assert np.array_equal(scale_h, plain)
        assert np.abs(zero.astype(np.int64)).max() <= 2048 * (2 ** bits - 1)


def test_8_bit_groups_far_from_zero_keep_an_int16_zero_point():
    """Values within 1/128 of their distance from zero: range / 255 would put the zero point past
    int16; the widened scale keeps it inside, every code stays in 0..255 and the round trip is
    still finer than the fp16 spacing of the data."""
    rng = np.random.default_rng(8)
    for base in (1000.0, -1000.0, 12.5, -0.37, 30000.0):
        x = (np.float16(base) + rng.integers(0, 4, (64, 32)) * np.spacing(np.float16(abs(base)))).astype(np.float16)
        mn, mx = x.min(1).astype(np.float32), x.max(1).astype(np.float32)
        assert np.all(np.abs(mn) / (mx - mn + 1e-30) > 128)               # the bound binds here
        scale_h, zero = O.group_params(mn, mx, np.full(64, 32), 8)
        assert np.abs(zero.astype(np.int64)).max() <= 32766
        codes = O.quantize_entries(x.astype(np.float32), scale_h[:, None], zero[:, None], 8, np.zeros(x.shape, bool))
        r = np.rint(x.astype(np.float64) / scale_h.astype(np.float64)[:, None]) + zero[:, None]
        assert r.min() >= 0 and r.max() <= 255                            # nothing was clamped
        back = O.dequantize_entries(codes, scale_h[:, None], zero[:, None]).astype(np.float64)
        err = np.abs(back - x.astype(np.float64)).max()
        assert err <= 0.51 * float(scale_h.max()) and err < 0.1 * float(np.spacing(np.float16(abs(base))))
    # and where the range is wide the bound is idle: the scale is range / 255 rounded up
    x = random_fp16(rng, (200, 32), "normal")
    mn, mx = x.min(1).astype(np.float32), x.max(1).astype(np.float32)
    scale_h, _ = O.group_params(mn, mx, np.full(200, 32), 8)
    assert np.array_equal(scale_h, O.fp32_to_fp16_round_up(((mx - mn) / np.float32(255)).astype(np.float32)))


def test_param_word_encoding():
    s = np.array([1.0, 0.5, 6.1e-5], np.float16)
    z = np.array([0, -3, 30720], np.int16)
    p = O.encode_params(s, z)
    assert p[0] == 0x00003C00 and p[1] == (0xFFFD << 16 | 0x3800)
    s2, z2 = O.decode_params(p)
    assert np.array_equal(s2, s) and np.array_equal(z2, z)


# ------------------------------------------------------------------------------ keep rows
def test_keep_rows_are_exact_copies_in_ascending_order():
    rng = np.random.default_rng(8)
    B, H, n, D = 2, 3, 256, 128
    K, V = random_fp16(rng, (B, H, n, D)), random_fp16(rng, (B, H, n, D), "wide")
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 14, 200]] = 1
    mask[1, [0, 1, 2, 3, 77]] = 1
    cache = O.quantize_kv(K, V, mask, 4, 128, keep_cap=6)
    assert cache.status == O.STATUS_OK
    assert cache.keep_cnt.tolist() == [3, 5] == mask.sum(1).tolist()
    assert cache.keep_idx[0].tolist() == [0, 14, 200, -1, -1, -1]
    assert cache.keep_idx[1].tolist() == [0, 1, 2, 3, 77, -1]
    for b in range(B):
        for j in range(cache.keep_cnt[b]):
            t = cache.keep_idx[b, j]
            assert np.array_equal(cache.keep_k[b, :, j].view(np.uint16), K[b, :, t].view(np.uint16))
            assert np.array_equal(cache.keep_v[b, :, j].view(np.uint16), V[b, :, t].view(np.uint16))
        assert not cache.keep_k[b, :, cache.keep_cnt[b]:].any()
    # kept tokens carry code 0 everywhere and do not influence their groups' statistics
    assert not cache.k_codes_logical[0, :, [0, 14, 200]].any()
    K2 = K.copy()
    K2[0, :, 14] = 30000                                            # a wild kept row changes nothing else
    cache2 = O.quantize_kv(K2, V, mask, 4, 128, keep_cap=6)
    assert np.array_equal(cache2.k_codes, cache.k_codes) and np.array_equal(cache2.k_params, cache.k_params)
    # capacity overflow is reported
    assert O.quantize_kv(K, V, mask, 4, 128, keep_cap=4).status == O.STATUS_CAPACITY


# ------------------------------------------------------------------------------ sparse
def test_sparse_threshold_against_full_sort():
    rng = np.random.default_rng(9)
    B, H, n, D = 2, 2, 128, 128
    X = random_fp16(rng, (B, H, n, D), "wide")
    X[0, 0, 5, :64] = X[0, 0, 6, 0]                                  # plant ties
    mask = np.zeros((B, n), np.uint8)
    mask[:, [0, 14]] = 1
    for frac in (0.01, 0.001, 0.05):
        tau = O.sparse_threshold(X, mask, frac)
        live = np.abs(X[:, :, mask[0] == 0, :].astype(np.float64)).ravel()   # same mask for both sequences
        m = int(np.ceil(np.float64(np.float32(frac)) * live.size))
        mth_largest = np.sort(live)[::-1][m - 1]
        assert float(np.uint16(tau).view(np.float16)) == mth_largest
        nnz = int((live >= mth_largest).sum())
        ties = int((live == mth_largest).sum())
        assert nnz >= m and nnz - ties < m


def test_sparse_csr_structure_and_reduction_to_dense():
    rng = np.random.default_rng(10)
    B, H, n, D = 1, 2, 128, 128
    K, V = random_fp16(rng, (B, H, n, D), "wide"), random_fp16(rng, (B, H, n, D))
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 3]] = 1
    cache = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.01)
    Vt = V.reshape(B, H, n // 128, 128, D).transpose(0, 1, 2, 4, 3)          # rows (b, h, tile, channel)
    for X, rowptr, col, val, tau, transposed in ((K, cache.k_rowptr, cache.k_col, cache.k_val, cache.k_tau, False),
                                                 (Vt, cache.v_rowptr, cache.v_col, cache.v_val, cache.v_tau, True)):
        tau_f = float(np.uint16(tau).view(np.float16))
        assert rowptr[0] == 0 and rowptr[-1] == len(col) == len(val) and np.all(np.diff(rowptr) >= 0)
        dense = np.zeros((B * H * n, D), bool)
        for r in range(B * H * n):
            cols = col[rowptr[r]:rowptr[r + 1]].astype(int)
            assert np.all(np.diff(cols) > 0)
            dense[r, cols] = True
            assert np.array_equal(val[rowptr[r]:rowptr[r + 1]], X.reshape(-1, D)[r, cols])
        dense = dense.reshape(X.shape)
        if transposed:                                              # back to (b, h, token, channel)
            dense = dense.transpose(0, 1, 2, 4, 3).reshape(B, H, n, D)
            X = V
        assert not dense[:, :, [0, 3]].any()                        # kept rows hold no sparse entries
        live = np.ones(n, bool)
        live[[0, 3]] = False
        assert np.all(np.abs(X[dense].astype(np.float32)) >= tau_f)
        assert np.all(np.abs(X[:, :, live][~dense[:, :, live]].astype(np.float32)) < tau_f)
        assert dense.sum() >= np.ceil(0.01 * B * H * (n - 2) * D)
    assert not cache.k_codes_logical[(np.abs(K.astype(np.float32)) >= float(np.uint16(cache.k_tau).view(np.float16)))].any()
    # a vanishing fraction isolates nothing and reproduces the dense path bit for bit
    dense_cache = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2)
    tiny = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=1e-12)
    assert len(tiny.k_col) <= 2 * 1 + 64                             # ceil(tiny * count) = 1 entry (+ ties)
    none = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.0)
    assert np.array_equal(none.k_codes, dense_cache.k_codes) and none.k_rowptr is None


def test_given_thresholds_isolate_exactly_what_reaches_them():
    """R19: with `taus` the oracle isolates every non-kept entry whose magnitude reaches the given
    threshold - counted here by brute force - and nothing else; the thresholds the search finds on
    the same data give the dynamic result; 32768 isolates nothing and gives the dense codes; the
    isolated entries leave the group statistics (a group's parameters are those of what is left)."""
    rng = np.random.default_rng(19)
    B, H, n, D = 1, 2, 128, 128
    K, V = random_fp16(rng, (B, H, n, D), "wide"), random_fp16(rng, (B, H, n, D))
    mask = np.zeros((B, n), np.uint8)
    mask[0, [0, 3]] = 1
    live = mask[0] == 0
    dyn = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.01)
    same = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.01, taus=(dyn.k_tau, dyn.v_tau))
    for name in ("k_codes", "v_codes", "k_params", "v_params", "k_rowptr", "k_col", "k_val", "v_rowptr", "v_col", "v_val"):
        assert np.array_equal(getattr(same, name), getattr(dyn, name)), name
    tk, tv = np.float16(1.5), np.float16(0.75)                       # thresholds of some other data
    taus = (int(tk.view(np.uint16)), int(tv.view(np.uint16)))
    given = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.01, taus=taus)
    want_k = int((np.abs(K[:, :, live].astype(np.float32)) >= 1.5).sum())
    want_v = int((np.abs(V[:, :, live].astype(np.float32)) >= 0.75).sum())
    assert len(given.k_col) == want_k == int(given.k_rowptr[-1]) and want_k > 0.02 * K[:, :, live].size
    assert len(given.v_col) == want_v == int(given.v_rowptr[-1])
    assert np.all(np.abs(given.k_val.astype(np.float32)) >= 1.5) and np.all(np.abs(given.v_val.astype(np.float32)) >= 0.75)
    # what is left of a Key group (one channel, the 126 live tokens) sets its parameters
    c = 17
    col = K[0, 0, :, c].astype(np.float32)
    rest = col[live & (np.abs(col) < 1.5)]
    scale = float(np.uint16(int(given.k_params[0, 0, 0, c]) & 0xFFFF).view(np.float16))
    assert (rest.max() - rest.min()) / 7 <= scale <= (rest.max() - rest.min()) / 7 * (1 + 2.0 ** -9)
    none = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2, sparse_frac=0.01, taus=(32768, 32768))
    dense = O.quantize_kv(K, V, mask, 3, 128, keep_cap=2)
    assert len(none.k_col) == 0 and len(none.v_col) == 0
    assert np.array_equal(none.k_codes, dense.k_codes) and np.array_equal(none.v_params, dense.v_params)
