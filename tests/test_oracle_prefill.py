"""Pins for the oracle's statement of Algorithm 1's loop order (prefill_layers): which layers are
quantised before the sink set exists, and that the set is filled exactly once, from the emergence
layer's hidden state."""
import numpy as np
import pytest

from oracle import kvsink_oracle as O
from tests.helpers import random_fp16


def _inputs(L, B=2, H=2, n=256, d=64, sinks=((0, 14, 100), (3, 14, 200)), channel=7, seed=0):
    rng = np.random.default_rng(seed)
    Ks = [random_fp16(rng, (B, H, n, 128)) for _ in range(L)]
    Vs = [random_fp16(rng, (B, H, n, 128)) for _ in range(L)]
    hidden = random_fp16(rng, (B, n, d))
    for b, toks in enumerate(sinks):
        for j, t in enumerate(toks):
            hidden[b, t, channel] = np.float16((-1) ** j * (700 + 10 * j))
    return Ks, Vs, hidden


@pytest.mark.parametrize("l_e", [0, 1, 3, 4])
def test_layers_up_to_the_emergence_layer_are_quantised_without_sinks(l_e):
    L, k = 4, 3
    Ks, Vs, hidden = _inputs(L)
    caches, sink_idx, early, keep = O.prefill_layers(Ks, Vs, hidden, l_e, [7], k, 0, 4, 64, keep_cap=4)
    assert sink_idx.tolist() == [[0, 14, 100], [3, 14, 200]]           # the planted tokens, by construction
    assert early.sum() == 0 and keep.sum(1).tolist() == [3, 3]
    for l in range(1, L + 1):
        c = caches[l - 1]
        X = Ks[l - 1]
        if l <= l_e:                                    # before the set exists: nothing is kept ...
            assert c.keep_cnt.tolist() == [0, 0] and not c.keep_mask.any()
            # ... so the sink rows are ordinary quantised rows (codes present, reconstruction inexact)
            Kd, _ = O.effective_kv(c, 0, 0)
            assert np.abs(Kd[14] - X[0, 0, 14].astype(np.float64)).max() > 0
            assert O.unpack_k(c.k_codes[0, 0], 4)[14].any()
        else:                                           # after it: rows stored bit for bit, slots empty
            assert c.keep_cnt.tolist() == [3, 3]
            assert np.array_equal(c.keep_idx[0, :3], [0, 14, 100])
            assert np.array_equal(c.keep_k[0, :, 1].view(np.uint16), X[0, :, 14].view(np.uint16))
            assert not O.unpack_k(c.k_codes[0, 0], 4)[14].any()
    # the last layer alone sees the set when l_E = L - 1; none does when l_E = L
    assert sum(int(c.keep_cnt.sum() > 0) for c in caches) == L - l_e


def test_each_layer_equals_a_plain_quantise_call_under_the_mask_of_its_phase():
    L, l_e, k, first_n = 3, 2, 2, 4
    Ks, Vs, hidden = _inputs(L, seed=3)
    caches, sink_idx, early, keep = O.prefill_layers(Ks, Vs, hidden, l_e, [7], k, first_n, 3, 32, keep_cap=6)
    assert early[:, :first_n].all() and early.sum() == 2 * first_n                     # PFN part only
    want = np.zeros_like(keep)
    want[:, :first_n] = 1
    want[0, [14, 100]] = 1                              # the two largest magnitudes, 710 and 720, sit at the
    want[1, [14, 200]] = 1                              # second and third planted token of each sequence
    assert np.array_equal(keep, want)
    for l in range(1, L + 1):
        ref = O.quantize_kv(Ks[l - 1], Vs[l - 1], early if l <= l_e else keep, 3, 32, 6)
        c = caches[l - 1]
        for name in ("k_codes", "v_codes", "k_params", "v_params", "keep_k", "keep_v", "keep_idx", "keep_cnt", "keep_mask"):
            assert np.array_equal(getattr(c, name), getattr(ref, name)), (l, name)


def test_the_set_is_filled_from_the_emergence_layers_hidden_state_only():
    # Changing K, V of any layer never changes the set; changing the hidden state changes only the
    # layers after l_E.
    L, l_e = 3, 1
    Ks, Vs, hidden = _inputs(L, seed=5)
    base, idx0, _, _ = O.prefill_layers(Ks, Vs, hidden, l_e, [7], 3, 0, 4, 128, keep_cap=3)
    Ks2 = [K * np.float16(2) for K in Ks]
    _, idx1, _, _ = O.prefill_layers(Ks2, Vs, hidden, l_e, [7], 3, 0, 4, 128, keep_cap=3)
    assert np.array_equal(idx0, idx1)
    hidden2 = hidden.copy()
    hidden2[0, 55, 7] = np.float16(5000)                # a new largest outlier in sequence 0
    moved, idx2, _, _ = O.prefill_layers(Ks, Vs, hidden2, l_e, [7], 3, 0, 4, 128, keep_cap=3)
    assert 55 in idx2[0].tolist() and np.array_equal(idx2[1], idx0[1])
    assert np.array_equal(moved[0].k_codes, base[0].k_codes)           # layer 1 <= l_E: untouched
    assert not np.array_equal(moved[1].keep_idx, base[1].keep_idx)     # layers 2, 3: the new set
