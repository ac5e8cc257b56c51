"""kvs_prefill_layers (the loop order of Algorithm 1 in one submission) against the oracle's
prefill_layers: every layer's cache bit-exact under the mask of its phase, the masks and sink
indices bit-exact, and every layer's decode within 2e-3."""
import numpy as np
import pytest
import torch

from oracle import kvsink_oracle as O
from paper_2508_04257_amd import binding as kb
from tests.helpers import random_fp16
from tests.test_gpu_parity import DEV, OUT_TOL, assert_cache_equal, assert_csr_equal, hip_decode, row_rel_err

pytestmark = pytest.mark.gpu


def _layers(L, B, H, n, d, channel, rng, heavy=False):
    Ks, Vs = [], []
    for _ in range(L):
        if heavy:
            Ks.append(np.clip(rng.standard_t(4, (B, H, n, 128)), -60000, 60000).astype(np.float16))
            Vs.append(np.clip(rng.standard_t(4, (B, H, n, 128)), -60000, 60000).astype(np.float16))
        else:
            Ks.append(random_fp16(rng, (B, H, n, 128)))
            Vs.append(random_fp16(rng, (B, H, n, 128)))
    hidden = random_fp16(rng, (B, n, d))
    for b in range(B):
        for j, t in enumerate([0, 14, int(rng.integers(16, n))]):
            hidden[b, t, channel] = np.float16((-1) ** j * (600 + 25 * j + b))
    return Ks, Vs, hidden


@pytest.mark.parametrize("l_e", [0, 1, 3, 4])
@pytest.mark.parametrize("bits,G,rep,first_n,sparse", [(4, 128, 1, 0, False), (3, 64, 4, 2, False), (3, 128, 1, 0, True)])
def test_prefill_layers_matches_the_oracle(l_e, bits, G, rep, first_n, sparse):
    rng = np.random.default_rng(100 * l_e + bits + G)
    L, B, H, n, d, k, channel = 4, 2, 2, 640, 96, 3, 41
    Ks, Vs, hidden = _layers(L, B, H, n, d, channel, rng, heavy=sparse)
    frac = 0.01 if sparse else 0.0
    scap = int(B * H * n * 128 * frac * 1.5) + 256 if sparse else 0
    cap = k + first_n
    desc = kb.make_desc(B, n, H * rep, H, bits, G, cap, sparse_frac=frac, sparse_cap=scap)
    caches = [kb.alloc_cache(desc, DEV) for _ in range(L)]
    ws = kb.alloc_workspace(desc, DEV)
    dev = lambda x: torch.from_numpy(x).to(DEV)
    Kd, Vd = [dev(x) for x in Ks], [dev(x) for x in Vs]
    sink_idx = torch.full((B, k), -1, dtype=torch.int32, device=DEV)
    early = torch.full((B, n), 9, dtype=torch.uint8, device=DEV)
    keep = torch.full((B, n), 9, dtype=torch.uint8, device=DEV)
    kb.kvs_prefill_layers(desc, l_e, Kd, Vd, dev(hidden), [channel], k, first_n, sink_idx, early, keep, caches, ws)
    torch.cuda.synchronize()
    ref, ref_idx, ref_early, ref_keep = O.prefill_layers(Ks, Vs, hidden, l_e, [channel], k, first_n, bits, G, cap,
                                                         sparse_frac=frac, sparse_cap=scap if sparse else None)
    assert np.array_equal(sink_idx.cpu().numpy(), ref_idx)
    assert np.array_equal(keep.cpu().numpy(), ref_keep)
    if l_e > 0:
        assert np.array_equal(early.cpu().numpy(), ref_early)
    else:
        assert bool((early == 9).all())                 # not needed, not written
    q = random_fp16(rng, (B, H * rep, 128))
    for l in range(L):
        assert_cache_equal(caches[l], ref[l])
        if sparse:
            assert_csr_equal(caches[l], ref[l])
        # layers up to l_E keep the first-N tokens only, later layers also the predicted ones
        assert caches[l].keep_cnt.cpu().numpy()[:B].tolist() == [first_n if l + 1 <= l_e else int(ref_keep[b].sum())
                                                                 for b in range(B)]
        out, _ = hip_decode(desc, caches[l], ws, q)
        assert row_rel_err(out, O.decode_attn(q, ref[l], Hq=H * rep)[2]) <= OUT_TOL
