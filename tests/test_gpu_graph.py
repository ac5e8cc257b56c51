"""The library's calls under HIP graph capture: a captured sequence of steps, replayed several
times with eager work and synchronisations in between, leaves the same caches (bit for bit) and
the same attention outputs (to the parity bar) as the eager calls."""
import numpy as np
import pytest
import torch

from paper_2508_04257_amd import pipeline, synth
from tests.test_gpu_parity import DEV, OUT_TOL

pytestmark = pytest.mark.gpu


def _snapshot(buf):
    c = buf.cache
    fields = ["k_codes", "v_codes", "k_params", "v_params", "keep_k", "keep_v", "keep_idx", "keep_cnt", "keep_mask"]
    if buf.desc.sparse_frac > 0:
        fields += ["k_rowptr", "v_rowptr"]
    return {f: getattr(c, f).clone() for f in fields}, buf.out.clone(), buf.lse.clone()


@pytest.mark.parametrize("name,kw", [
    ("dense", dict(B=2, n=1024, Hq=8, Hkv=8, bits=4, group=128, k_sinks=2)),
    ("gqa_int3", dict(B=2, n=1152, Hq=8, Hkv=2, bits=3, group=64, k_sinks=3, first_n=2)),
    ("sparse", dict(B=2, n=1024, Hq=4, Hkv=4, bits=3, group=128, k_sinks=2, sparse_frac=0.01, student_t=True)),
    ("sparse_gqa", dict(B=2, n=1024, Hq=8, Hkv=2, bits=4, group=64, k_sinks=2, sparse_frac=0.01, student_t=True)),
    # heads that take several decode launches: 8 heads at G 32 (8 bit), per-token Keys at G 32
    ("int8_gqa8", dict(B=1, n=1152, Hq=16, Hkv=2, bits=8, group=32, k_sinks=2)),
    ("per_token_g32", dict(B=2, n=1024, Hq=8, Hkv=2, bits=4, group=32, k_sinks=2, key_per_token=True)),
])
def test_captured_steps_replay_like_eager_calls(name, kw):
    w = synth.Workload(name, **kw)
    slots = 3
    hidden, q = synth.make_hidden(w, DEV), synth.make_query(w, DEV)
    inputs = [synth.make_kv(w, DEV, layer=s) for s in range(slots)]
    bufs = [pipeline.alloc_step(w, DEV) for _ in range(slots)]

    for i in range(slots):                              # every cache quantised once before anything decodes it
        pipeline.run_step(w, hidden, inputs[i][0], inputs[i][1], q, bufs[i])
    torch.cuda.synchronize()

    def eager_round():
        for i in range(slots):
            pipeline.step_in_bench_order(w, hidden, inputs[i][0], inputs[i][1], q, bufs[i], bufs[(i + 1) % slots])
        torch.cuda.synchronize()

    eager_round()
    eager_round()                                       # the state a steady loop is in
    want = [_snapshot(b) for b in bufs]
    assert all(int(b.cache.status.cpu()[0]) == 0 for b in bufs)

    graph = pipeline.capture_steps(w, hidden, inputs, q, bufs)
    for replay in range(3):
        for b in bufs:                                  # eager work between replays: wipe what a replay must rewrite
            b.out.zero_()
            b.cache.k_codes.zero_()
            b.cache.keep_cnt.zero_()
        pipeline.decode(q, bufs[0])                     # and an eager library call on the same buffers
        torch.cuda.synchronize()
        graph.replay()
        graph.replay()                                  # twice: the decode of step i reads slot i + 1, rewritten by the first
        torch.cuda.synchronize()
        for b, (cache_want, out_want, lse_want) in zip(bufs, want):
            for f, t in cache_want.items():
                used = t.numel() if f not in ("keep_idx", "keep_cnt") else (b.desc.B * b.desc.keep_cap if f == "keep_idx" else b.desc.B)
                assert torch.equal(getattr(b.cache, f)[:used], t[:used]), (replay, f)
            got, ref = b.out.double().cpu().numpy(), out_want.double().cpu().numpy()
            err = (np.abs(got - ref).max(-1) / np.abs(ref).max(-1)).max()
            assert err <= OUT_TOL, (replay, err)
            assert torch.allclose(b.lse, lse_want, rtol=0, atol=1e-3)
