"""Snapshot and resume: the cache is its five device buffers plus the token counts (Appendix D.1).  A run that is
interrupted at some step, copied into a fresh cache and continued gives the same bytes and the same outputs as the
uninterrupted run."""
import numpy as np
import pytest
import torch

import paper_2512_19206_amd as M
from gpu_common import dev

pytestmark = pytest.mark.gpu


def _inputs(seed, B, Hq, Hkv, T, steps):
    rng = np.random.default_rng(seed)
    K = (rng.standard_normal((B, Hkv, T + steps, 128)) * rng.uniform(0.3, 6, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T + steps, 128)).astype(np.float16)
    Qp = rng.standard_normal((B, Hq, 16, 128)).astype(np.float16)
    qs = rng.standard_normal((steps, B, Hq, 128)).astype(np.float16)
    return dev(K), dev(V), dev(Qp), dev(qs)


def _run(gc, K, V, qs, T, t0, t1):
    outs = []
    for t in range(t0, t1):
        out, lse = M.mixkvq_decode_step(gc, K[:, :, T + t:T + t + 1], V[:, :, T + t:T + t + 1], qs[t], accumulate_q=True)
        outs.append((out.clone(), lse.clone()))
    return outs


@pytest.mark.parametrize("kw,T,cut", [
    (dict(B=2, Hq=14, Hkv=2, D=128, T_max=1024, Gk=128, Gv=128, R=128, k4=16, k16=0), 300, 77),
    (dict(B=1, Hq=5, Hkv=1, D=128, T_max=768, Gk=32, Gv=32, R=64, k4=8, k16=4, sink=32, flush_mode=1), 200, 64),
    (dict(B=2, Hq=8, Hkv=2, D=128, T_max=1024, Gk=128, Gv=128, R=128, k4=0, k16=12, policy=1, tau16=1.0, tau4=0.2), 257, 130),
])
def test_a_resumed_run_equals_the_uninterrupted_one(kw, T, cut):
    steps = 200
    K, V, Qp, qs = _inputs(5, kw["B"], kw["Hq"], kw["Hkv"], T, steps)
    whole = M.Cache(M.make_config(**kw))
    sel = M.mixkvq_select_channels(whole, Qp, K[:, :, :T]) if not kw.get("policy") else None
    M.mixkvq_quantize_append(whole, K[:, :, :T], V[:, :, :T], sel=sel)
    ref = _run(whole, K, V, qs, T, 0, steps)

    first = M.Cache(M.make_config(**kw))
    if not kw.get("policy"):
        M.mixkvq_select_channels(first, Qp, K[:, :, :T])
    M.mixkvq_quantize_append(first, K[:, :, :T], V[:, :, :T], sel=sel)
    a = _run(first, K, V, qs, T, 0, cut)
    torch.cuda.synchronize()
    snap = first.snapshot()
    del first

    second = M.Cache(M.make_config(**kw))
    for t in (second.blocks, second.res_k, second.res_v, second.qacc):
        t.fill_(0xA5)                                    # whatever the fresh buffers hold is overwritten by the snapshot
    second.restore(snap)
    assert second.state() == snap[1][0][:2]
    b = _run(second, K, V, qs, T, cut, steps)
    torch.cuda.synchronize()

    for t, ((o, l), (ro, rl)) in enumerate(zip(a + b, ref)):
        assert torch.equal(o, ro) and torch.equal(l, rl), f"step {t} differs after the resume at {cut}"
    assert second.state() == whole.state() and second.sink_count() == whole.sink_count()
    nq, r = whole.state()
    nb = nq // whole.rec_tokens
    assert torch.equal(second.block_records()[:, :nb], whole.block_records()[:, :nb])
    rows = whole.cfg.sink + r
    for x, y in zip(second.fp16_rows(), whole.fp16_rows()):
        assert torch.equal(x[:, :rows].view(torch.int16), y[:, :rows].view(torch.int16))
    assert all(torch.equal(x, y) for x, y in zip(second.query_accumulator(), whole.query_accumulator()))


def test_unreachable_counts_are_refused():
    gc = M.Cache(M.make_config(B=2, Hq=4, Hkv=2, D=128, T_max=512, Gk=128, Gv=128, R=128, k4=16, k16=0))
    lib = M.load_library()
    for nq, nr, ns in [(64, 5, 0), (640, 5, 0), (128, 0, 0), (0, 129, 0), (0, 5, 32), (-128, 1, 0)]:
        assert lib.mixkvq_cache_set_state(gc.handle, nq, nr, ns) == -1
    assert lib.mixkvq_cache_set_state(gc.handle, 256, 128, 0) == 0 and gc.state() == (256, 128)
    assert lib.mixkvq_cache_set_state_seq(gc.handle, 1, 128, 7, 0) == 0 and gc.state_seq(1) == (128, 7, 0)
    assert lib.mixkvq_cache_set_state_seq(gc.handle, 2, 128, 7, 0) == -1
