"""GPU parity for batches whose sequences differ in length: requests prefilled one by one into the slots of a
batch (the *_seq calls), then decoded together.  Every sequence is checked against its own single-sequence oracle."""
import numpy as np
import pytest
import torch

from oracle import mixkvq_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_common
    return gpu_common


def _check_seq(H, gc, b, oc, P_per_seq):
    """Bit-exact state of sequence b against its oracle."""
    torch.cuda.synchronize()
    nq, r, ns = gc.state_seq(b)
    assert (nq, r, ns) == (oc.n_quant, oc.n_res, oc.n_sink), (b, nq, r, ns)
    p0 = b * P_per_seq
    nb = nq // oc.cfg.R
    if nb:
        got = gc.block_records()[p0:p0 + P_per_seq, :nb].cpu().numpy()
        assert np.array_equal(got, oc.packed_blocks()), f"records of sequence {b} differ"
    rk, rv = gc.residual()
    assert np.array_equal(rk[p0:p0 + P_per_seq, :r].cpu().numpy().view(np.uint16), oc.res_k[:, :r].view(np.uint16))
    assert np.array_equal(rv[p0:p0 + P_per_seq, :r].cpu().numpy().view(np.uint16), oc.res_v[:, :r].view(np.uint16))
    if ns:
        sk, _ = gc.sink()
        assert np.array_equal(sk[p0:p0 + P_per_seq, :ns].cpu().numpy().view(np.uint16), oc.sink_k[:, :ns].view(np.uint16))
    acc, cnt = gc.query_accumulator()
    assert np.array_equal(acc[p0:p0 + P_per_seq].cpu().numpy().astype(np.uint64), oc.qacc)
    assert np.array_equal(cnt[p0:p0 + P_per_seq].cpu().numpy().astype(np.uint64), oc.qcnt)


@pytest.mark.parametrize("R,Gk,Gv,k4,g,sink", [(128, 128, 128, 16, 7, 0), (64, 32, 64, 16, 4, 32), (32, 32, 32, 8, 3, 0)])
def test_sequences_of_different_lengths(H, R, Gk, Gv, k4, g, sink):
    import paper_2512_19206_amd as M
    rng = np.random.default_rng(1200 + R + g)
    B, Hkv = 4, 2
    kw = dict(Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=0, sink=sink)
    gc = M.Cache(M.make_config(B=B, **kw))
    ocs = [O.OracleCache(O.OracleConfig(B=1, **kw)) for _ in range(B)]
    lengths = [3 * R + 17, 5, 0, R + sink]            # sequence 2 stays empty for now
    ch = rng.uniform(0.3, 8, 128)
    for b, n in enumerate(lengths):
        if n == 0:
            continue
        K = (rng.standard_normal((1, Hkv, n, 128)) * ch).astype(np.float16)
        V = rng.standard_normal((1, Hkv, n, 128)).astype(np.float16)
        Qp = (rng.standard_normal((1, Hkv * g, 24, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        sel_ref = ocs[b].select_channels(Qp, K)
        sel = gc.select_channels_seq(b, H.dev(Qp)[0], H.dev(K)[0])
        assert np.array_equal(sel.cpu().numpy(), sel_ref[0])
        ocs[b].append(K, V, sel_ref)
        gc.quantize_append_seq(b, H.dev(K)[0], H.dev(V)[0], sel=sel)
    for b in range(B):
        _check_seq(H, gc, b, ocs[b], Hkv)
    with pytest.raises(M.MixKVQError) as ei:
        gc.state()
    assert ei.value.code == -6

    def attend(accumulate):
        q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        out, lse = gc.decode_attention(H.dev(q), accumulate_q=accumulate)
        torch.cuda.synchronize()
        go, gl = out.float().cpu().numpy(), lse.cpu().numpy()
        for b in range(B):
            if ocs[b].n_quant + ocs[b].n_res + ocs[b].n_sink == 0:
                assert not go[b].any() and np.all(np.isneginf(gl[b]))      # an empty slot is skipped
                continue
            ro, rl = ocs[b].decode_attention(q[b:b + 1], accumulate_q=accumulate)
            err = np.abs(go[b] - ro[0])
            assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (b, float(err.max()))
            assert np.all(np.abs(gl[b] - rl[0]) <= H.LSE_ATOL + 1e-4 * np.abs(rl[0])), b

    attend(False)
    attend(True)
    for b in range(B):
        _check_seq(H, gc, b, ocs[b], Hkv)

    # decode steps for the whole batch: every sequence appends one token from its own state (flushes fall on
    # different steps); the empty slot starts its sequence with the first of them
    for step in range(R + 5):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * ch).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        go = out.float().cpu().numpy()
        for b in range(B):
            ocs[b].append(k1[b:b + 1], v1[b:b + 1])
            ro, rl = ocs[b].decode_attention(q1[b:b + 1], accumulate_q=True)
            err = np.abs(go[b] - ro[0])
            assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (step, b, float(err.max()))
        if step % 40 == 39:
            for b in range(B):
                _check_seq(H, gc, b, ocs[b], Hkv)

    # a finished request leaves its slot, a new one takes it
    gc.reset_seq(1)
    ocs[1] = O.OracleCache(O.OracleConfig(B=1, **kw))
    K = (rng.standard_normal((1, Hkv, 2 * R + 3, 128)) * ch).astype(np.float16)
    V = rng.standard_normal((1, Hkv, 2 * R + 3, 128)).astype(np.float16)
    ocs[1].append(K, V)
    gc.quantize_append_seq(1, H.dev(K)[0], H.dev(V)[0])
    for b in range(B):
        _check_seq(H, gc, b, ocs[b], Hkv)
    attend(True)
