"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (same inputs, same calls, default split count).

The library runs the whole batch; the oracle recomputes sampled (batch, KV head)
pairs one by one from the same seeded inputs: channel selection, every packed
block record of the pair, the residual window and the |q| accumulator bit for bit,
attention outputs of the pair's query heads within the stated tolerance."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_common
    return gpu_common


def _host_pair(host, w, b, j, hb):
    """Host copies of what bench.build_inputs put on the device for batch entry b, KV head j."""
    g = w.Hq // w.Hkv
    src, roll = b % hb, 7 * (b // hb)
    K = np.roll(host["K"][src, j], roll, axis=-1)[None, None]
    V = np.roll(host["V"][src, j], roll, axis=-1)[None, None]
    Qp = np.roll(host["Qp"][src, j * g:(j + 1) * g], roll, axis=-1)[None]
    qs = np.roll(host["qs"][src, j * g:(j + 1) * g], roll, axis=-1)[None]     # [1, g, 8, D]
    return K, V, Qp, qs


@pytest.mark.parametrize("cfg_id,host_batch,samples,n_steps,over", [
    (1, 2, [(0, 0), (1, 3), (5, 2), (7, 1)], 3, {}),
    (3, 1, [(0, 0), (3, 5)], 2, {}),
    (2, 1, [(0, 7), (37, 2)], 2, {}),
    # the shape of configuration 1 with the paper's group size, every block scored on its own tokens
    (1, 2, [(2, 1), (7, 3)], 2, dict(Gk=32, Gv=32, per_block=True)),
    # ... and with the three-tier threshold policy (room for 8 fp16 and 16 four-bit channels per block)
    (1, 2, [(3, 0), (6, 2)], 2, dict(k4=16, k16=8, policy=1, tau16=20.0, tau4=4.0, per_block=True)),
])
def test_full_size_sampled_pairs(H, cfg_id, host_batch, samples, n_steps, over):
    import bench
    import paper_2512_19206_amd as M
    import synth_inputs as S
    from oracle import mixkvq_oracle as O
    w = S.WORKLOADS[cfg_id]
    g = w.Hq // w.Hkv
    print(f"full size: {w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} T={w.T}", flush=True)
    dk, dv, dqp, dq, host = bench.build_inputs(cfg_id, w, host_batch)
    hb = min(host_batch, w.B)
    kw = dict(D=w.D, T_max=w.T + 2 * w.R, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    over = dict(over)
    per_block = over.pop("per_block", False)
    kw.update(over)
    gc = M.Cache(M.make_config(B=w.B, Hq=w.Hq, Hkv=w.Hkv, **kw))
    sel = M.mixkvq_select_channels(gc, dqp, dk)
    M.mixkvq_quantize_append(gc, dk, dv, sel=None if per_block else sel)
    outs = []
    for t in range(n_steps):
        out, lse = M.mixkvq_decode_step(gc, dk[:, :, t:t + 1], dv[:, :, t:t + 1], dq[t], accumulate_q=True)
        assert M.mixkvq_decode_path(gc) == M.PATH_MATRIX      # the kernel bench.py times
        outs.append((out.float().cpu().numpy(), lse.cpu().numpy()))
    torch.cuda.synchronize()
    nq, r = gc.state()
    sel_h = sel.cpu().numpy()
    acc, cnt = gc.query_accumulator()
    acc_h, cnt_h = acc.cpu().numpy().astype(np.uint64), cnt.cpu().numpy().astype(np.uint64)
    rk, rv = gc.residual()

    for b, j in samples:
        print(f"  oracle for pair (b={b}, kv head={j})", flush=True)
        p = b * w.Hkv + j
        K, V, Qp, qs = _host_pair(host, w, b, j, hb)
        oc = O.OracleCache(O.OracleConfig(B=1, Hq=g, Hkv=1, **kw))
        sel_ref = oc.select_channels(Qp, K)
        assert np.array_equal(sel_h[b, j], sel_ref[0, 0]), f"selection differs for pair ({b}, {j})"
        oc.append(K, V, None if per_block else sel_ref)
        for t in range(n_steps):
            oc.append(K[:, :, t:t + 1], V[:, :, t:t + 1])
            ro, rl = oc.decode_attention(np.ascontiguousarray(qs[:, :, t]), accumulate_q=True)
            go, gl = outs[t][0][b, j * g:(j + 1) * g], outs[t][1][b, j * g:(j + 1) * g]
            err = np.abs(go - ro[0])
            assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (b, j, t, float(err.max()))
            assert np.all(np.abs(gl - rl[0]) <= H.LSE_ATOL + 1e-4 * np.abs(rl[0])), (b, j, t)
        assert (nq, r) == (oc.n_quant, oc.n_res)
        nb = nq // w.R
        got = gc.block_records()[p, :nb].cpu().numpy()
        assert np.array_equal(got, oc.packed_blocks()[0]), f"block records differ for pair ({b}, {j})"
        assert np.array_equal(rk[p, :r].cpu().numpy().view(np.uint16), oc.res_k[0, :r].view(np.uint16))
        assert np.array_equal(rv[p, :r].cpu().numpy().view(np.uint16), oc.res_v[0, :r].view(np.uint16))
        assert np.array_equal(acc_h[p], oc.qacc[0]) and cnt_h[p] == oc.qcnt[0]


def test_prefill_configuration_at_its_own_shape(H):
    """Configuration 4 as bench.py runs it: 16 sequences x 32768 tokens, 40 query / 8 KV heads, 32768 prompt queries.
    Channel scoring over the whole prompt (Eq. 6-8), top-k, mixed-precision pack; two sampled pairs against the
    oracle: selection, every block record, the residual window, the |q| sums and counts, bit for bit."""
    import bench
    import paper_2512_19206_amd as M
    import synth_inputs as S
    from oracle import mixkvq_oracle as O
    w = S.WORKLOADS[4]
    g = w.Hq // w.Hkv
    print(f"full size: {w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} T={w.T} Lq={w.T}", flush=True)
    dk, dv, dq, host = bench.build_prefill_inputs(4, w, w.T)
    kw = dict(D=w.D, T_max=w.T, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    gc = M.Cache(M.make_config(B=w.B, Hq=w.Hq, Hkv=w.Hkv, **kw))
    sel = M.mixkvq_prefill(gc, dq, dk, dv)      # scoring + selection + pack in one call, as bench.py's step
    torch.cuda.synchronize()
    del dq
    nq, r = gc.state()
    assert (nq, r) == (w.T - w.R, w.R)
    sel_h = sel.cpu().numpy()
    acc, cnt = gc.query_accumulator()
    acc_h, cnt_h = acc.cpu().numpy().astype(np.uint64), cnt.cpu().numpy().astype(np.uint64)
    assert np.all(cnt_h == np.uint64(g * w.T))
    rk, rv = gc.residual()
    for b, j in [(0, 3), (13, 6)]:
        print(f"  oracle for pair (b={b}, kv head={j})", flush=True)
        p = b * w.Hkv + j
        K = np.roll(host["K"][0, j], 7 * b, axis=-1)[None, None]
        V = np.roll(host["V"][0, j], 7 * b, axis=-1)[None, None]
        Q = np.roll(host["Q"][0, j * g:(j + 1) * g], 7 * b, axis=-1)[None]
        oc = O.OracleCache(O.OracleConfig(B=1, Hq=g, Hkv=1, **kw))
        sel_ref = oc.select_channels(Q, K)
        assert np.array_equal(acc_h[p], oc.qacc[0]) and cnt_h[p] == oc.qcnt[0], f"|q| sums differ for pair ({b}, {j})"
        assert np.array_equal(sel_h[b, j], sel_ref[0, 0]), f"selection differs for pair ({b}, {j})"
        oc.append(K, V, sel_ref)
        assert (nq, r) == (oc.n_quant, oc.n_res)
        got = gc.block_records()[p, :nq // w.R].cpu().numpy()
        assert np.array_equal(got, oc.packed_blocks()[0]), f"block records differ for pair ({b}, {j})"
        assert np.array_equal(rk[p, :r].cpu().numpy().view(np.uint16), oc.res_k[0, :r].view(np.uint16))
        assert np.array_equal(rv[p, :r].cpu().numpy().view(np.uint16), oc.res_v[0, :r].view(np.uint16))


def test_long_decode_across_two_flushes(H):
    """Configuration 3 (131072 cached tokens) over 130 consecutive decode steps: the window is flushed at step 0 and
    again at step 128, each time with the channels re-selected from the running |q| sums (Appendix D.1, D.2).  One
    sampled pair against the oracle: attention at the steps around the flushes, the whole state at the end."""
    import bench
    import paper_2512_19206_amd as M
    import synth_inputs as S
    from oracle import mixkvq_oracle as O
    w = S.WORKLOADS[3]
    g = w.Hq // w.Hkv
    n_steps, checked = 130, (0, 1, 127, 128, 129)
    print(f"full size: {w.name} B={w.B} T={w.T}, {n_steps} decode steps", flush=True)
    dk, dv, dqp, dq, host = bench.build_inputs(3, w, 1)
    kw = dict(D=w.D, T_max=w.T + 2 * w.R, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    gc = M.Cache(M.make_config(B=w.B, Hq=w.Hq, Hkv=w.Hkv, **kw))
    sel = M.mixkvq_select_channels(gc, dqp, dk)
    M.mixkvq_quantize_append(gc, dk, dv, sel=sel)
    outs, flush_steps = {}, []
    for t in range(n_steps):
        nq_before = gc.state()[0]
        out, lse = M.mixkvq_decode_step(gc, dk[:, :, t:t + 1], dv[:, :, t:t + 1], dq[t % 8], accumulate_q=True)
        assert M.mixkvq_decode_path(gc) == M.PATH_MATRIX
        if gc.state()[0] != nq_before:
            flush_steps.append(t)
        if t in checked:
            outs[t] = (out.float().cpu().numpy(), lse.cpu().numpy())
    torch.cuda.synchronize()
    assert flush_steps == [0, 128]
    nq, r = gc.state()
    acc, cnt = gc.query_accumulator()
    rk, rv = gc.residual()
    b, j = 2, 5
    p = b * w.Hkv + j
    K, V, Qp, qs = _host_pair(host, w, b, j, 1)
    oc = O.OracleCache(O.OracleConfig(B=1, Hq=g, Hkv=1, **kw))
    sel_ref = oc.select_channels(Qp, K)
    assert np.array_equal(sel.cpu().numpy()[b, j], sel_ref[0, 0])
    oc.append(K, V, sel_ref)
    for t in range(n_steps):
        oc.append(K[:, :, t:t + 1], V[:, :, t:t + 1])
        q1 = np.ascontiguousarray(qs[:, :, t % 8])
        if t in checked:
            print(f"  oracle attention at step {t}", flush=True)
            ro, rl = oc.decode_attention(q1, accumulate_q=True)
            go, gl = outs[t][0][b, j * g:(j + 1) * g], outs[t][1][b, j * g:(j + 1) * g]
            err = np.abs(go - ro[0])
            assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (t, float(err.max()))
            assert np.all(np.abs(gl - rl[0]) <= H.LSE_ATOL + 1e-4 * np.abs(rl[0])), t
        else:
            oc.accumulate_queries(q1)
    assert (nq, r) == (oc.n_quant, oc.n_res) == (w.T + w.R, 2)
    nb = nq // w.R
    ref = oc.packed_blocks()[0]
    got = gc.block_records()[p, :nb].cpu().numpy()
    assert np.array_equal(got, ref), "block records differ"
    # the two blocks flushed while decoding were scored on their own tokens with the running sums: their channel
    # lists are their own
    lay = O.block_layout(oc.cfg)
    idx = ref[:, lay.off_idx:lay.off_idx + w.k4 + w.k16]
    print("  channel lists: prompt", idx[0].tolist(), "flush 1", idx[nb - 2].tolist(), "flush 2", idx[nb - 1].tolist(), flush=True)
    assert np.array_equal(rk[p, :r].cpu().numpy().view(np.uint16), oc.res_k[0, :r].view(np.uint16))
    assert np.array_equal(rv[p, :r].cpu().numpy().view(np.uint16), oc.res_v[0, :r].view(np.uint16))
    assert np.array_equal(acc[p].cpu().numpy().astype(np.uint64), oc.qacc[0])
    assert int(cnt[p]) == int(oc.qcnt[0])
