"""GPU parity: the HIP path behind the C ABI against the CPU oracle, on the same
seeded inputs.  Indices, packed codes, scales, zero-points, residual rows and the
|q| accumulator must be bit-exact; attention outputs within
2e-3 + 1e-2*|oracle| (fp32 accumulation against the fp64 oracle)."""
import numpy as np
import pytest
import torch

import paper_2512_19206_amd as M
import synth_inputs as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_common
    return gpu_common


def _kw(w: S.Workload, T_max=None, **over):
    kw = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, D=w.D, T_max=T_max or w.T, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    kw.update(over)
    return kw


# ---------------------------------------------------------------------------
# configuration 0, whole: 1 head, 1024 tokens, G = 32, 8 salient channels at 4 bit
# ---------------------------------------------------------------------------
def test_cfg0_end_to_end(H):
    w = S.WORKLOADS[0]
    K, V, Qp, q = S.cfg0_tensors()
    oc, gc = H.make_pair(**_kw(w))
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    assert {5, 37, 70, 101} <= set(sel_ref[0, 0].tolist())
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    assert gc.state() == (992, 32)
    H.check_attention(oc, gc, q)


# ---------------------------------------------------------------------------
# slices of the large configurations: several blocks, ragged residual tail
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_id,B,T", [(1, 2, 1000), (2, 1, 777), (3, 1, 1300), (1, 1, 4096)])
def test_prefill_slice(H, cfg_id, B, T):
    w = S.scaled_workload(cfg_id, B=B, T=T)
    K, V, _ = S.heavy_tailed_kv(cfg_id, B, w.Hkv, T)
    Qp = S.outlier_queries(cfg_id, B, w.Hq, 64)
    q = S.outlier_queries(cfg_id, B, w.Hq, 1, stream=3)[:, :, 0]
    oc, gc = H.make_pair(**_kw(w, T_max=(T + w.R - 1) // w.R * w.R))
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    H.check_attention(oc, gc, q, accumulate_q=True)
    H.check_state(oc, gc)


@pytest.mark.parametrize("g,k4,k16,Gk,Gv,R", [(1, 0, 0, 16, 16, 16), (5, 8, 4, 32, 64, 64), (8, 0, 32, 128, 128, 128),
                                              (7, 24, 0, 64, 32, 128), (2, 8, 0, 16, 128, 48), (6, 16, 0, 128, 32, 128),
                                              (8, 8, 0, 32, 32, 64)])
def test_shapes_and_tiers(H, g, k4, k16, Gk, Gv, R):
    rng = np.random.default_rng(100 + g)
    B, Hkv, T = 2, 2, 5 * R + 7
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16)
    K = (rng.standard_normal((B, Hkv, T, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, 128)).astype(np.float16)
    Qp = rng.standard_normal((B, Hkv * g, 33, 128)).astype(np.float16)
    q = rng.standard_normal((B, Hkv * g, 128)).astype(np.float16)
    oc, gc = H.make_pair(**kw)
    if k4 + k16:
        sel_ref = oc.select_channels(Qp, K)
        sel = gc.select_channels(H.dev(Qp), H.dev(K))
        assert np.array_equal(sel.cpu().numpy(), sel_ref)
    else:
        sel_ref, sel = None, None
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    H.check_attention(oc, gc, q)
    H.check_attention(oc, gc, q, scale=0.31)


def _random_configs(n, seed):
    """Seeded random valid configurations: every matrix-core kernel variant (tiers x value groups x R/Gk) and
    shapes that take the general kernels."""
    rng = np.random.default_rng(seed)
    mfma_tiers = [(16, 0), (0, 12), (8, 0), (0, 0), (24, 0), (32, 0), (8, 4), (0, 32), (0, 4), (0, 8), (0, 16), (0, 24),
                  (16, 4), (16, 8)]
    out = []
    for i in range(n):
        if i % 3 != 2:     # matrix-core path: R, Gk, Gv multiples of 64
            k4, k16 = mfma_tiers[int(rng.integers(len(mfma_tiers)))]
            R = int(rng.choice([64, 128]))
            Gk = int(rng.choice([g for g in (64, 128) if R % g == 0]))
            Gv = int(rng.choice([64, 128])) if (k4, k16) in ((16, 0), (0, 12)) else 128
        else:              # anything the layout allows
            k4, k16 = int(rng.choice([0, 8, 16, 40])), int(rng.choice([0, 4, 20]))
            R = int(rng.choice([16, 32, 48, 80, 96, 112, 128, 256]))
            Gk = int(rng.choice([g for g in (16, 32, 48, 64, 80, 96, 112, 128) if min(R, 128) % g == 0]))
            Gv = int(rng.choice([16, 32, 64, 128]))
        g = int(rng.integers(1, 9))
        out.append((g, k4, k16, Gk, Gv, R, int(rng.integers(1, 4)), int(rng.integers(0, R + 1)),
                    int(rng.integers(0, 2)), 1000 + i))
    return out


@pytest.mark.parametrize("g,k4,k16,Gk,Gv,R,n_blocks,n_extra,flush_mode,seed", _random_configs(42, 5))
def test_random_configurations(H, g, k4, k16, Gk, Gv, R, n_blocks, n_extra, flush_mode, seed):
    rng = np.random.default_rng(seed)
    B, Hkv = 1, 2
    T = R * n_blocks + n_extra
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=R * (n_blocks + 3), Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16,
              flush_mode=flush_mode)
    K = (rng.standard_normal((B, Hkv, T, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = (rng.standard_normal((B, Hkv, T, 128)) * rng.uniform(0.5, 2, (T, 1))).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, 9, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    oc, gc = H.make_pair(**kw)
    sel_ref = sel = None
    if k4 + k16:
        sel_ref = oc.select_channels(Qp, K)
        sel = gc.select_channels(H.dev(Qp), H.dev(K))
        assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    if oc.n_quant + oc.n_res == 0:
        return
    for _ in range(3):      # decode steps: append + attention fused, flushes included
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), float(err.max())
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    H.check_state(oc, gc)


# ---------------------------------------------------------------------------
# decode loop: per-step append, |q| accumulation, re-selection at every flush
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("flush_mode,qreset", [(0, 0), (1, 0), (0, 1)])
def test_decode_steps_with_flushes(H, flush_mode, qreset):
    rng = np.random.default_rng(7)
    B, Hkv, g, R = 2, 2, 5, 32
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=32, Gv=128, R=R, k4=16, k16=0, flush_mode=flush_mode,
              qacc_reset_on_flush=qreset)
    oc, gc = H.make_pair(**kw)
    n0 = 45
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)
    Qp = rng.standard_normal((B, Hkv * g, n0, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    for step in range(100):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        gc.quantize_append(H.dev(k1), H.dev(v1))
        H.check_attention(oc, gc, q1, accumulate_q=True)
        if step % 16 == 15 or step == 99:
            H.check_state(oc, gc)
    assert oc.n_flush_calls >= 3


@pytest.mark.parametrize("R,Gk,k4,k16,flush_mode", [(64, 64, 16, 0, 0), (128, 128, 0, 12, 0), (32, 32, 8, 0, 1)])
def test_fused_decode_step(H, R, Gk, k4, k16, flush_mode):
    """mixkvq_decode_step = append of one token + attention, across block flushes."""
    rng = np.random.default_rng(17)
    B, Hkv, g = 2, 2, 7
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=6 * R, Gk=Gk, Gv=128, R=R, k4=k4, k16=k16, flush_mode=flush_mode)
    oc, gc = H.make_pair(**kw)
    n0 = 2 * R + 11
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)
    Qp = rng.standard_normal((B, Hkv * g, 16, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    for step in range(2 * R + 5):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
        if step % 37 == 36 or step == 2 * R + 4:
            H.check_state(oc, gc)
    assert oc.n_flush_calls >= 2


@pytest.mark.parametrize("R,Gv,k4,k16,g,policy", [(128, 128, 16, 0, 7, 0), (64, 64, 16, 0, 5, 0), (128, 128, 8, 0, 8, 0),
                                                  (128, 128, 0, 0, 3, 0), (128, 128, 16, 0, 4, 1), (128, 32, 16, 0, 7, 0), (128, 32, 16, 0, 5, 1),
                                                  (128, 32, 0, 12, 2, 0), (128, 32, 16, 8, 7, 1), (128, 128, 16, 8, 4, 1),
                                                  (128, 32, 8, 4, 3, 0), (128, 32, 0, 12, 8, 1), (64, 32, 16, 8, 5, 1), (128, 32, 16, 16, 7, 1)])
def test_key_groups_of_32_tokens(H, R, Gv, k4, k16, g, policy):
    """The paper's group size (Section 5, "Settings": G = 32) with a residual length of 64 or 128: four (two) key
    groups per block, value words interleaved over the two key groups of a 64-token span."""
    rng = np.random.default_rng(300 + R + Gv + k4 + g)
    B, Hkv = 2, 2
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=32, Gv=Gv, R=R, k4=k4, k16=k16)
    if policy:
        kw.update(policy=1, tau16=12.0 if k16 else np.inf, tau4=6.0 if k4 else np.inf)
    oc, gc = H.make_pair(**kw)
    assert gc.layout.v_interleave == 1
    n0 = 3 * R + 21
    # every 32-token group gets its own magnitude, so that a scale taken from the wrong group cannot pass
    grp_mag = np.repeat(rng.uniform(0.2, 1.25, (n0 + 31) // 32), 32)[:n0, None]
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128) * grp_mag).astype(np.float16)
    V = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.5, 2, (n0, 1))).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, 16, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    if k4 + k16:        # feed the |q| accumulator (the selection itself is redone per block)
        oc.accumulate_queries(Qp)
        gc.select_channels(H.dev(Qp), H.dev(K))
    oc.append(K, V)
    gc.quantize_append(H.dev(K), H.dev(V))
    H.check_state(oc, gc)
    for step in range(R + 3):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    H.check_state(oc, gc)
    assert oc.n_flush_calls >= 4
    assert gc.decode_path() == M.PATH_MATRIX         # every listed combination has a matrix-core variant


@pytest.mark.parametrize("Gv,k4,k16,g,sink,n_blocks,policy", [(32, 16, 0, 7, 0, 40, 0), (32, 8, 0, 1, 32, 9, 0),
                                                              (128, 16, 0, 5, 0, 130, 0), (32, 0, 0, 8, 0, 17, 0),
                                                              (32, 8, 4, 3, 64, 25, 0), (32, 16, 8, 7, 0, 30, 1),
                                                              (32, 16, 0, 4, 32, 12, 1)])
def test_records_of_32_tokens(H, Gv, k4, k16, g, sink, n_blocks, policy):
    """The shorter residual length of the paper's throughput runs (R = 32, with G = 32): one key group and half a
    64-token span per record, on the matrix-core kernel."""
    rng = np.random.default_rng(3200 + Gv + k4 + g + n_blocks)
    B, Hkv, R = 2, 2, 32
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=R * (n_blocks + 4), Gk=32, Gv=Gv, R=R, k4=k4, k16=k16, sink=sink)
    if policy:
        kw.update(policy=1, tau16=8.0 if k16 else np.inf, tau4=3.0)
    oc, gc = H.make_pair(**kw)
    n0 = sink + R * n_blocks + 13
    grp_mag = np.repeat(rng.uniform(0.2, 1.25, (n0 + 31) // 32), 32)[:n0, None]     # a magnitude of its own per record
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128) * grp_mag).astype(np.float16)
    V = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.5, 2, (n0, 1))).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, 16, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    if k4 + k16:
        oc.accumulate_queries(Qp)
        gc.select_channels(H.dev(Qp), H.dev(K))
    oc.append(K, V)                       # every record with its own channel list
    gc.quantize_append(H.dev(K), H.dev(V))
    H.check_state(oc, gc)
    q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    H.check_attention(oc, gc, q)
    for step in range(R + 5):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    H.check_state(oc, gc)
    assert gc.decode_path() == M.PATH_MATRIX         # not the fallback kernel


@pytest.mark.parametrize("R,Gk,sink,k4,g,flush_mode", [(128, 128, 32, 16, 7, 0), (64, 64, 128, 16, 5, 0), (128, 32, 64, 8, 8, 1),
                                                      (32, 32, 32, 8, 3, 0), (128, 128, 128, 0, 2, 0)])
def test_sink_tokens(H, R, Gk, sink, k4, g, flush_mode):
    """The first `sink` tokens stay in fp16 (Appendix E): token by token while the sink fills, a prefill chunk that
    straddles its end, then decode steps across flushes."""
    rng = np.random.default_rng(500 + R + sink)
    B, Hkv = 2, 2
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=6 * R, Gk=Gk, Gv=128, R=R, k4=k4, k16=0, sink=sink,
              flush_mode=flush_mode)
    oc, gc = H.make_pair(**kw)
    n0 = sink + 2 * R + 9
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)

    def step(k1, v1):
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), float(err.max())
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))

    for t in range(5):                       # the sink fills token by token
        step(K[:, :, t:t + 1], V[:, :, t:t + 1])
    H.check_state(oc, gc)
    assert gc.sink_count() == 5 and gc.state() == (0, 0)
    oc.append(K[:, :, 5:], V[:, :, 5:])      # the rest of the sink, whole blocks and a window in one call
    gc.quantize_append(H.dev(K)[:, :, 5:], H.dev(V)[:, :, 5:])
    H.check_state(oc, gc)
    assert gc.sink_count() == sink
    for t in range(R + 3):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        step(k1, v1)
    H.check_state(oc, gc)
    assert oc.n_sink + oc.n_quant + oc.n_res == n0 + R + 3


def test_dominant_token_with_flat_tail(H):
    """The attention-sink shape at a batch so large that a pair gets ONE workgroup (512 pairs): one token carries
    weight 1 and thousands of tokens 2^-17 of it, together an eighth of the mass.  A quarter of them share the
    dominant token's wavefront, whose running maximum they are measured against; their weights must survive the
    fp16 rounding on the way to the matrix cores."""
    import math
    import paper_2512_19206_amd as M
    from oracle import mixkvq_oracle as O
    rng = np.random.default_rng(900)
    B, Hkv, g, R, T = 64, 8, 2, 128, 8192 + 64
    kw = dict(Hq=g, Hkv=1, D=128, T_max=(T + 2 * R) // R * R, Gk=128, Gv=128, R=R, k4=16, k16=0)
    gc = M.Cache(M.make_config(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, **{k: v for k, v in kw.items() if k not in ("Hq", "Hkv", "D")}))
    Kd = torch.zeros((B, Hkv, T, 128), dtype=torch.float16, device="cuda")
    Vd = torch.zeros_like(Kd)
    qd = torch.zeros((B, Hkv * g, 128), dtype=torch.float16, device="cuda")
    scale = 1.0 / math.sqrt(128)
    cases = []
    for (b, j, spike) in ((3, 5, 17), (40, 0, 5000)):        # spike in the first record of its wavefront / mid-way
        K = (rng.standard_normal((1, 1, T, 128)) * 0.5).astype(np.float16)
        K[..., 0] = 0
        K[0, 0, spike, 0] = 8.0
        V = (1.0 + 0.3 * rng.standard_normal((1, 1, T, 128))).astype(np.float16)
        V[0, 0, spike] = -5.0
        q = np.zeros((1, g, 128), dtype=np.float16)
        q[:, :, 0] = (17 * math.log(2)) / (8.0 * scale)       # the crowd sits at 2^-17 of the spike
        Kd[b, j], Vd[b, j], qd[b, j * g:(j + 1) * g] = H.dev(K)[0, 0], H.dev(V)[0, 0], H.dev(q)[0]
        cases.append((b, j, K, V, q))
    gc.quantize_append(Kd, Vd)
    out, lse = gc.decode_attention(qd)
    torch.cuda.synchronize()
    for b, j, K, V, q in cases:
        oc = O.OracleCache(O.OracleConfig(B=1, **kw))
        oc.append(K, V)
        ro, rl = oc.decode_attention(q)
        go = out[b, j * g:(j + 1) * g].float().cpu().numpy()
        gl = lse[b, j * g:(j + 1) * g].cpu().numpy()
        assert abs(float(ro[0, 0, 5]) + 5.0) > 0.3            # the crowd really carries weight
        err = np.abs(go - ro[0])
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (b, j, float(err.max()))
        assert np.all(np.abs(gl - rl[0]) <= H.LSE_ATOL + 1e-4 * np.abs(rl[0])), (b, j, float(np.abs(gl - rl[0]).max()))
        assert float(err.max()) < 5e-3, (b, j, float(err.max()))   # far inside the tolerance: no weight is dropped


def test_chunked_append_without_selection_matches_oracle(H):
    """sel = NULL on a multi-token append: every flushed block is scored on its own."""
    rng = np.random.default_rng(8)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=1024, Gk=64, Gv=128, R=128, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    Qp = (rng.standard_normal((1, 4, 50, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    oc.accumulate_queries(Qp)
    K = (rng.standard_normal((1, 2, 700, 128)) * rng.uniform(0.3, 8, (2, 1, 128))).astype(np.float16)
    V = rng.standard_normal((1, 2, 700, 128)).astype(np.float16)
    gc.select_channels(H.dev(Qp), H.dev(K))        # only to feed the accumulator
    for lo, hi in ((0, 100), (100, 101), (101, 600), (600, 700)):
        oc.append(K[:, :, lo:hi], V[:, :, lo:hi])
        # strided views of the big tensors exercise the stride arguments
        gc.quantize_append(H.dev(K)[:, :, lo:hi], H.dev(V)[:, :, lo:hi])
        H.check_state(oc, gc)


# ---------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------
def test_everything_in_the_residual_window(H):
    rng = np.random.default_rng(9)
    kw = dict(B=2, Hq=14, Hkv=2, D=128, T_max=128, Gk=128, Gv=128, R=128, k4=16, k16=0)
    for n in (1, 5, 128):
        oc, gc = H.make_pair(**kw)
        K = rng.standard_normal((2, 2, n, 128)).astype(np.float16)
        V = rng.standard_normal((2, 2, n, 128)).astype(np.float16)
        q = rng.standard_normal((2, 14, 128)).astype(np.float16)
        oc.append(K, V)
        gc.quantize_append(H.dev(K), H.dev(V))
        assert gc.state() == (0, n)
        H.check_state(oc, gc)
        H.check_attention(oc, gc, q)


@pytest.mark.parametrize("B,Hkv,g,n_blocks,n_res", [(1, 1, 8, 70, 5), (1, 2, 7, 33, 64), (1, 1, 3, 200, 33)])
def test_few_pairs_many_splits(H, B, Hkv, g, n_blocks, n_res):
    """Few (batch, KV head) pairs: the split count reaches its ceiling (64 partials of up to 8 heads each to
    merge) and the residual sub-units share wavefronts with block records."""
    rng = np.random.default_rng(31)
    R = 64
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=R * (n_blocks + 2), Gk=64, Gv=128, R=R, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    n = R * n_blocks + n_res
    K = (rng.standard_normal((B, Hkv, n, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n, 128)).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, 8, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    assert gc.state() == (R * n_blocks, n_res)
    for _ in range(2):
        q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        H.check_attention(oc, gc, q, accumulate_q=True)
    H.check_state(oc, gc)


def test_quotients_on_rounding_boundaries(H):
    """Integer-valued inputs make (x - z)/s land exactly on k + 1/2 (ties go to even) and right next to it: the
    quantize kernel's reciprocal shortcut must hand these to the exact division."""
    rng = np.random.default_rng(41)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=512, Gk=64, Gv=128, R=128, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    n = 300
    K = rng.integers(0, 7, size=(1, 2, n, 128)).astype(np.float16)          # range 6 -> scale 2 -> quotients k/2
    K[..., :16] = rng.integers(0, 31, size=(1, 2, n, 16)).astype(np.float16)  # range 30 -> 4-bit scale 2
    V = rng.integers(-3, 4, size=(1, 2, n, 128)).astype(np.float16)
    V[:, :, ::3] *= np.float16(1.0009765625)                                 # neighbours of the ties
    Qp = rng.standard_normal((1, 4, 8, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)


def test_groups_far_from_zero(H):
    """Groups whose zero-point is many scale steps away from zero (channel / token offsets of up to +-2000 with a
    spread of a few units, with and without exact ties): the quantize kernel's fused form of Eq. 2 loses accuracy
    with |z/s| and must hand such groups to the exact division."""
    rng = np.random.default_rng(43)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=512, Gk=64, Gv=64, R=128, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    n = 400
    offs = np.array([0, 3, -3, 8, -8, 16, -21, 40, -64, 100, -300, 1024, -2000, 0.5, -0.25, 7])
    K = rng.standard_normal((1, 2, n, 128)) + offs[rng.integers(0, 16, (1, 2, 1, 128))]
    K[..., 64:] = rng.integers(0, 7, (1, 2, n, 64)) + offs[rng.integers(0, 13, (1, 2, 1, 64))].round()   # ties
    V = rng.standard_normal((1, 2, n, 128)) * 0.5 + offs[rng.integers(0, 16, (1, 2, n, 1))]
    V[:, :, ::2] = rng.integers(-3, 4, (1, 2, (n + 1) // 2, 128)) + offs[rng.integers(0, 13, (1, 2, (n + 1) // 2, 1))].round()
    K, V = K.astype(np.float16), V.astype(np.float16)
    Qp = rng.standard_normal((1, 4, 8, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    # the same data scored block by block inside the pack kernel
    oc2, gc2 = H.make_pair(**kw)
    oc2.append(K, V)
    gc2.quantize_append(H.dev(K), H.dev(V))
    H.check_state(oc2, gc2)


def test_eager_mode_with_empty_window_and_single_block(H):
    rng = np.random.default_rng(10)
    kw = dict(B=1, Hq=7, Hkv=1, D=128, T_max=256, Gk=128, Gv=128, R=128, k4=16, k16=0, flush_mode=1)
    oc, gc = H.make_pair(**kw)
    K = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    V = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    q = rng.standard_normal((1, 7, 128)).astype(np.float16)
    oc.append(K, V)
    gc.quantize_append(H.dev(K), H.dev(V))
    assert gc.state() == (128, 0)
    H.check_state(oc, gc)
    H.check_attention(oc, gc, q)


def test_degenerate_groups(H):
    """Constant groups (scale 0), all-zero tensors with both signs of zero, extreme magnitudes, subnormals."""
    rng = np.random.default_rng(11)
    kw = dict(B=1, Hq=2, Hkv=1, D=128, T_max=256, Gk=32, Gv=32, R=64, k4=8, k16=4, flush_mode=1)
    oc, gc = H.make_pair(**kw)
    K = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    V = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    K[0, 0, :32, :] = 1.5                               # constant groups
    K[0, 0, 32:64, ::2] = -0.0                          # mixed zero signs
    K[0, 0, 32:64, 1::2] = 0.0
    K[0, 0, 64:96, 3] = 65504.0                         # largest fp16 against the rest
    K[0, 0, 96:, 7] = (rng.integers(-30, 30, 32) * 2.0 ** -24).astype(np.float16)   # subnormals only
    V[0, 0, 5, :] = -0.0
    V[0, 0, 6, :64] = 60000.0
    V[0, 0, 6, 64:] = -60000.0
    V[0, 0, 7, :] = (rng.integers(-3, 3, 128) * 2.0 ** -24).astype(np.float16)
    Qp = rng.standard_normal((1, 2, 8, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    # attention over these blocks: a plain query, then one aligned with the token whose values are +-60000
    # (values beyond 2048: the absolute term of the bar follows their magnitude, see value_atol)
    atol = H.value_atol(60000.0)
    q = rng.standard_normal((1, 2, 128)).astype(np.float16)
    H.check_attention(oc, gc, q, atol=atol)
    q[0, 0] = (K[0, 0, 6].astype(np.float32) * 0.6).astype(np.float16)
    q[0, 1, 3] = 0.0      # (a query with weight on the 65504 channel would give logits near 4e7, beyond binary32's grain)
    H.check_attention(oc, gc, q, atol=atol)


def test_error_only_score_mode_and_ties(H):
    rng = np.random.default_rng(12)
    kw = dict(B=1, Hq=2, Hkv=1, D=128, T_max=128, Gk=64, Gv=128, R=64, k4=8, k16=8, score_mode=1)
    oc, gc = H.make_pair(**kw)
    K = rng.integers(-4, 5, (1, 1, 64, 128)).astype(np.float16)   # many equal ranges -> ties
    Qp = rng.standard_normal((1, 2, 4, 128)).astype(np.float16)
    assert np.array_equal(gc.select_channels(H.dev(Qp), H.dev(K)).cpu().numpy(), oc.select_channels(Qp, K))
    kw["score_mode"] = 0
    oc, gc = H.make_pair(**kw)
    Qz = np.zeros((1, 2, 4, 128), dtype=np.float16)               # all scores 0 -> lowest indices win
    ref = oc.select_channels(Qz, K)
    assert ref[0, 0].tolist() == list(range(16))
    assert np.array_equal(gc.select_channels(H.dev(Qz), H.dev(K)).cpu().numpy(), ref)


def test_capacity_and_empty_errors_leave_the_cache_unchanged(H):
    import paper_2512_19206_amd as M
    rng = np.random.default_rng(13)
    kw = dict(B=1, Hq=1, Hkv=1, D=128, T_max=64, Gk=32, Gv=32, R=32, k4=8, k16=0)
    oc, gc = H.make_pair(**kw)
    q = H.dev(rng.standard_normal((1, 1, 128)).astype(np.float16))
    with pytest.raises(M.MixKVQError) as e:
        gc.decode_attention(q)
    assert e.value.code == -5
    K = rng.standard_normal((1, 1, 96, 128)).astype(np.float16)
    oc.append(K, K)
    gc.quantize_append(H.dev(K), H.dev(K))
    assert gc.state() == (64, 32)
    with pytest.raises(M.MixKVQError) as e:
        gc.quantize_append(H.dev(K[:, :, :1]), H.dev(K[:, :, :1]))
    assert e.value.code == -2
    assert gc.state() == (64, 32)
    H.check_state(oc, gc)
    # misaligned rows are refused
    with pytest.raises(M.MixKVQError):
        gc.quantize_append(H.dev(K)[:, :, :1, 1:], H.dev(K)[:, :, :1, 1:])


def test_results_are_deterministic(H):
    rng = np.random.default_rng(14)
    w = S.scaled_workload(1, B=1, T=2048)
    K, V, _ = S.heavy_tailed_kv(1, 1, w.Hkv, 2048)
    Qp = S.outlier_queries(1, 1, w.Hq, 32)
    q = H.dev(S.outlier_queries(1, 1, w.Hq, 1, stream=3)[:, :, 0])
    outs, recs = [], []
    for _ in range(3):
        _, gc = H.make_pair(**_kw(w))
        sel = gc.select_channels(H.dev(Qp), H.dev(K))
        gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
        out, lse = gc.decode_attention(q)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy().view(np.uint16))
        recs.append(gc.block_records()[:, :gc.state()[0] // w.R].cpu().numpy())
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    assert all(np.array_equal(recs[0], r) for r in recs[1:])


def test_decode_attention_replayed_from_a_hip_graph(H):
    """The attention call enqueues kernels only (no allocation, no host read-back, no memset), so a caller can capture
    it into a HIP graph.  Every replay, with new queries copied in and eager work in between, must equal the eager call."""
    rng = np.random.default_rng(2000)
    B, Hkv, g, R = 2, 2, 7, 128
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=128, Gv=128, R=R, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    n0 = 5 * R + 40
    K = (rng.standard_normal((B, Hkv, n0, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)
    oc.append(K, V)
    gc.quantize_append(H.dev(K), H.dev(V))
    q_static = torch.zeros((B, Hkv * g, 128), dtype=torch.float16, device="cuda")
    out_static, lse_static = torch.empty_like(q_static), torch.empty((B, Hkv * g), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gc.decode_attention(q_static, out=out_static, lse=lse_static)        # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gc.decode_attention(q_static, out=out_static, lse=lse_static)
    for rep in range(4):
        q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        q_static.copy_(H.dev(q))
        graph.replay()
        torch.cuda.synchronize()
        got, got_lse = out_static.clone(), lse_static.clone()
        eager, eager_lse = gc.decode_attention(H.dev(q))                      # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got, eager) and torch.equal(got_lse, eager_lse), rep
        ro, rl = oc.decode_attention(q)
        err = np.abs(got.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (rep, float(err.max()))
