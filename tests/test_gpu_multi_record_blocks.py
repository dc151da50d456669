"""GPU parity for blocks that are stored as several records: the residual length R = 256 (the largest of the
ablation in Appendix E; two records of 128 tokens) and R = 96 with G = 32 (three records of 32 tokens).  A block is
scored as a whole; records, window and accumulator are compared bit for bit against the oracle, attention within
tolerance."""
import numpy as np
import pytest
import torch

import paper_2512_19206_amd as M

from oracle import mixkvq_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_common
    return gpu_common


def _kvq(rng, B, Hkv, g, n, ch):
    K = (rng.standard_normal((B, Hkv, n, 128)) * ch).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n, 128)).astype(np.float16)
    return K, V


@pytest.mark.parametrize("R,Gk,Gv,k4,k16,g,sink,flush_mode", [(256, 128, 128, 16, 0, 7, 0, 0), (256, 64, 64, 16, 0, 5, 32, 0),
                                                            (256, 32, 32, 16, 0, 4, 0, 1), (256, 128, 128, 0, 12, 8, 64, 0),
                                                            (96, 32, 32, 16, 0, 7, 0, 0), (96, 32, 128, 16, 0, 5, 32, 1),
                                                            (96, 16, 32, 8, 0, 2, 0, 0)])
def test_prefill_then_decode_steps(H, R, Gk, Gv, k4, k16, g, sink, flush_mode):
    rng = np.random.default_rng(2560 + R + Gk + k16 + sink)
    B, Hkv = 2, 2
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16, sink=sink,
              flush_mode=flush_mode)
    oc, gc = H.make_pair(**kw)
    ch = rng.uniform(0.3, 8, 128)
    n0 = 3 * R + 77 + sink
    K, V = _kvq(rng, B, Hkv, g, n0, ch)
    Qp = (rng.standard_normal((B, Hkv * g, 20, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    assert gc.rec_tokens == (128 if R == 256 else 32) == O.rec_tokens(oc.cfg)
    H.check_state(oc, gc)
    q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    H.check_attention(oc, gc, q)
    # decode steps through the next flush: the block is scored over the R tokens of the window
    for step in range(R - oc.n_res + 40):
        k1, v1 = _kvq(rng, B, Hkv, g, 1, ch)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    assert oc.n_quant == 4 * R
    H.check_state(oc, gc)
    assert gc.decode_path() == (M.PATH_VECTOR if Gk == 16 else M.PATH_MATRIX)


@pytest.mark.parametrize("R,Gk,counts", [(256, 64, (1536, 21)), (96, 32, (1536, 21))])
def test_blocks_scored_one_by_one_across_window_and_new_tokens(H, R, Gk, counts):
    """Appends without a given selection: the first block of the second call lies partly in the window, partly in
    the new tokens, and each block takes its own channel list from its own R tokens."""
    rng = np.random.default_rng(2561 + R)
    B, Hkv, g = 2, 2, 5
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R + 1536, Gk=Gk, Gv=128, R=R, k4=16, k16=0)
    oc, gc = H.make_pair(**kw)
    Qp = (rng.standard_normal((B, Hkv * g, 16, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    Kd = rng.standard_normal((B, Hkv, 16, 128)).astype(np.float16)      # only to get the queries into the accumulator
    oc.select_channels(Qp, Kd)
    gc.select_channels(H.dev(Qp), H.dev(Kd))
    for n in (100, 700, 256, 1, 500):
        ch = rng.uniform(0.3, 8, 128)                      # the wide channels move from call to call
        K, V = _kvq(rng, B, Hkv, g, n, ch)
        oc.append(K, V)
        gc.quantize_append(H.dev(K), H.dev(V))
        H.check_state(oc, gc)
    assert oc.n_quant + oc.n_res == 1557 and oc.n_quant % R == 0 and 0 < oc.n_res <= R
    lists = {tuple(b.sel) for blocks in oc.blocks for b in blocks}
    assert len(lists) > 2                                   # the blocks really differ in their selection
    q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    H.check_attention(oc, gc, q)


def test_bfloat16_tensors_and_paged_records(H):
    """The same with bfloat16 tensors (the window holds binary16, the new tokens bfloat16) and a block table with one
    entry per 128-token record."""
    rng = np.random.default_rng(2562)
    B, Hkv, g, NB = 2, 2, 7, 12
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=NB * 128, Gk=128, Gv=128, R=256, k4=16, k16=0, in_dtype=1)
    oc, gc = H.make_pair(**kw)
    table = rng.permutation(B * NB).astype(np.int32).reshape(B, NB)
    gc.set_block_table(H.dev(table))

    def bf(shape, scale=1.0):
        t = torch.from_numpy((rng.standard_normal(shape) * scale).astype(np.float32)).to(torch.bfloat16)
        return t.cuda(), O.bf16_bits_to_f16(t.view(torch.int16).numpy().view(np.uint16))

    ch = rng.uniform(0.3, 8, 128)
    for n in (300, 600):
        Kd, K = bf((B, Hkv, n, 128), ch)
        Vd, V = bf((B, Hkv, n, 128))
        oc.append(K, V)
        gc.quantize_append(Kd, Vd)
    torch.cuda.synchronize()
    assert gc.state() == (oc.n_quant, oc.n_res) == (768, 132)
    pool = gc.pool_records().cpu().numpy()
    ref = oc.packed_blocks()
    assert ref.shape[1] == 6
    for p in range(ref.shape[0]):
        for rec in range(ref.shape[1]):
            assert np.array_equal(pool[int(table[p // Hkv, rec]), p % Hkv], ref[p, rec]), (p, rec)
    qd, q = bf((B, Hkv * g, 128), rng.uniform(0.2, 5, 128))
    out, lse = gc.decode_attention(qd)
    torch.cuda.synchronize()
    ro, rl = oc.decode_attention(q)
    err = np.abs(out.float().cpu().numpy() - ro)
    assert np.all(err <= H.ATOL + (H.RTOL + 2.0 ** -8) * np.abs(ro)), float(err.max())
    assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
