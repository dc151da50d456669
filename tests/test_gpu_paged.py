"""GPU parity of the paged layout: block records live in the slots of a pool that a caller-owned block table assigns.
The records found through the table must be the oracle's, bit for bit, and attention over them within tolerance."""
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


def _check_records(gc, table, oc, Hkv):
    torch.cuda.synchronize()
    pool = gc.pool_records().cpu().numpy()
    ref = oc.packed_blocks()                         # [P, nb, rec_bytes]
    for p in range(ref.shape[0]):
        for blk in range(ref.shape[1]):
            slot = int(table[p // Hkv, blk])
            assert np.array_equal(pool[slot, p % Hkv], ref[p, blk]), f"pair {p} block {blk} (slot {slot}) differs"


@pytest.mark.parametrize("R,Gk,k4,k16,g", [(128, 128, 16, 0, 7), (64, 32, 16, 0, 5), (32, 32, 8, 4, 3)])
def test_block_table(H, R, Gk, k4, k16, g):
    rng = np.random.default_rng(1500 + R)
    B, Hkv, NB = 3, 2, 6
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=NB * R, Gk=Gk, Gv=128, R=R, k4=k4, k16=k16)
    oc, gc = H.make_pair(**kw)
    table = rng.permutation(B * NB).astype(np.int32).reshape(B, NB)
    gc.set_block_table(H.dev(table))
    n0 = 3 * R + 9
    ch = rng.uniform(0.3, 8, 128)
    K = (rng.standard_normal((B, Hkv, n0, 128)) * ch).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, 20, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    _check_records(gc, table, oc, Hkv)
    for step in range(R + 3):
        k1 = (rng.standard_normal((B, Hkv, 1, 128)) * ch).astype(np.float16)
        v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
        q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
        torch.cuda.synchronize()
        err = np.abs(out.float().cpu().numpy() - ro)
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    assert oc.n_quant == 4 * R
    _check_records(gc, table, oc, Hkv)
    assert gc.state() == (oc.n_quant, oc.n_res)
    # the table cannot be swapped under stored blocks
    import paper_2512_19206_amd as M
    with pytest.raises(M.MixKVQError):
        gc.set_block_table(None)


def test_block_table_with_sequences_of_different_lengths(H):
    import paper_2512_19206_amd as M
    rng = np.random.default_rng(1600)
    B, Hkv, g, R, NB = 3, 2, 7, 128, 5
    kw = dict(Hq=Hkv * g, Hkv=Hkv, D=128, T_max=NB * R, Gk=128, Gv=128, R=R, k4=16, k16=0)
    gc = M.Cache(M.make_config(B=B, **kw))
    table = rng.permutation(B * NB).astype(np.int32).reshape(B, NB)
    gc.set_block_table(H.dev(table))
    ocs = [O.OracleCache(O.OracleConfig(B=1, **kw)) for _ in range(B)]
    for b, n in enumerate((4 * R + 30, 40, 2 * R + 1)):
        K = (rng.standard_normal((1, Hkv, n, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
        V = rng.standard_normal((1, Hkv, n, 128)).astype(np.float16)
        ocs[b].append(K, V)
        gc.quantize_append_seq(b, H.dev(K)[0], H.dev(V)[0])
    torch.cuda.synchronize()
    pool = gc.pool_records().cpu().numpy()
    for b in range(B):
        ref = ocs[b].packed_blocks() if ocs[b].n_quant else np.zeros((Hkv, 0, 1), dtype=np.uint8)
        for j in range(Hkv):
            for blk in range(ref.shape[1]):
                assert np.array_equal(pool[int(table[b, blk]), j], ref[j, blk]), (b, j, blk)
    q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    out, lse = gc.decode_attention(H.dev(q))
    torch.cuda.synchronize()
    for b in range(B):
        ro, rl = ocs[b].decode_attention(q[b:b + 1])
        err = np.abs(out[b].float().cpu().numpy() - ro[0])
        assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro[0])), (b, float(err.max()))
