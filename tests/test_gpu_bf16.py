"""GPU parity with bfloat16 tensors at the boundary (cfg.in_dtype = 1; the precision of the paper's models):
q, k, v enter as the nearest binary16, `out` leaves as bfloat16.  The oracle gets the converted binary16 arrays."""
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


def _bf16(rng, shape, scale=1.0, plant=()):
    """(bfloat16 device tensor, the binary16 array the cache must see); `plant`: (index, value) pairs."""
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    for idx, val in plant:
        x[idx] = val
    t = torch.from_numpy(x).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    return t.cuda(), O.bf16_bits_to_f16(bits)


@pytest.mark.parametrize("R,Gk,Gv,k4,k16,g", [(128, 128, 128, 16, 0, 7), (64, 32, 64, 16, 0, 5), (32, 32, 32, 8, 4, 3),
                                              (128, 128, 128, 0, 12, 8)])
def test_bfloat16_tensors(H, R, Gk, Gv, k4, k16, g):
    rng = np.random.default_rng(700 + R + k4)
    B, Hkv = 2, 2
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=6 * R, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16)
    oc, gc = H.make_pair(in_dtype=1, **kw)
    n0 = 2 * R + 13
    ch = rng.uniform(0.3, 8, 128)
    ch[9] = 1e-6                                     # lands in the binary16 subnormals: rounded on entry
    Kd, K = _bf16(rng, (B, Hkv, n0, 128), ch)
    Vd, V = _bf16(rng, (B, Hkv, n0, 128))
    Qd, Qp = _bf16(rng, (B, Hkv * g, 40, 128), rng.uniform(0.2, 5, 128))
    assert np.any((K != 0) & (np.abs(K.astype(np.float32)) < 2.0 ** -14))
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(Qd, Kd)
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    # a strided view of the prompt tensors, then the remainder without a selection (scored per block)
    oc.append(K[:, :, :R + 5], V[:, :, :R + 5], sel_ref)
    gc.quantize_append(Kd[:, :, :R + 5], Vd[:, :, :R + 5], sel=sel)
    oc.append(K[:, :, R + 5:], V[:, :, R + 5:])
    gc.quantize_append(Kd[:, :, R + 5:], Vd[:, :, R + 5:])
    H.check_state(oc, gc)
    for step in range(R // 2 + 3):
        k1d, k1 = _bf16(rng, (B, Hkv, 1, 128), rng.uniform(0.3, 8, 128))
        v1d, v1 = _bf16(rng, (B, Hkv, 1, 128))
        q1d, q1 = _bf16(rng, (B, Hkv * g, 128), rng.uniform(0.2, 5, 128))
        oc.append(k1, v1)
        ro, rl = oc.decode_attention(q1, accumulate_q=True)
        out, lse = gc.decode_step(k1d, v1d, q1d, accumulate_q=True)
        torch.cuda.synchronize()
        assert out.dtype == torch.bfloat16
        err = np.abs(out.float().cpu().numpy() - ro)
        # the bfloat16 output carries 8 significant bits: half a unit in the last place is 2^-9 relative
        assert np.all(err <= H.ATOL + (H.RTOL + 2.0 ** -9) * np.abs(ro)), (step, float(err.max()))
        assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl))
    H.check_state(oc, gc)
    # attention alone (no append), same tolerance
    q1d, q1 = _bf16(rng, (B, Hkv * g, 128))
    out, lse = gc.decode_attention(q1d)
    ro, rl = oc.decode_attention(q1)
    torch.cuda.synchronize()
    err = np.abs(out.float().cpu().numpy() - ro)
    assert np.all(err <= H.ATOL + (H.RTOL + 2.0 ** -9) * np.abs(ro))


def test_bfloat16_values_beyond_binary16_saturate(H):
    """Values far beyond binary16's range enter as +-65504: selection, block records and window rows are those of the
    saturated binary16 inputs, bit for bit."""
    rng = np.random.default_rng(77)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=512, Gk=64, Gv=64, R=128, k4=16, k16=0)
    oc, gc = H.make_pair(in_dtype=1, **kw)
    plant = [((0, 1, 5, 3), 1e6), ((0, 0, 140, 77), -3e5), ((0, 0, 290, 0), 7e4)]
    Kd, K = _bf16(rng, (1, 2, 300, 128), rng.uniform(0.3, 8, 128), plant=plant)
    Vd, V = _bf16(rng, (1, 2, 300, 128), plant=plant)
    Qd, Qp = _bf16(rng, (1, 4, 16, 128), plant=[((0, 2, 3, 9), -1e9)])
    assert V.astype(np.float32).max() == 65504.0 and K.astype(np.float32).min() == -65504.0
    assert Qp.astype(np.float32).min() == -65504.0
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(Qd, Kd)
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(Kd, Vd, sel=sel)
    H.check_state(oc, gc)
