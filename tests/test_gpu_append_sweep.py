"""GPU parity over seeded random sequences of appends: residual lengths 32 ... 256 (one, two or three records per
block), group sizes, tiers, sink lengths, both flush modes, with and without a given selection.  After every append
the stored bytes, the window, the sink and the |q| accumulator equal the oracle's bit for bit; at the end attention
agrees within tolerance."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_common
    return gpu_common


@pytest.mark.parametrize("seed", range(8))
def test_random_append_sequences(H, seed):
    rng = np.random.default_rng(9000 + seed)
    runs = blocks = 0
    for _ in range(12):
        R = int(rng.choice([32, 64, 96, 128, 256]))
        rec = 128 if R == 256 else R
        Gk = int(rng.choice([g for g in (16, 32, 64, 128) if rec % g == 0]))
        Gv = int(rng.choice([32, 64, 128]))
        k4, k16 = [(16, 0), (8, 0), (0, 12), (8, 4), (0, 0)][int(rng.integers(5))]
        g, sink, fm = int(rng.integers(1, 9)), int(rng.choice([0, 0, 32, 64])), int(rng.integers(2))
        B, Hkv = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=R * 12, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16, sink=sink,
                  flush_mode=fm, qacc_reset_on_flush=int(rng.integers(2)))
        oc, gc = H.make_pair(**kw)
        total = 0
        for _ in range(int(rng.integers(2, 6))):
            n = int(rng.choice([1, 2, 7, 31, 100, 129, 300, 517]))
            if total + n > R * 9:
                break
            total += n
            K = (rng.standard_normal((B, Hkv, n, 128)) * rng.uniform(0.3, 8, 128)).astype(np.float16)
            V = rng.standard_normal((B, Hkv, n, 128)).astype(np.float16)
            sel_ref = sel = None
            if k4 + k16:
                Qp = rng.standard_normal((B, Hkv * g, 5, 128)).astype(np.float16)
                sel_ref = oc.select_channels(Qp, K)
                sel = gc.select_channels(H.dev(Qp), H.dev(K))
                assert np.array_equal(sel.cpu().numpy(), sel_ref), kw
                if rng.integers(2):
                    sel_ref = sel = None          # score every block on its own tokens instead
            oc.append(K, V, sel_ref)
            gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
            H.check_state(oc, gc)
        if oc.n_quant + oc.n_res + oc.n_sink:
            q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
            H.check_attention(oc, gc, q)
            runs += 1
            blocks += oc.n_quant // R
    assert runs >= 8 and blocks >= 10
