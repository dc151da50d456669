"""GPU parity over seeded random decode loops: a prefill of random length, then decode steps (append + attention in one
call, flushes included) on random configurations: residual lengths 32 ... 256, group sizes, tiers under both
policies, sink lengths, flush modes.  Attention within tolerance at every step, stored state bit for bit at the end."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_common
    return gpu_common


@pytest.mark.parametrize("seed", range(6))
def test_random_decode_loops(H, seed):
    rng = np.random.default_rng(9100 + seed)
    steps = flushes = 0
    for _ in range(7):
        R = int(rng.choice([32, 64, 96, 128, 256]))
        rec = 128 if R == 256 else R
        Gk = 32 if R == 96 else int(rng.choice([g for g in (32, 64, 128) if rec % g == 0]))
        Gv = int(rng.choice([32, 64, 128]))
        k4, k16 = [(16, 0), (8, 0), (0, 12), (8, 4), (0, 0), (16, 8)][int(rng.integers(6))]
        policy = int(rng.integers(3) == 0) if (k4, k16) in ((16, 8), (16, 0), (8, 4), (0, 12)) else 0
        g, sink, fm = int(rng.integers(1, 9)), int(rng.choice([0, 0, 32, 128])), int(rng.integers(2))
        B, Hkv = int(rng.integers(1, 4)), int(rng.integers(1, 3))
        kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=R * 16, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16, sink=sink,
                  flush_mode=fm)
        if policy:
            kw.update(policy=1, tau16=6.0 if k16 else float("inf"), tau4=3.0)
        oc, gc = H.make_pair(**kw)
        n0 = int(rng.integers(1, 8 * R))
        ch = rng.uniform(0.3, 8, 128)
        K = (rng.standard_normal((B, Hkv, n0, 128)) * ch).astype(np.float16)
        V = rng.standard_normal((B, Hkv, n0, 128)).astype(np.float16)
        Qp = (rng.standard_normal((B, Hkv * g, 7, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
        sel_ref = sel = None
        if k4 + k16:
            sel_ref = oc.select_channels(Qp, K)
            sel = gc.select_channels(H.dev(Qp), H.dev(K))
            if policy or rng.integers(2):
                sel_ref = sel = None
        oc.append(K, V, sel_ref)
        gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
        nf0 = oc.n_flush_calls
        for step in range(int(rng.integers(3, 2 * min(R, 64)))):
            k1 = (rng.standard_normal((B, Hkv, 1, 128)) * ch).astype(np.float16)
            v1 = rng.standard_normal((B, Hkv, 1, 128)).astype(np.float16)
            q1 = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
            oc.append(k1, v1)
            ro, rl = oc.decode_attention(q1, accumulate_q=True)
            out, lse = gc.decode_step(H.dev(k1), H.dev(v1), H.dev(q1), accumulate_q=True)
            torch.cuda.synchronize()
            err = np.abs(out.float().cpu().numpy() - ro)
            assert np.all(err <= H.ATOL + H.RTOL * np.abs(ro)), (kw, step, float(err.max()))
            assert np.all(np.abs(lse.cpu().numpy() - rl) <= H.LSE_ATOL + 1e-4 * np.abs(rl)), (kw, step)
            steps += 1
        flushes += oc.n_flush_calls - nf0
        H.check_state(oc, gc)
    assert steps > 100
