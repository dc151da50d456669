"""Which attention kernel a configuration gets: residual lengths 32 ... 256 x group sizes 32 / 64 / 128 x tier pairs
x both policies x both storage layouts must all run on the matrix-core kernel (the vector-ALU kernel is 15-30 times
slower, so sliding onto it would be a silent performance cliff).  Parity of these variants is covered by the other
GPU tests and sweeps; this one only looks at the path and at the output being finite."""
import itertools

import numpy as np
import pytest
import torch

import paper_2512_19206_amd as M

pytestmark = pytest.mark.gpu

TIERS = [(16, 0), (8, 0), (0, 12), (0, 8), (0, 16), (8, 4), (16, 8), (0, 0)]


@pytest.mark.parametrize("R", [32, 64, 96, 128, 256])
def test_listed_configurations_run_on_the_matrix_core_kernel(R):
    assert torch.cuda.is_available(), "these tests need the GPU"
    rng = np.random.default_rng(R)
    checked = 0
    for G, (k4, k16), policy, paged in itertools.product([32, 64, 128], TIERS, [0, 1], [0, 1]):
        rec = 128 if R == 256 else (32 if (R == 96 and G == 32) else R)
        if rec % G or (policy and k4 + k16 == 0):
            continue
        kw = dict(B=2, Hq=10, Hkv=2, D=128, T_max=4 * R, Gk=G, Gv=G, R=R, k4=k4, k16=k16)
        if policy:
            kw.update(policy=1, tau16=5.0, tau4=2.0)
        gc = M.Cache(M.make_config(**kw))
        if paged:
            nb = 4 * R // rec
            gc.set_block_table(torch.arange(2 * nb, dtype=torch.int32, device="cuda").view(2, nb).contiguous())
        n = 2 * R + 5
        K = torch.from_numpy(rng.standard_normal((2, 2, n, 128)).astype(np.float16)).cuda()
        gc.quantize_append(K, K)
        q = torch.from_numpy(rng.standard_normal((2, 10, 128)).astype(np.float16)).cuda()
        out, lse = gc.decode_attention(q)
        torch.cuda.synchronize()
        assert gc.decode_path() == M.PATH_MATRIX, kw
        assert bool(torch.isfinite(out.float()).all()) and bool(torch.isfinite(lse).all()), kw
        checked += 1
    assert checked >= 30


def test_an_unlisted_configuration_reports_the_fallback():
    assert torch.cuda.is_available(), "these tests need the GPU"
    gc = M.Cache(M.make_config(B=1, Hq=2, Hkv=1, D=128, T_max=256, Gk=16, Gv=16, R=64, k4=8, k16=0))
    assert gc.decode_path() == M.PATH_NONE
    K = torch.randn((1, 1, 100, 128), device="cuda").half()
    gc.quantize_append(K, K)
    gc.decode_attention(torch.randn((1, 2, 128), device="cuda").half())
    torch.cuda.synchronize()
    assert gc.decode_path() == M.PATH_VECTOR
