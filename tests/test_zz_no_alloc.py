"""The entry point that allocates nothing (mixkvq_decode_attention_noalloc) against mixkvq_decode_attention:
two calls in a row on the same GPU, the second on a smaller cache, so the library's built-in partials buffer
still holds the first call's contents when the second runs."""
import numpy as np
import pytest
import torch

import paper_2512_19206_amd as M
from gpu_common import ATOL, RTOL, LSE_ATOL, dev

pytestmark = pytest.mark.gpu


def _filled_cache(seed, B, Hq, Hkv, T, R=128, k4=16, k16=0):
    rng = np.random.default_rng(seed)
    kw = dict(B=B, Hq=Hq, Hkv=Hkv, D=128, T_max=(T + R - 1) // R * R, Gk=R, Gv=128, R=R, k4=k4, k16=k16)
    K = (rng.standard_normal((B, Hkv, T, 128)) * rng.uniform(0.3, 6, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, 128)).astype(np.float16)
    Qp = rng.standard_normal((B, Hq, 16, 128)).astype(np.float16)
    q = rng.standard_normal((B, Hq, 128)).astype(np.float16)
    gc = M.Cache(M.make_config(**kw))
    sel = M.mixkvq_select_channels(gc, dev(Qp), dev(K))
    M.mixkvq_quantize_append(gc, dev(K), dev(V), sel=sel)
    return gc, dev(q)


def _compare(gc, q):
    ref_out, ref_lse = M.mixkvq_decode_attention(gc, q)
    torch.cuda.synchronize()
    out = torch.full_like(ref_out, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    M.mixkvq_decode_attention_noalloc(gc, q, out, lse)
    torch.cuda.synchronize()
    a, r = out.float().cpu().numpy().astype(np.float64), ref_out.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(a - r) <= ATOL + RTOL * np.abs(r)), f"max abs diff {np.abs(a - r).max():.3e}"
    la, lr = lse.cpu().numpy().astype(np.float64), ref_lse.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(la - lr) <= LSE_ATOL + 1e-4 * np.abs(lr))
    # the same kernels in the same launch shape: the bits agree too
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    return gc.decode_path()


def test_two_calls_in_a_row_the_second_smaller():
    big, q_big = _filled_cache(11, B=2, Hq=14, Hkv=2, T=4096 + 77)        # 4 pairs x 32 splits of partials
    small, q_small = _filled_cache(12, B=1, Hq=5, Hkv=1, T=300, k4=0, k16=12)   # 1 pair x 2 splits
    assert _compare(big, q_big) == M.PATH_MATRIX
    assert _compare(small, q_small) == M.PATH_MATRIX
    # and once more the other way round (the buffer now holds the small call's partials)
    assert _compare(big, q_big) == M.PATH_MATRIX


def test_vector_alu_kernel_and_window_only():
    # a configuration without a matrix-core variant (key groups of 16 tokens), then a cache with fp16 rows only
    rng = np.random.default_rng(5)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=256, Gk=16, Gv=16, R=64, k4=8, k16=0)
    gc = M.Cache(M.make_config(**kw))
    K = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    V = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    q = dev(rng.standard_normal((1, 4, 128)).astype(np.float16))
    M.mixkvq_quantize_append(gc, dev(K), dev(V))
    assert _compare(gc, q) == M.PATH_VECTOR
    gc2 = M.Cache(M.make_config(**dict(kw, Gk=64, Gv=128)))
    M.mixkvq_quantize_append(gc2, dev(K[:, :, :40]), dev(V[:, :, :40]))
    _compare(gc2, q)


def test_too_large_a_launch_is_refused_and_an_empty_cache_reported():
    lib = M.load_library()
    # 4096 pairs of 8 query heads each: 4096 x 1 split x 8 x 130 floats = 17 MB of partials
    gc = M.Cache(M.make_config(B=512, Hq=64, Hkv=8, D=128, T_max=128, Gk=128, Gv=128, R=128, k4=16, k16=0))
    q = torch.zeros((512, 64, 128), dtype=torch.float16, device="cuda")
    out, lse = torch.empty_like(q), torch.empty((512, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(M.MixKVQError) as ei:
        M.mixkvq_decode_attention_noalloc(gc, q, out, lse)
    assert ei.value.code == -5          # empty cache comes first, as in mixkvq_decode_attention
    kv = torch.zeros((512, 8, 1, 128), dtype=torch.float16, device="cuda")
    M.mixkvq_quantize_append(gc, kv, kv)
    with pytest.raises(M.MixKVQError) as ei:
        M.mixkvq_decode_attention_noalloc(gc, q, out, lse)
    assert ei.value.code == -7 and b"scratch" in lib.mixkvq_strerror(-7)
    M.mixkvq_decode_attention(gc, q, out=out, lse=lse)      # the workspace path still serves it
    torch.cuda.synchronize()
