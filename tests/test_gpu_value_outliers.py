"""Attention over value groups in which one element lies far from the others (Eq. 3: x~ = c s + z with |z| >> |x~| for
the ordinary elements).  The kernel folds Eq. 3 into sum (p s) c + sum p z; the two sums then nearly cancel, and the
result is only right if p s keeps far more than 11 bits.  Softmax weights are spread or moderately concentrated on
purpose: a weight of exactly 1 makes p s exact and hides the effect."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_common
    return gpu_common


def _case(H, X, G, focus, T=700, seed=0, k4=16, k16=0):
    rng = np.random.default_rng(seed)
    kw = dict(B=1, Hq=7, Hkv=1, D=128, T_max=1024, Gk=G, Gv=G, R=128, k4=k4, k16=k16)
    oc, gc = H.make_pair(**kw)
    K = rng.standard_normal((1, 1, T, 128)).astype(np.float16)
    V = rng.standard_normal((1, 1, T, 128)).astype(np.float16)
    for t in range(0, T, 5):                       # every fifth token: one element of each value group is -X or +X
        for g0 in range(0, 128, G):
            V[0, 0, t, g0 + (t % G)] = -X if (t // 5) % 2 == 0 else X
    Qp = rng.standard_normal((1, 7, 8, 128)).astype(np.float16)
    q = rng.standard_normal((1, 7, 128)).astype(np.float16)
    if focus:                                      # heads that lean on one outlier token each, with weights well below 1
        for h in range(7):
            q[0, h] = (K[0, 0, 5 * h].astype(np.float32) * focus + q[0, h]).astype(np.float16)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    import paper_2512_19206_amd as M
    err = H.check_attention(oc, gc, q, atol=H.value_atol(X))
    assert gc.decode_path() == M.PATH_MATRIX
    return err


@pytest.mark.parametrize("G", [128, 32])
@pytest.mark.parametrize("focus", [0.0, 0.35])
@pytest.mark.parametrize("X", [8.0, 100.0, 300.0, 512.0])
def test_one_far_element_per_value_group_meets_the_plain_bar(H, X, G, focus):
    """Up to |value| = 512 the bar is the plain one (2e-3 + 1e-2 |ref|)."""
    assert H.value_atol(X) == H.ATOL
    _case(H, X, G, focus)


@pytest.mark.parametrize("G", [128, 32])
@pytest.mark.parametrize("X", [1000.0, 2000.0, 8000.0, 65504.0])
def test_far_elements_beyond_512_meet_the_bar_scaled_to_their_magnitude(H, X, G):
    """Absolute term 2^-18 of the magnitude (binary32 sums).  These groups have value scales above 255, i.e. their
    records take the kernel's guarded form."""
    _case(H, X, G, 0.0)
    _case(H, X, G, 0.35, seed=1)


def test_far_elements_with_an_fp16_key_tier_and_mixed_tiers(H):
    _case(H, 1000.0, 128, 0.35, k4=0, k16=12, seed=2)
    _case(H, 1000.0, 32, 0.0, k4=8, k16=4, seed=3)
