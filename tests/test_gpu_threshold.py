"""GPU parity of the three-tier threshold policy (Section 4.2): channel lists with their unused entries, block
records with tiers of varying size, and attention over them, against the CPU oracle.  Same bars as the other
parity tests: bytes bit-exact, attention within 2e-3 + 1e-2*|oracle|."""
import math

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


def _inputs(rng, B, Hkv, g, n, Lq):
    K = (rng.standard_normal((B, Hkv, n, 128)) * rng.uniform(0.3, 8, (B, Hkv, 1, 128))).astype(np.float16)
    V = rng.standard_normal((B, Hkv, n, 128)).astype(np.float16)
    Qp = (rng.standard_normal((B, Hkv * g, Lq, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    return K, V, Qp


def _thresholds(Qp, K, g, n16, n4):
    """Thresholds in real units that about n16 / n16 + n4 channels of pair 0 pass over the given keys."""
    A = O.salience(O.abs_query_sum(Qp[0, :g]), O.key_range(K[0, 0])) * 2.0 ** -48 / (g * Qp.shape[2] * 3.0)
    srt = np.sort(A)[::-1]
    return float((srt[n16 - 1] + srt[n16]) / 2), float((srt[n16 + n4 - 1] + srt[n16 + n4]) / 2)


def _tier_sizes(oc):
    return [tuple(len(t) for t in O.tier_lists(b.sel, oc.cfg.k16)) for blocks in oc.blocks for b in blocks]


@pytest.mark.parametrize("tau16,tau4", [(None, None), (0.0, 0.0), (math.inf, math.inf), (3.0, 5.0)])
def test_select_channels_with_thresholds(H, tau16, tau4):
    rng = np.random.default_rng(31)
    B, Hkv, g = 2, 2, 7
    K, V, Qp = _inputs(rng, B, Hkv, g, 300, 40)
    if tau16 is None:
        tau16, tau4 = _thresholds(Qp, K, g, 5, 9)
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=512, Gk=128, Gv=128, R=128, k4=16, k16=8, policy=1,
              tau16=tau16, tau4=tau4)
    oc, gc = H.make_pair(**kw)
    sel_ref = oc.select_channels(Qp, K)
    sel = gc.select_channels(H.dev(Qp), H.dev(K))
    assert np.array_equal(sel.cpu().numpy(), sel_ref)
    n_used = int((sel_ref != O.NO_CHANNEL).sum())
    if tau16 == 0.0:
        assert n_used == sel_ref.size               # the capacities decide
    if tau16 == math.inf:
        assert n_used == 0
    # a prefill with that selection: every block carries it
    oc.append(K, V, sel_ref)
    gc.quantize_append(H.dev(K), H.dev(V), sel=sel)
    H.check_state(oc, gc)
    q = (rng.standard_normal((B, Hkv * g, 128)) * rng.uniform(0.2, 5, 128)).astype(np.float16)
    H.check_attention(oc, gc, q)


@pytest.mark.parametrize("R,Gk,Gv,k4,k16,g,flush_mode", [
    (128, 128, 128, 16, 8, 7, 0),     # matrix-core kernel, both side tiers
    (64, 64, 128, 16, 0, 5, 1),       # matrix-core kernel, 4-bit tier only, eager flush
    (128, 64, 128, 0, 12, 8, 0),      # fp16 tier only
    (32, 32, 32, 8, 4, 3, 0),         # the paper's group size 32: vector-ALU decode kernel
])
def test_decode_steps_with_thresholds(H, R, Gk, Gv, k4, k16, g, flush_mode):
    """Blocks scored one by one (sel = NULL) during a prefill and a run of decode steps: tier sizes differ from
    block to block and sometimes hit the capacities."""
    rng = np.random.default_rng(100 + R + k4)
    B, Hkv = 2, 2
    n0 = 3 * R + 7
    K, V, Qp = _inputs(rng, B, Hkv, g, n0, 24)
    n16 = max(1, k16 - 2) if k16 else 1
    tau16, tau4 = _thresholds(Qp, K[:, :, :R], g, n16, max(2, k4 - 3))
    if k16 == 0:
        tau16 = math.inf
    kw = dict(B=B, Hq=Hkv * g, Hkv=Hkv, D=128, T_max=8 * R, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16, flush_mode=flush_mode,
              policy=1, tau16=tau16, tau4=tau4)
    oc, gc = H.make_pair(**kw)
    oc.accumulate_queries(Qp)
    gc.select_channels(H.dev(Qp), H.dev(K))        # only to feed the accumulator
    oc.append(K, V)
    gc.quantize_append(H.dev(K), H.dev(V))
    H.check_state(oc, gc)
    for step in range(R + 9):
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
        if step % 29 == 28 or step == R + 8:
            H.check_state(oc, gc)
    sizes = _tier_sizes(oc)
    assert len(set(sizes)) > 1, sizes               # the tiers really vary
    assert all(a <= k16 and b <= k4 for a, b in sizes)


def test_thresholds_before_any_query_keep_everything_two_bit(H):
    """No query seen yet: I_d = 0 for every channel, nothing passes a positive threshold."""
    rng = np.random.default_rng(33)
    kw = dict(B=1, Hq=4, Hkv=2, D=128, T_max=512, Gk=128, Gv=128, R=128, k4=16, k16=8, policy=1, tau16=0.5, tau4=0.1)
    oc, gc = H.make_pair(**kw)
    K, V, _ = _inputs(rng, 1, 2, 2, 300, 1)
    oc.append(K, V)
    gc.quantize_append(H.dev(K), H.dev(V))
    H.check_state(oc, gc)
    assert _tier_sizes(oc) == [(0, 0)] * 4
    q = rng.standard_normal((1, 4, 128)).astype(np.float16)
    H.check_attention(oc, gc, q)
