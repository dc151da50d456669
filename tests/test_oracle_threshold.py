"""Pins of the oracle's three-tier threshold rule (Section 4.2: A_d > tau_BF16 ->
full precision, tau_UINT4 < A_d <= tau_BF16 -> 4 bit, otherwise 2 bit; Appendix C
for the effective bit-width).  CPU only."""
import math
from fractions import Fraction

import numpy as np

from oracle import mixkvq_oracle as O


def _exact_scores(Q16, K16):
    """Eq. 6-8 in exact rational arithmetic, straight from the fp16 inputs."""
    Q = Q16.reshape(-1, Q16.shape[-1])
    A = []
    for d in range(Q.shape[1]):
        I = sum(Fraction(abs(float(v))) for v in Q[:, d]) / Q.shape[0]          # Eq. 6
        col = [Fraction(float(v)) for v in K16[:, d]]
        A.append(I * (max(col) - min(col)) / 3)                                  # Eq. 7 (B = 2), Eq. 8
    return A


def _inputs(seed, D=32, L=48, Lq=20, heads=3):
    rng = np.random.default_rng(seed)
    K = (rng.standard_normal((L, D)) * rng.uniform(0.2, 4, D)).astype(np.float16)
    Q = (rng.standard_normal((heads, Lq, D)) * rng.uniform(0.2, 4, D)).astype(np.float16)
    return Q, K


def _oracle_tiers(Q, K, tau16, tau4, cap16, cap4):
    qacc, cnt = O.abs_query_sum(Q), Q.shape[0] * Q.shape[1]
    A = O.salience(qacc, O.key_range(K))
    sel = O.select_channels_threshold(A, O.threshold_in_score_units(tau16, cnt), O.threshold_in_score_units(tau4, cnt),
                                      cap16, cap4)
    return sel, A


def test_three_inequalities_in_exact_arithmetic():
    """With room for every channel the tiers are exactly the three sets of Section 4.2."""
    for seed in range(6):
        Q, K = _inputs(100 + seed)
        exact = _exact_scores(Q, K)
        srt = sorted(float(a) for a in exact)
        tau4, tau16 = (srt[18] + srt[19]) / 2, (srt[26] + srt[27]) / 2      # well between two scores
        sel, _ = _oracle_tiers(Q, K, tau16, tau4, 32, 32)
        hi16, hi4 = O.tier_lists(sel, 32)
        want16 = [d for d in range(32) if exact[d] > Fraction(tau16)]
        want4 = [d for d in range(32) if Fraction(tau4) < exact[d] <= Fraction(tau16)]
        assert hi16.tolist() == want16 and hi4.tolist() == want4
        assert len(want16) == 5 and len(want4) == 8
        # unused entries of both lists are marked, each tier is ascending
        assert np.all(sel[len(want16):32] == O.NO_CHANNEL) and np.all(sel[32 + len(want4):] == O.NO_CHANNEL)


def test_threshold_units_match_real_valued_score():
    """threshold_in_score_units: the integer-product score exceeds the converted threshold exactly when the
    real-valued A_d = I_d * S_d exceeds tau (checked in rational arithmetic away from rounding ties)."""
    Q, K = _inputs(7, D=64, L=40, Lq=33, heads=5)
    exact = _exact_scores(Q, K)
    cnt = 5 * 33
    A = O.salience(O.abs_query_sum(Q), O.key_range(K))
    n_checked = 0
    for tau in (0.1, 0.41, 0.63, 0.79, 1.44, 1.52, 2.0):
        thr = O.threshold_in_score_units(tau, cnt)
        for d in range(64):
            if abs(float(exact[d]) - tau) > 1e-9 * tau:
                assert (A[d] > thr) == (exact[d] > Fraction(tau))
                n_checked += 1
    assert n_checked >= 7 * 60
    # error-only score: S_d alone
    rng_units = O.key_range(K).astype(np.float64)
    for d in range(64):
        S = (max(Fraction(float(v)) for v in K[:, d]) - min(Fraction(float(v)) for v in K[:, d])) / 3
        assert (rng_units[d] > O.threshold_in_score_units(0.5, cnt, 1)) == (S > Fraction(0.5))


def test_zero_thresholds_with_capacities_reduce_to_topk():
    """tau = 0 lets every channel with a positive score pass, so the capacities decide: the top-k rule."""
    for seed in range(4):
        Q, K = _inputs(200 + seed)
        sel, A = _oracle_tiers(Q, K, 0.0, 0.0, 4, 8)
        assert np.all(A > 0)
        assert sel.tolist() == O.select_channels(A, 4, 8).tolist()


def test_infinite_thresholds_keep_everything_two_bit():
    Q, K = _inputs(5)
    sel, _ = _oracle_tiers(Q, K, math.inf, math.inf, 4, 8)
    assert np.all(sel == O.NO_CHANNEL)
    assert O.lo_channels(sel, 32).tolist() == list(range(32))


def test_overflow_of_the_fp16_tier_falls_to_four_bit_then_two_bit():
    Q, K = _inputs(9)
    exact = _exact_scores(Q, K)
    order = sorted(range(32), key=lambda d: (-exact[d], d))
    srt = [float(exact[d]) for d in order]
    tau16 = (srt[9] + srt[10]) / 2          # ten channels pass tau16
    # tau4 above tau16 (as for two of the paper's models, Appendix C): the 4-bit band is empty ...
    sel, _ = _oracle_tiers(Q, K, tau16, tau16 * 1.5, 12, 8)
    hi16, hi4 = O.tier_lists(sel, 12)
    assert sorted(order[:10]) == hi16.tolist() and len(hi4) == 0
    # ... but with room for only four fp16 channels the other six take 4-bit places
    sel, _ = _oracle_tiers(Q, K, tau16, tau16 * 1.5, 4, 8)
    hi16, hi4 = O.tier_lists(sel, 4)
    assert hi16.tolist() == sorted(order[:4]) and hi4.tolist() == sorted(order[4:10])
    # and with room for four + four the last two stay at 2 bit
    sel, _ = _oracle_tiers(Q, K, tau16, tau16 * 1.5, 4, 4)
    hi16, hi4 = O.tier_lists(sel, 4)
    assert hi16.tolist() == sorted(order[:4]) and hi4.tolist() == sorted(order[4:8])
    assert set(order[8:10]) <= set(O.lo_channels(sel, 32).tolist())


def test_tiers_shrink_as_thresholds_rise():
    Q, K = _inputs(11)
    prev16, prev_any = 33, 33
    for tau in (0.0, 0.05, 0.2, 0.5, 1.0, 2.0, 8.0, math.inf):
        sel, _ = _oracle_tiers(Q, K, tau, tau / 2, 32, 32)
        hi16, hi4 = O.tier_lists(sel, 32)
        assert len(hi16) <= prev16 and len(hi16) + len(hi4) <= prev_any
        assert not set(hi16.tolist()) & set(hi4.tolist())
        prev16, prev_any = len(hi16), len(hi16) + len(hi4)
    assert prev_any == 0


def _cfg(**kw):
    base = dict(B=1, Hq=2, Hkv=1, D=128, T_max=256, Gk=32, Gv=32, R=32, k4=16, k16=8, policy=1)
    base.update(kw)
    return O.OracleConfig(**base)


def test_block_with_thresholds_off_equals_plain_two_bit_block():
    """No channel promoted: codes, scales and dequantized keys are those of the k4 = k16 = 0 cache, and the
    planes of the unused tiers are zero."""
    rng = np.random.default_rng(3)
    K = rng.standard_normal((32, 128)).astype(np.float16)
    V = rng.standard_normal((32, 128)).astype(np.float16)
    cfg_t, cfg_0 = _cfg(), _cfg(policy=0, k4=0, k16=0)
    none = np.full(24, O.NO_CHANNEL, dtype=np.uint8)
    bt = O.quantize_block(cfg_t, K, V, none)
    b0 = O.quantize_block(cfg_0, K, V, np.zeros(0, dtype=np.uint8))
    assert np.array_equal(bt.lo_codes, b0.lo_codes) and np.array_equal(bt.lo_s, b0.lo_s)
    assert np.array_equal(O.dequant_block_keys(cfg_t, bt), O.dequant_block_keys(cfg_0, b0))
    rec, lay = O.pack_record(cfg_t, bt), O.block_layout(cfg_t)
    assert lay.NL == 128 and np.all(rec[lay.off_idx:lay.off_idx + 24] == O.NO_CHANNEL)
    assert not rec[lay.off_k4_s:lay.off_klo].any() and not rec[lay.off_k4:lay.off_v].any()
    rec0, lay0 = O.pack_record(cfg_0, b0), O.block_layout(cfg_0)
    assert np.array_equal(rec[lay.off_klo:lay.off_k4], rec0[lay0.off_klo:lay0.off_k4])


def test_partly_filled_tiers_dequantize_within_their_error_bounds():
    """Eq. 3 error bound per tier (s/2 with the tier's own scale; exact for the fp16 tier) with tiers that are
    neither empty nor full, and padding of the planes is zero."""
    rng = np.random.default_rng(4)
    K = (rng.standard_normal((32, 128)) * rng.uniform(0.5, 3, 128)).astype(np.float16)
    V = rng.standard_normal((32, 128)).astype(np.float16)
    cfg = _cfg()
    sel = np.full(24, O.NO_CHANNEL, dtype=np.uint8)
    sel[:3] = [7, 40, 99]
    sel[8:13] = [0, 5, 64, 100, 127]
    blk = O.quantize_block(cfg, K, V, sel)
    assert blk.k16.shape == (32, 3) and blk.k4_codes.shape == (32, 5) and blk.lo_codes.shape == (32, 120)
    Kh = O.dequant_block_keys(cfg, blk)
    K64 = K.astype(np.float64)
    assert np.array_equal(Kh[:, [7, 40, 99]], K64[:, [7, 40, 99]])
    rng4 = K64[:, [0, 5, 64, 100, 127]].max(0) - K64[:, [0, 5, 64, 100, 127]].min(0)
    assert np.all(np.abs(Kh - K64)[:, [0, 5, 64, 100, 127]] <= rng4 / 15 / 2 * 1.002 + 1e-4)
    lo = O.lo_channels(sel, 128)
    rng2 = K64[:, lo].max(0) - K64[:, lo].min(0)
    assert np.all(np.abs(Kh - K64)[:, lo] <= rng2 / 3 / 2 * 1.002 + 1e-4)
    assert np.abs(Kh - K64)[:, [0, 5, 64, 100, 127]].max() < np.abs(Kh - K64)[:, lo].max()
    rec, lay = O.pack_record(cfg, blk), O.block_layout(cfg)
    k4s = rec[lay.off_k4_s:lay.off_k4_z].view(np.float16).reshape(1, 16)
    assert not k4s[:, 5:].any()
    k16p = rec[lay.off_k16:lay.off_v].view(np.float16).reshape(32, 8)
    assert np.array_equal(k16p[:, :3], K[:, [7, 40, 99]]) and not k16p[:, 3:].any()


def test_cache_with_thresholds_selects_per_block_and_attends():
    """Through the state machine: every flushed block carries its own tier sizes; the mean bit-width of the
    key channels is the B_eff of Appendix C; attention equals the brute-force softmax over the dequantized cache."""
    rng = np.random.default_rng(6)
    cfg = _cfg(T_max=128, tau16=1.2, tau4=0.5)
    oc = O.OracleCache(cfg)
    scale_d = np.where(np.arange(128) % 16 == 3, 6.0, 1.0)
    k = (rng.standard_normal((1, 1, 100, 128)) * scale_d).astype(np.float16)
    v = rng.standard_normal((1, 1, 100, 128)).astype(np.float16)
    oc.accumulate_queries(rng.standard_normal((1, 2, 50, 128)).astype(np.float16))
    oc.append(k, v)
    assert oc.n_quant == 96 and oc.n_res == 4
    sizes = [tuple(len(t) for t in O.tier_lists(b.sel, cfg.k16)) for b in oc.blocks[0]]
    assert all(0 < n16 <= 8 and n4 <= 16 for n16, n4 in sizes)
    for blk, (n16, n4) in zip(oc.blocks[0], sizes):
        bits = [16] * n16 + [4] * n4 + [2] * (128 - n16 - n4)
        assert math.isclose(sum(bits) / 128, O.effective_key_bits(128, n16, n4))
        # the block was scored on its own tokens with the accumulator of that moment
        assert blk.sel.tolist() == oc.score_and_select(0, O_block_keys(oc, blk, k)).tolist()
    q = rng.standard_normal((1, 2, 128)).astype(np.float16)
    out, _ = oc.decode_attention(q)
    Kh, Vh = oc.dequantized(0)
    for h in range(2):
        logits = np.array([float(np.dot(q[0, h].astype(np.float64), Kh[t])) for t in range(100)]) / math.sqrt(128)
        w = np.exp(logits - logits.max())
        assert np.allclose(out[0, h], (w / w.sum()) @ Vh, rtol=1e-12, atol=1e-14)


def O_block_keys(oc, blk, k):
    i = [id(b) for b in oc.blocks[0]].index(id(blk))
    return k[0, 0, i * oc.cfg.R:(i + 1) * oc.cfg.R]
