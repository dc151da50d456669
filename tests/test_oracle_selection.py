"""Pins of the oracle's salience score and channel selection (Section 4.2,
Eq. 6-8; Appendix D for grouped-query aggregation).  CPU only."""
from fractions import Fraction

import numpy as np

from oracle import mixkvq_oracle as O


def _exact_topk(Q16, K16, k):
    """Eq. 6-8 in exact rational arithmetic, straight from the fp16 inputs."""
    Q = Q16.reshape(-1, Q16.shape[-1])
    D = Q.shape[1]
    A = []
    for d in range(D):
        I = sum(Fraction(abs(float(v))) for v in Q[:, d]) / Q.shape[0]          # Eq. 6
        col = [Fraction(float(v)) for v in K16[:, d]]
        S = (max(col) - min(col)) / 3                                            # Eq. 7 with B = 2
        A.append(I * S)                                                          # Eq. 8
    order = sorted(range(D), key=lambda d: (-A[d], d))
    return sorted(order[:k]), A


def test_topk_equals_exact_rational_score():
    rng = np.random.default_rng(10)
    for trial in range(4):
        D, L, Lq = 32, 48, 20
        K = (rng.standard_normal((L, D)) * rng.uniform(0.5, 4, D)).astype(np.float16)
        Q = (rng.standard_normal((3, Lq, D)) * rng.uniform(0.5, 4, D)).astype(np.float16)
        A = O.salience(O.abs_query_sum(Q), O.key_range(K))
        sel = O.select_channels(A, 0, 8)
        ref, _ = _exact_topk(Q, K, 8)
        assert sel.tolist() == ref


def test_score_matches_float64_formula():
    """I from the mean of |Q| and S from Eq. 7 in float64 reproduce the
    fixed-point score up to its constant factor 2^-48 / (count * 3)."""
    rng = np.random.default_rng(11)
    D, L, Lq = 128, 256, 64
    K = rng.standard_normal((L, D)).astype(np.float16)
    Q = rng.standard_normal((7, Lq, D)).astype(np.float16)
    A = O.salience(O.abs_query_sum(Q), O.key_range(K))
    I = np.abs(Q.astype(np.float64)).reshape(-1, D).mean(axis=0)
    S = (K.astype(np.float64).max(axis=0) - K.astype(np.float64).min(axis=0)) / 3.0
    ref = I * S
    got = A * 2.0 ** -48 / (7 * Lq * 3.0)
    assert np.allclose(got, ref, rtol=1e-12, atol=0)


def test_outlier_key_channels_are_selected_with_iid_queries():
    rng = np.random.default_rng(12)
    D = 128
    K = rng.standard_normal((1024, D)).astype(np.float32)
    K[:, [5, 37, 70, 101]] *= 15
    Q = rng.standard_normal((1024, D)).astype(np.float16)
    A = O.salience(O.abs_query_sum(Q), O.key_range(K.astype(np.float16)))
    sel = O.select_channels(A, 0, 8).tolist()
    assert {5, 37, 70, 101} <= set(sel)
    assert sel == sorted(sel)


def test_large_key_channel_with_silent_query_is_not_selected():
    """Section 4.1: a key channel with large activations is not critical when
    its query activations are small."""
    rng = np.random.default_rng(13)
    D = 64
    K = rng.standard_normal((256, D)).astype(np.float32)
    K[:, 9] *= 40
    Q = rng.standard_normal((256, D)).astype(np.float32)
    Q[:, 9] = 0
    K16, Q16 = K.astype(np.float16), Q.astype(np.float16)
    sel = O.select_channels(O.salience(O.abs_query_sum(Q16), O.key_range(K16)), 0, 8)
    assert 9 not in sel.tolist()
    # the error-only ablation (A = S) does pick it
    sel_s = O.select_channels(O.salience(O.abs_query_sum(Q16), O.key_range(K16), score_mode=1), 0, 8)
    assert 9 in sel_s.tolist()


def test_error_only_mode_is_topk_of_ranges():
    rng = np.random.default_rng(14)
    K = (rng.standard_normal((128, 64)) * rng.uniform(0.5, 3, 64)).astype(np.float16)
    Q = rng.standard_normal((16, 64)).astype(np.float16)
    r = O.key_range(K)
    sel = O.select_channels(O.salience(O.abs_query_sum(Q), r, score_mode=1), 0, 8)
    ref = sorted(sorted(range(64), key=lambda d: (-int(r[d]), d))[:8])
    assert sel.tolist() == ref


def test_invariant_to_token_and_head_order():
    rng = np.random.default_rng(15)
    K = rng.standard_normal((64, 32)).astype(np.float16)
    Q = rng.standard_normal((4, 16, 32)).astype(np.float16)
    a = O.salience(O.abs_query_sum(Q), O.key_range(K))
    Kp = K[rng.permutation(64)]
    Qp = Q[rng.permutation(4)][:, rng.permutation(16)]
    b = O.salience(O.abs_query_sum(Qp), O.key_range(Kp))
    assert np.array_equal(a, b)


def test_ties_go_to_lower_index_and_tiers_are_ordered():
    A = np.array([1.0, 5.0, 5.0, 0.0, 7.0, 5.0, 2.0, 7.0])
    sel = O.select_channels(A, 2, 2)
    # best two (7.0 at 4 and 7) -> fp16 tier; next two among the 5.0 ties -> lower indices 1, 2
    assert sel.tolist() == [4, 7, 1, 2]
    assert O.lo_channels(sel, 8).tolist() == [0, 3, 5, 6]


def test_gqa_group_aggregation():
    """Appendix D: query magnitudes of all query heads sharing a KV head are aggregated."""
    cfg = O.OracleConfig(B=1, Hq=4, Hkv=2, D=16, T_max=64, Gk=16, Gv=16, R=16, k4=8, k16=0)
    cache = O.OracleCache(cfg)
    rng = np.random.default_rng(16)
    Q = rng.standard_normal((1, 4, 5, 16)).astype(np.float16)
    cache.accumulate_queries(Q)
    for j in range(2):
        ref = np.abs(Q[0, 2 * j:2 * j + 2].astype(np.float64)).reshape(-1, 16).sum(axis=0) * 2.0 ** 24
        assert np.array_equal(cache.qacc[j].astype(np.float64), ref)
        assert int(cache.qcnt[j]) == 10


def test_fix24_is_exact_for_every_finite_fp16():
    allbits = np.arange(0, 1 << 16, dtype=np.uint16).view(np.float16)
    finite = allbits[np.isfinite(allbits)]
    f = O.fix24(finite)
    assert np.array_equal(f.astype(np.float64) * 2.0 ** -24, finite.astype(np.float64))
    assert int(np.abs(f).max()) < 1 << 40


def test_selection_lowers_logit_error():
    """Eq. 4-5: keeping the channels with the largest expected |Q eps| at higher
    precision lowers the logit error; the query-aware score does at least as
    well as the error-only one on data whose query outliers are independent of
    the key outliers, and both beat plain 2-bit."""
    import synth_inputs as S
    K, V, _ = S.heavy_tailed_kv(1, 1, 2, 512)
    Q = S.outlier_queries(1, 1, 14, 64)
    R, Gk = 128, 128

    def logit_rmse(score_mode, k4):
        cfg = O.OracleConfig(B=1, Hq=14, Hkv=2, D=128, T_max=512, Gk=Gk, Gv=128, R=R, k4=k4, k16=0,
                             score_mode=score_mode, flush_mode=1)
        c = O.OracleCache(cfg)
        c.accumulate_queries(Q)
        c.append(K, V)
        err = 0.0
        for j in range(2):
            Kh, _ = c.dequantized(j)
            E = Q[0, 7 * j:7 * j + 7].astype(np.float64).reshape(-1, 128) @ (K[0, j].astype(np.float64) - Kh).T
            err += float((E ** 2).mean())
        return err ** 0.5

    none, s_only, full = logit_rmse(1, 0), logit_rmse(1, 16), logit_rmse(0, 16)
    assert full <= s_only * 1.001 <= none * 1.001
    assert full < none * 0.9
