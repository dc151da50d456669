"""Pins of the oracle's packed layout and of its attention (Section 3.1, Eq. 1,
over keys/values dequantized by Eq. 3).  CPU only."""
import dataclasses
import math

import numpy as np
import pytest

from oracle import mixkvq_oracle as O


def _f16(raw, off):
    return float(np.frombuffer(raw[off:off + 2].tobytes(), dtype=np.float16)[0])


def _u32(raw, off):
    return int(np.frombuffer(raw[off:off + 4].tobytes(), dtype=np.uint32)[0])


def _bit2(i):
    """Bit offset of two-bit code i of a word: even codes low half-word, odd codes high half-word."""
    return 16 * (i & 1) + 2 * (i >> 1)


def _bit4(i):
    return 16 * (i & 1) + 4 * (i >> 1)


def brute_force_from_bytes(cfg, recs, res_k, res_v, n_res, q16, scale):
    """Decode attention written as explicit Python loops that read the packed
    block records bit by bit (layout as documented in block_layout) and apply
    Eq. 3 and Eq. 1 in Python floats (binary64)."""
    lay = O.block_layout(cfg)
    P, nb, _ = recs.shape
    out = np.zeros((cfg.B, cfg.Hq, cfg.D))
    lse = np.zeros((cfg.B, cfg.Hq))
    for p in range(P):
        Kt, Vt = [], []
        for blk in range(nb):
            raw = recs[p, blk]
            sel = [int(raw[lay.off_idx + i]) for i in range(cfg.ks)]
            hi16, hi4 = sel[:cfg.k16], sel[cfg.k16:]      # 255 marks an unused entry (threshold policy)
            lo = [d for d in range(cfg.D) if d not in sel]
            for t in range(O.rec_tokens(cfg)):
                grp = t // cfg.Gk
                krow = [0.0] * cfg.D
                for i, d in enumerate(lo):
                    w = _u32(raw, lay.off_klo + 4 * (t * lay.Wlo + i // 16))
                    c = (w >> _bit2(i % 16)) & 3
                    s = _f16(raw, lay.off_klo_s + 2 * (grp * lay.NLp + i))
                    z = _f16(raw, lay.off_klo_z + 2 * (grp * lay.NLp + i))
                    krow[d] = c * s + z
                for i, d in enumerate(hi4):
                    if d == 255:
                        continue
                    w = _u32(raw, lay.off_k4 + 4 * (t * lay.W4 + i // 8))
                    c = (w >> _bit4(i % 8)) & 15
                    s = _f16(raw, lay.off_k4_s + 2 * (grp * cfg.k4 + i))
                    z = _f16(raw, lay.off_k4_z + 2 * (grp * cfg.k4 + i))
                    krow[d] = c * s + z
                for i, d in enumerate(hi16):
                    if d == 255:
                        continue
                    krow[d] = _f16(raw, lay.off_k16 + 2 * (t * cfg.k16 + i))
                vrow = [0.0] * cfg.D
                if lay.v_interleave:
                    # word j of a 64-token span: codes 0..7 = tokens 8j.. of its first 32 tokens, 8..15 = 8j.. of its second 32
                    span, r = divmod(t, 64)
                    word, code = 4 * span + (r % 32) // 8, r % 8 + 8 * (r // 32)
                else:
                    word, code = t // 16, t % 16
                for d in range(cfg.D):
                    w = _u32(raw, lay.off_v + 4 * (word * cfg.D + d))
                    c = (w >> _bit2(code)) & 3
                    vg = d // cfg.Gv
                    s = _f16(raw, lay.off_v_s + 2 * (t * lay.NVG + vg))
                    z = _f16(raw, lay.off_v_z + 2 * (t * lay.NVG + vg))
                    vrow[d] = c * s + z
                Kt.append(krow)
                Vt.append(vrow)
        for t in range(n_res):
            Kt.append([float(x) for x in res_k[p, t]])
            Vt.append([float(x) for x in res_v[p, t]])
        b, j = divmod(p, cfg.Hkv)
        for hh in range(cfg.g):
            h = j * cfg.g + hh
            qv = [float(x) for x in q16[b, h]]
            logits = [scale * sum(qv[d] * kr[d] for d in range(cfg.D)) for kr in Kt]
            m = max(logits)
            e = [math.exp(x - m) for x in logits]
            l = sum(e)
            for d in range(cfg.D):
                out[b, h, d] = sum(e[t] * Vt[t][d] for t in range(len(Vt))) / l
            lse[b, h] = m + math.log(l)
    return out, lse


def _tiny_cache(k4, k16, Gk=16, Gv=16, D=32, R=16, T=56, Hq=4, Hkv=2, B=2, seed=20, flush_mode=0, **more):
    rng = np.random.default_rng(seed)
    cfg = O.OracleConfig(B=B, Hq=Hq, Hkv=Hkv, D=D, T_max=128, Gk=Gk, Gv=Gv, R=R, k4=k4, k16=k16,
                         flush_mode=flush_mode, **more)
    K = (rng.standard_normal((B, Hkv, T, D)) * rng.uniform(0.5, 6, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    Qp = rng.standard_normal((B, Hq, 9, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    cache = O.OracleCache(cfg)
    sel = cache.select_channels(Qp, K)
    cache.append(K, V, sel)
    return cfg, cache, K, V, q


@pytest.mark.parametrize("k4,k16,Gk,Gv", [(8, 0, 16, 16), (0, 4, 8, 32), (8, 6, 16, 8), (0, 0, 16, 32)])
def test_attention_equals_brute_force_over_packed_bytes(k4, k16, Gk, Gv):
    cfg, cache, K, V, q = _tiny_cache(k4, k16, Gk, Gv)
    assert cache.n_quant == 48 and cache.n_res == 8
    out, lse = cache.decode_attention(q)
    ref_out, ref_lse = brute_force_from_bytes(cfg, cache.packed_blocks(), cache.res_k, cache.res_v,
                                              cache.n_res, q, 1.0 / math.sqrt(cfg.D))
    assert np.allclose(out, ref_out, rtol=1e-11, atol=1e-12)
    assert np.allclose(lse, ref_lse, rtol=1e-12, atol=1e-12)


def test_brute_force_over_packed_bytes_with_interleaved_value_words_and_thresholds():
    """Key groups of 32 tokens in blocks of 64 (value words interleaved over the two key groups) and the threshold
    policy with partly used channel lists: the bytes still decode to what the oracle attends over."""
    cfg, cache, K, V, q = _tiny_cache(8, 4, Gk=32, Gv=16, R=64, T=100, B=1, policy=1, tau16=8.0, tau4=6.0)
    assert cache.n_quant == 64 and cache.n_res == 36 and O.block_layout(cfg).v_interleave == 1
    used = [int((b.sel != O.NO_CHANNEL).sum()) for blocks in cache.blocks for b in blocks]
    assert all(0 < u < 12 for u in used), used
    out, lse = cache.decode_attention(q)
    ref_out, ref_lse = brute_force_from_bytes(cfg, cache.packed_blocks(), cache.res_k, cache.res_v,
                                              cache.n_res, q, 1.0 / math.sqrt(cfg.D))
    assert np.allclose(out, ref_out, rtol=1e-11, atol=1e-12)
    assert np.allclose(lse, ref_lse, rtol=1e-12, atol=1e-12)


def test_residual_length_256_is_stored_as_two_records_per_block():
    """R = 256 (the largest residual length of the ablation in Appendix E): a block is scored over its 256 tokens and
    stored as two records of 128 tokens with the same channel list; the bytes decode to what the oracle attends
    over, and the counts follow the closed form n_q = R (ceil(n / R) - 1)."""
    rng = np.random.default_rng(77)
    B, Hq, Hkv, D, T = 1, 2, 1, 32, 600
    cfg = O.OracleConfig(B=B, Hq=Hq, Hkv=Hkv, D=D, T_max=1024, Gk=64, Gv=16, R=256, k4=8, k16=0)
    assert O.rec_tokens(cfg) == 128
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    # a channel that is wide only in the SECOND half of the first block: the block's one selection must see it
    K[0, 0, 128:256, 5] *= np.float16(40.0)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    cache = O.OracleCache(cfg)
    cache.accumulate_queries(np.abs(rng.standard_normal((B, Hq, 8, D))).astype(np.float16) + np.float16(1.0))
    cache.append(K, V)                                    # every block scored on its own 256 tokens
    assert (cache.n_quant, cache.n_res) == (512, 88)
    recs = cache.packed_blocks()
    lay = O.block_layout(cfg)
    assert recs.shape == (1, 4, lay.rec_bytes) and lay.NG == 2
    idx = recs[0, :, lay.off_idx:lay.off_idx + cfg.ks]
    assert np.array_equal(idx[0], idx[1]) and np.array_equal(idx[2], idx[3]) and 5 in idx[0]
    assert not np.array_equal(recs[0, 0], recs[0, 1])
    out, lse = cache.decode_attention(q)
    ref_out, ref_lse = brute_force_from_bytes(cfg, recs, cache.res_k, cache.res_v, cache.n_res, q, 1.0 / math.sqrt(D))
    assert np.allclose(out, ref_out, rtol=1e-11, atol=1e-12)
    assert np.allclose(lse, ref_lse, rtol=1e-12, atol=1e-12)
    # one token at a time gives the same bytes
    step = O.OracleCache(cfg)
    step.qacc[:], step.qcnt[:] = cache.qacc, cache.qcnt
    for t in range(T):
        step.append(K[:, :, t:t + 1], V[:, :, t:t + 1])
    assert np.array_equal(step.packed_blocks(), recs)


def test_residual_length_96_with_groups_of_32_is_stored_as_three_records():
    rng = np.random.default_rng(78)
    B, Hq, Hkv, D, T = 1, 2, 1, 32, 250
    cfg = O.OracleConfig(B=B, Hq=Hq, Hkv=Hkv, D=D, T_max=480, Gk=32, Gv=16, R=96, k4=8, k16=0)
    assert O.rec_tokens(cfg) == 32 and O.rec_tokens(dataclasses.replace(cfg, Gk=96)) == 96
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    K[0, 0, 64:96, 7] *= np.float16(40.0)        # wide only in the LAST third of the first block
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    cache = O.OracleCache(cfg)
    cache.accumulate_queries(np.abs(rng.standard_normal((B, Hq, 8, D))).astype(np.float16) + np.float16(1.0))
    cache.append(K, V)
    assert (cache.n_quant, cache.n_res) == (192, 58)
    recs, lay = cache.packed_blocks(), O.block_layout(cfg)
    assert recs.shape == (1, 6, lay.rec_bytes) and lay.NG == 1 and lay.v_interleave == 0
    idx = recs[0, :, lay.off_idx:lay.off_idx + cfg.ks]
    assert np.array_equal(idx[0], idx[1]) and np.array_equal(idx[0], idx[2]) and 7 in idx[0]
    out, lse = cache.decode_attention(q)
    ref_out, ref_lse = brute_force_from_bytes(cfg, recs, cache.res_k, cache.res_v, cache.n_res, q, 1.0 / math.sqrt(D))
    assert np.allclose(out, ref_out, rtol=1e-11, atol=1e-12)
    assert np.allclose(lse, ref_lse, rtol=1e-12, atol=1e-12)


def _exact_attention(K, V, q, g, scale):
    """softmax(q K^T / sqrt(D)) V on the fp16 inputs in binary64, via logsumexp."""
    from scipy.special import logsumexp
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D))
    lse = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hq):
            kk = K[b, h // g].astype(np.float64)
            x = kk @ q[b, h].astype(np.float64) * scale
            lse[b, h] = logsumexp(x)
            out[b, h] = np.exp(x - lse[b, h]) @ V[b, h // g].astype(np.float64)
    return out, lse


def test_everything_in_residual_window_is_exact_attention():
    rng = np.random.default_rng(21)
    cfg = O.OracleConfig(B=1, Hq=6, Hkv=2, D=32, T_max=64, Gk=16, Gv=16, R=32, k4=8, k16=0)
    K = rng.standard_normal((1, 2, 32, 32)).astype(np.float16)
    V = rng.standard_normal((1, 2, 32, 32)).astype(np.float16)
    q = rng.standard_normal((1, 6, 32)).astype(np.float16)
    cache = O.OracleCache(cfg)
    cache.append(K, V)
    assert cache.n_quant == 0 and cache.n_res == 32
    out, lse = cache.decode_attention(q)
    ro, rl = _exact_attention(K, V, q, 3, 1 / math.sqrt(32))
    assert np.allclose(out, ro, rtol=1e-12, atol=1e-13) and np.allclose(lse, rl, rtol=1e-12)


def test_full_fp16_channel_budget_gives_exact_logits():
    """With every key channel in the fp16 tier the logits (hence lse) are those
    of full-precision attention; the output differs only through 2-bit values."""
    cfg, cache, K, V, q = _tiny_cache(k4=0, k16=32, T=64, flush_mode=1)
    assert cache.n_res == 0
    out, lse = cache.decode_attention(q)
    _, rl = _exact_attention(K, V, q, cfg.g, 1 / math.sqrt(cfg.D))
    assert np.allclose(lse, rl, rtol=1e-12, atol=1e-12)
    # outputs: the same attention weights applied to the dequantized values
    for p in range(cfg.B * cfg.Hkv):
        _, Vh = cache.dequantized(p)
        b, j = divmod(p, cfg.Hkv)
        ro, _ = _exact_attention(K[b:b + 1, j:j + 1], Vh[None, None].astype(np.float64),
                                 q[b:b + 1, j * cfg.g:(j + 1) * cfg.g], cfg.g, 1 / math.sqrt(cfg.D))
        assert np.allclose(out[b, j * cfg.g:(j + 1) * cfg.g], ro[0], rtol=1e-11, atol=1e-12)


def test_output_is_a_convex_combination_of_values():
    cfg, cache, K, V, q = _tiny_cache(8, 0)
    out, _ = cache.decode_attention(q)
    for p in range(cfg.B * cfg.Hkv):
        _, Vh = cache.dequantized(p)
        b, j = divmod(p, cfg.Hkv)
        o = out[b, j * cfg.g:(j + 1) * cfg.g]
        assert np.all(o <= Vh.max(axis=0) + 1e-12) and np.all(o >= Vh.min(axis=0) - 1e-12)


def test_split_softmax_merge_identity():
    """Attention over token ranges merged by log-sum-exp weights equals attention
    over the whole range (the identity the split-K GPU kernel relies on)."""
    cfg, cache, K, V, q = _tiny_cache(8, 0, T=56)
    out, lse = cache.decode_attention(q)
    scale = 1 / math.sqrt(cfg.D)
    for nsplit in (1, 2, 7):
        for p in range(cfg.B * cfg.Hkv):
            Kh, Vh = cache.dequantized(p)
            b, j = divmod(p, cfg.Hkv)
            for hh in range(cfg.g):
                h = j * cfg.g + hh
                bounds = np.linspace(0, Kh.shape[0], nsplit + 1).astype(int)
                ms, ls, os_ = [], [], []
                for a, e in zip(bounds[:-1], bounds[1:]):
                    x = Kh[a:e] @ q[b, h].astype(np.float64) * scale
                    m = x.max()
                    w = np.exp(x - m)
                    ms.append(m), ls.append(w.sum()), os_.append(w @ Vh[a:e])
                M = max(ms)
                L = sum(l * math.exp(m - M) for m, l in zip(ms, ls))
                Ov = sum(o * math.exp(m - M) for m, o in zip(ms, os_)) / L
                assert np.allclose(Ov, out[b, h], rtol=1e-11, atol=1e-13)
                assert abs(M + math.log(L) - lse[b, h]) < 1e-11


def test_accumulate_q_in_decode_adds_abs_query():
    cfg, cache, K, V, q = _tiny_cache(8, 0)
    before = cache.qacc.copy()
    cache.decode_attention(q, accumulate_q=True)
    add = np.abs(q.astype(np.float64)).reshape(cfg.B, cfg.Hkv, cfg.g, cfg.D).sum(axis=2) * 2.0 ** 24
    assert np.array_equal((cache.qacc - before).astype(np.float64).reshape(cfg.B, cfg.Hkv, cfg.D), add)
