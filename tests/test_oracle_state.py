"""Pins of the oracle's cache state machine (Appendix D.1: residual buffer and
lazy flush every R tokens) and of the closed forms used for reporting.  CPU only."""
import os

import numpy as np
import pytest

from oracle import mixkvq_oracle as O


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_figures.txt")
    vals = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def _cfg(R=16, flush_mode=0, **kw):
    base = dict(B=1, Hq=2, Hkv=1, D=32, T_max=256, Gk=16, Gv=16, R=R, k4=8, k16=0, flush_mode=flush_mode)
    base.update(kw)
    return O.OracleConfig(**base)


def _kv(rng, n, D=32):
    return (rng.standard_normal((1, 1, n, D)).astype(np.float16),
            rng.standard_normal((1, 1, n, D)).astype(np.float16))


@pytest.mark.parametrize("n", [1, 15, 16, 17, 32, 33, 100, 128])
def test_deferred_prefill_counts_closed_form(n):
    """The newest <= R tokens stay in full precision: n_q = R (ceil(n/R) - 1)."""
    rng = np.random.default_rng(30)
    c = O.OracleCache(_cfg())
    c.append(*_kv(rng, n))
    assert c.n_quant == 16 * (-(-n // 16) - 1)
    assert c.n_res == n - c.n_quant and 1 <= c.n_res <= 16
    assert len(c.blocks[0]) == c.n_quant // 16


def test_configured_prompts_leave_a_full_window():
    for n, R, nq in ((1024, 32, 992), (32768, 128, 32640), (131072, 128, 130944)):
        assert R * (-(-n // R) - 1) == nq


@pytest.mark.parametrize("n", [1, 16, 17, 47, 48])
def test_eager_counts(n):
    rng = np.random.default_rng(31)
    c = O.OracleCache(_cfg(flush_mode=1))
    c.append(*_kv(rng, n))
    assert c.n_quant == 16 * (n // 16) and c.n_res == n % 16


@pytest.mark.parametrize("flush_mode", [0, 1])
def test_one_by_one_equals_chunked(flush_mode):
    rng = np.random.default_rng(32)
    K, V = _kv(rng, 75)
    Q = rng.standard_normal((1, 2, 11, 32)).astype(np.float16)
    a = O.OracleCache(_cfg(flush_mode=flush_mode))
    b = O.OracleCache(_cfg(flush_mode=flush_mode))
    d = O.OracleCache(_cfg(flush_mode=flush_mode))
    for c in (a, b, d):
        c.accumulate_queries(Q)
    a.append(K, V)
    for t in range(75):
        b.append(K[:, :, t:t + 1], V[:, :, t:t + 1])
    for lo, hi in ((0, 5), (5, 40), (40, 41), (41, 75)):
        d.append(K[:, :, lo:hi], V[:, :, lo:hi])
    for c in (b, d):
        assert (c.n_quant, c.n_res) == (a.n_quant, a.n_res)
        assert np.array_equal(c.packed_blocks(), a.packed_blocks())
        assert np.array_equal(c.res_k[:, :c.n_res], a.res_k[:, :a.n_res])
        assert np.array_equal(c.res_v[:, :c.n_res], a.res_v[:, :a.n_res])


def test_flush_rate_is_one_per_R_decode_steps():
    """Appendix F: with R = 32 channel selection runs on 3.13 % (= 1/32) of decode steps."""
    g = _golden()
    rng = np.random.default_rng(33)
    c = O.OracleCache(_cfg(R=32, Gk=32, T_max=32 * 40))
    c.append(*_kv(rng, 32))
    steps = 32 * 20
    for _ in range(steps):
        c.append(*_kv(rng, 1))
    assert c.n_flush_calls * 32 == steps
    assert abs(100.0 * c.n_flush_calls / steps - g["selection_call_rate_percent"]) <= 0.005 + 1e-9   # 3.125 printed as 3.13


def test_each_decode_flush_reselects_from_running_accumulator():
    rng = np.random.default_rng(34)
    cfg = _cfg(R=16)
    c = O.OracleCache(cfg)
    K, V = _kv(rng, 16)
    c.append(K, V)
    q1 = np.zeros((1, 2, 32), dtype=np.float16)
    q1[..., :8] = 1.0
    c.decode_attention(q1, accumulate_q=True)
    K2, V2 = _kv(rng, 16)
    c.append(K2[:, :, :1], V2[:, :, :1])              # triggers the flush of the first block
    assert c.blocks[0][0].sel.tolist() == list(range(8))
    q2 = np.zeros((1, 2, 32), dtype=np.float16)
    q2[..., 20:28] = 50.0
    c.decode_attention(q2, accumulate_q=True)
    c.append(K2[:, :, 1:], V2[:, :, 1:])
    c.append(K[:, :, :1], V[:, :, :1])                # flush of the second block
    assert c.blocks[0][1].sel.tolist() == list(range(20, 28))


def test_windowed_accumulator_resets_on_flush():
    rng = np.random.default_rng(35)
    c = O.OracleCache(_cfg(R=16, qacc_reset_on_flush=1))
    c.accumulate_queries(rng.standard_normal((1, 2, 4, 32)).astype(np.float16))
    c.append(*_kv(rng, 16))
    assert c.qacc.any()
    c.append(*_kv(rng, 1))
    assert not c.qacc.any() and not c.qcnt.any()


def test_capacity_overflow_raises_and_leaves_cache_unchanged():
    rng = np.random.default_rng(36)
    c = O.OracleCache(_cfg(T_max=32))
    c.append(*_kv(rng, 48))
    assert c.n_quant == 32
    with pytest.raises(OverflowError):
        c.append(*_kv(rng, 17))
    assert c.n_quant == 32 and c.n_res == 16


def test_record_layout_closed_form():
    cfg = O.OracleConfig(B=8, Hq=28, Hkv=4, D=128, T_max=32768, Gk=128, Gv=128, R=128, k4=16, k16=0)
    lay = O.block_layout(cfg)
    assert (lay.NL, lay.Wlo, lay.W4, lay.NG, lay.NVG) == (112, 7, 2, 1, 1)
    # the record is the algorithmic bytes of 128 tokens plus the 16-byte plane of derived scale maxima
    assert lay.rec_bytes == 9744 + 16
    assert (lay.rec_bytes - 16) * 255 + 128 * 128 * 4 + 7 * 128 * 4 == O.algorithmic_bytes_per_pair(cfg, 32640, 128)
    for name in ("off_idx", "off_kmax", "off_klo_s", "off_klo_z", "off_k4_s", "off_k4_z", "off_klo", "off_k4", "off_k16",
                 "off_v", "off_v_s", "off_v_z"):
        assert getattr(lay, name) % 16 == 0


def test_algorithmic_bytes_per_configuration():
    mk = lambda **kw: O.OracleConfig(T_max=1 << 20, **kw)
    c0 = mk(B=1, Hq=1, Hkv=1, D=128, Gk=32, Gv=32, R=32, k4=8, k16=0)
    c1 = mk(B=8, Hq=28, Hkv=4, D=128, Gk=128, Gv=128, R=128, k4=16, k16=0)
    c2 = mk(B=64, Hq=40, Hkv=8, D=128, Gk=128, Gv=128, R=128, k4=0, k16=12)
    c3 = mk(B=4, Hq=40, Hkv=8, D=128, Gk=128, Gv=128, R=128, k4=16, k16=0)
    assert O.algorithmic_bytes_per_pair(c0, 992, 32) == 114360
    assert O.algorithmic_bytes_per_pair(c1, 32640, 128) == 2553840
    assert O.algorithmic_bytes_per_pair(c2, 32640, 128) == 3094436
    assert O.algorithmic_bytes_per_pair(c3, 130944, 128) == 10036208


def test_effective_bits_closed_form():
    """Appendix C: B_eff = mean of b_i over the key channels, b_i in {16, 4, 2}."""
    g = _golden()
    assert O.effective_key_bits(128, 0, 16) == 2.25
    assert O.effective_key_bits(128, 12, 0) == 3.3125
    assert O.effective_key_bits(128, 0, 8) == 2.125
    assert O.effective_key_bits(128, 128, 0) == 16 and O.effective_key_bits(128, 0, 0) == 2
    # "16-bit -> 3.4-bit" saving
    assert 100 * (1 - g["effective_bits_r1_qwen_7b"] / 16) > g["memory_saving_percent_floor"]


def test_fp16_footprint_example_of_the_introduction():
    g = _golden()
    total = (g["kv_example_layers"] * g["kv_example_batch"] * g["kv_example_kv_heads"] * g["kv_example_tokens"]
             * g["kv_example_head_dim"] * 2 * 2)
    assert total / 2 ** 30 == g["kv_fp16_footprint_gb"]


@pytest.mark.parametrize("Gk,R,interleave", [(32, 128, 1), (32, 64, 1), (32, 32, 0), (64, 128, 0), (16, 64, 0)])
def test_value_words_hold_every_token_once(Gk, R, interleave):
    """Value codes read back from the packed record with the bit positions of the layout comment (code i at bit
    16 (i & 1) + 2 (i >> 1)) and the word's token list: every (token, channel) code is recovered, whether the
    words take consecutive tokens or are interleaved over the two key groups of a 64-token span."""
    rng = np.random.default_rng(21)
    cfg = O.OracleConfig(B=1, Hq=1, Hkv=1, D=128, T_max=R, Gk=Gk, Gv=64, R=R, k4=8, k16=0)
    lay = O.block_layout(cfg)
    assert lay.v_interleave == interleave
    K = rng.standard_normal((R, 128)).astype(np.float16)
    V = rng.standard_normal((R, 128)).astype(np.float16)
    blk = O.quantize_block(cfg, K, V, np.arange(8, dtype=np.uint8))
    rec = O.pack_record(cfg, blk)
    words = rec[lay.off_v:lay.off_v_s].view(np.uint32).reshape(R // 16, 128)
    seen = np.zeros(R, dtype=int)
    for tg in range(R // 16):
        toks = [O.value_word_token(tg, i, interleave) for i in range(16)]
        for i, t in enumerate(toks):
            seen[t] += 1
            got = (words[tg] >> np.uint32(16 * (i & 1) + 2 * (i >> 1))) & np.uint32(3)
            assert np.array_equal(got.astype(np.uint8), blk.v_codes[t])
        if interleave:   # codes 0..7 from the first key group of the span, codes 8..15 from the second
            assert {t // 32 for t in toks[:8]} == {2 * (tg // 4)} and {t // 32 for t in toks[8:]} == {2 * (tg // 4) + 1}
        else:
            assert toks == list(range(16 * tg, 16 * tg + 16))
    assert np.all(seen == 1)


@pytest.mark.parametrize("n", [1, 31, 32, 33, 48, 49, 100])
@pytest.mark.parametrize("flush_mode", [0, 1])
def test_sink_tokens_counts_and_contents(n, flush_mode):
    """The first `sink` tokens never leave full precision (Appendix E fixes a sink length of 32); everything after
    them follows the window / flush rules as if the sequence started there."""
    rng = np.random.default_rng(40)
    K, V = _kv(rng, n)
    c = O.OracleCache(_cfg(sink=32, flush_mode=flush_mode))
    for lo, hi in ((0, min(n, 5)), (min(n, 5), min(n, 40)), (min(n, 40), n)):     # chunks that straddle the sink's end
        if hi > lo:
            c.append(K[:, :, lo:hi], V[:, :, lo:hi])
    assert c.n_sink == min(n, 32)
    assert np.array_equal(c.sink_k[0, :c.n_sink], K[0, 0, :c.n_sink]) and np.array_equal(c.sink_v[0, :c.n_sink], V[0, 0, :c.n_sink])
    rest = n - c.n_sink
    plain = O.OracleCache(_cfg(flush_mode=flush_mode))
    if rest:
        plain.append(K[:, :, 32:], V[:, :, 32:])
    assert (c.n_quant, c.n_res) == (plain.n_quant, plain.n_res)
    assert c.n_sink + c.n_quant + c.n_res == n
    assert np.array_equal(c.res_k[0, :c.n_res], plain.res_k[0, :plain.n_res])
    if c.n_quant:
        assert np.array_equal(c.packed_blocks(), plain.packed_blocks())
    Kh, Vh = c.dequantized(0)
    assert Kh.shape == (n, 32) and np.array_equal(Kh[:c.n_sink], K[0, 0, :c.n_sink].astype(np.float64))


def test_attention_is_exact_when_all_tokens_sit_in_sink_and_window():
    rng = np.random.default_rng(41)
    K, V = _kv(rng, 44)
    c = O.OracleCache(_cfg(sink=32))
    c.append(K, V)
    assert (c.n_sink, c.n_quant, c.n_res) == (32, 0, 12)
    q = rng.standard_normal((1, 2, 32)).astype(np.float16)
    out, lse = c.decode_attention(q)
    K64, V64 = K[0, 0].astype(np.float64), V[0, 0].astype(np.float64)
    for h in range(2):
        logits = K64 @ q[0, h].astype(np.float64) / np.sqrt(32.0)
        w = np.exp(logits - logits.max())
        assert np.allclose(out[0, h], (w / w.sum()) @ V64, rtol=1e-13, atol=1e-15)
        assert np.isclose(lse[0, h], logits.max() + np.log(w.sum()), rtol=1e-13)
