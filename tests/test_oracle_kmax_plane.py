"""Pin of the derived `kmax` plane of a block record: per key group the largest stored scale over the 2-bit and
the 4-bit tier, then the block's largest value scale.  The plane is read back from the packed bytes with a reader
of its own and compared with the maxima of the scale planes read from the same bytes.  CPU only."""
import struct

import numpy as np
import pytest

from oracle import mixkvq_oracle as O


def _f16s(raw: np.ndarray, off: int, n: int):
    return list(struct.unpack("<%de" % n, raw[off:off + 2 * n].tobytes()))


def _expected_from_bytes(cfg, lay, raw):
    """kmax as its definition says, from the scale planes of the record itself."""
    exp = []
    for grp in range(lay.NG):
        lo = _f16s(raw, lay.off_klo_s + 2 * grp * lay.NLp, lay.NLp)
        hi = _f16s(raw, lay.off_k4_s + 2 * grp * cfg.k4, cfg.k4) if cfg.k4 else []
        exp.append(max(lo + hi))
    vs = _f16s(raw, lay.off_v_s, O.rec_tokens(cfg) * lay.NVG)
    exp.append(max(vs))
    return exp


CASES = [
    dict(R=128, Gk=128, Gv=128, k4=16, k16=0),
    dict(R=128, Gk=32, Gv=32, k4=16, k16=8),
    dict(R=128, Gk=64, Gv=64, k4=0, k16=12),
    dict(R=64, Gk=16, Gv=16, k4=8, k16=0),
    dict(R=256, Gk=128, Gv=128, k4=16, k16=0),       # two records per block
    dict(R=96, Gk=32, Gv=128, k4=8, k16=4),          # three records per block
    dict(R=128, Gk=32, Gv=32, k4=16, k16=8, policy=1, tau16=2.0, tau4=0.3),
    dict(R=32, Gk=32, Gv=128, k4=0, k16=0),
]


@pytest.mark.parametrize("kw", CASES, ids=lambda k: "R%d_G%d_%d_%d%s" % (k["R"], k["Gk"], k["k4"], k["k16"], "_thr" if k.get("policy") else ""))
def test_kmax_plane_is_the_largest_scale_of_each_key_group_and_of_the_values(kw):
    rng = np.random.default_rng(1000 + CASES.index(kw))
    R = kw["R"]
    cfg = O.OracleConfig(B=1, Hq=4, Hkv=2, D=128, T_max=4 * R, **kw)
    lay = O.block_layout(cfg)
    T = 3 * R + 5
    # key groups of different spread along the tokens (so the per-group maxima differ), channels of different spread
    # (so that the largest scale sits in the 4-bit tier for some groups and in the 2-bit tier for others), and value
    # rows of different spread (so the largest value scale sits in one token of one group)
    grp_of_tok = np.arange(T) // kw["Gk"]
    tok_scale = rng.uniform(0.2, 5.0, size=T // kw["Gk"] + 1)[grp_of_tok][None, None, :, None]
    # a few outlier channels: 40 x in even key groups (their 4-bit scale, range / 15, then tops every 2-bit scale,
    # range / 3) and 2 x in odd key groups (where a 2-bit channel has the largest scale)
    # (k16 + 4 of them: the fp16 tier takes the k16 with the widest range, the 4-bit tier the other four)
    outlier = np.zeros(128, dtype=bool)
    outlier[rng.choice(128, size=kw["k16"] + 4, replace=False)] = True
    ch_scale = np.where(outlier[None, :], np.where(grp_of_tok % 2 == 0, 40.0, 2.0)[:, None], 1.0)[None, None]
    K = (rng.standard_normal((1, 2, T, 128)) * tok_scale * ch_scale).astype(np.float16)
    V = (rng.standard_normal((1, 2, T, 128)) * rng.uniform(0.1, 30.0, size=(1, 2, T, 1))).astype(np.float16)
    Q = rng.standard_normal((1, 4, 8, 128)).astype(np.float16)
    oc = O.OracleCache(cfg)
    oc.accumulate_queries(Q)
    oc.append(K, V)                      # every block scored on its own tokens: the tiers differ from block to block
    recs = oc.packed_blocks()
    assert recs.shape[1] == 3 * (R // O.rec_tokens(cfg))
    top_tier = set()
    for p in range(recs.shape[0]):
        for b in range(recs.shape[1]):
            raw = recs[p, b]
            got = _f16s(raw, lay.off_kmax, lay.NG + 1)
            exp = _expected_from_bytes(cfg, lay, raw)
            assert got == exp, (p, b, got, exp)
            assert all(x >= 0 for x in got)
            # the bytes after the plane's NG + 1 entries are padding
            pad0, pad1 = lay.off_kmax + 2 * (lay.NG + 1), lay.off_klo_s
            assert not raw[pad0:pad1].any()
            if cfg.k4:
                for grp in range(lay.NG):
                    hi = max(_f16s(raw, lay.off_k4_s + 2 * grp * cfg.k4, cfg.k4))
                    top_tier.add("k4" if hi == got[grp] else "klo")
    if cfg.k4 and not kw.get("policy"):
        # the data exercise both outcomes, so a plane built from one tier alone would fail above
        assert top_tier == {"k4", "klo"}, top_tier


def test_kmax_entries_differ_between_groups_and_from_the_value_entry():
    """Guards the test above against a vacuous pass: on its kind of data the entries of the plane are all different,
    so a plane with the maxima in another order, or with the value entry in a key slot, cannot equal the expected one."""
    rng = np.random.default_rng(3)
    cfg = O.OracleConfig(B=1, Hq=2, Hkv=1, D=128, T_max=256, R=128, Gk=32, Gv=32, k4=16, k16=0)
    lay = O.block_layout(cfg)
    per_token = np.concatenate([np.repeat(np.array([0.5, 1.0, 2.0, 4.0]), 32), [1.0]])      # four key groups + 1 token
    K = (rng.standard_normal((1, 1, 129, 128)) * per_token[None, None, :, None]).astype(np.float16)
    V = (rng.standard_normal((1, 1, 129, 128)) * 9.0).astype(np.float16)
    oc = O.OracleCache(cfg)
    oc.accumulate_queries(rng.standard_normal((1, 2, 4, 128)).astype(np.float16))
    oc.append(K, V)
    raw = oc.packed_blocks()[0, 0]
    got = _f16s(raw, lay.off_kmax, lay.NG + 1)
    assert len(set(got)) == lay.NG + 1
    assert got[0] < got[1] < got[2] < got[3]          # key groups in token order
    assert got[4] == max(_f16s(raw, lay.off_v_s, 128 * lay.NVG))
