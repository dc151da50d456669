"""CPU oracle for the MixKVQ hot path (TEST INFRASTRUCTURE, not a product path).

A plain, slow, numpy implementation of what the GPU library computes: the
asymmetric min/max quantizer (Section 3.2, Eq. 2-3), the query-aware channel
salience score (Section 4.2, Eq. 6-8) with a top-k channel budget or the
three-tier threshold rule of Section 4.2, the lazy residual-buffer flush (Appendix D.1), the running |q| accumulator
(Appendix D.2) and decode attention (Section 3.1, Eq. 1) over the resulting
mixed-precision cache, in fp64.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

Precision rules (so that "bit-exact" has a meaning):
  * quantizer parameters and codes follow IEEE binary32 steps, listed in
    `group_params` and `encode`;
  * the |q| accumulator and the key range are exact integers (units of 2^-24,
    the spacing of the smallest fp16 subnormal), so sums are order-independent;
  * the score is one binary64 product of the two (converted) integers;
  * attention is binary64 throughout.

Pins (tests/test_oracle_*.py): Eq. 2-3 error bound |x - x~| <= s/2, code
monotonicity and end points, top-k against exact rational arithmetic, Eq. 6-8
in float64, brute-force attention loops, exact attention when every channel is
kept in fp16 / every token sits in the residual window, split invariance,
closed-form state-machine counts and byte counts; the threshold rule against
the three inequalities of Section 4.2 in exact rational arithmetic and against
the top-k rule where the two must coincide.  The paper's model-quality
numbers (accuracy, perplexity) are parity unpinned here: they need weights and
datasets that are not available.
"""
from __future__ import annotations

import dataclasses
import math
import numpy as np

FIX_SHIFT = 24  # every finite fp16 is an integer multiple of 2**-24


# --------------------------------------------------------------------------
# configuration
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class OracleConfig:
    B: int
    Hq: int
    Hkv: int
    D: int
    T_max: int
    Gk: int
    Gv: int
    R: int
    k4: int
    k16: int
    flush_mode: int = 0           # 0 deferred (newest <= R tokens stay fp16), 1 eager
    score_mode: int = 0           # 0: A = I*S (Eq. 8); 1: A = S (error-only ablation, Appendix E)
    qacc_reset_on_flush: int = 0  # 0: running since sequence start (Appendix D.2); 1: per window (Section 4.2)
    policy: int = 0               # 0: the k16 + k4 best channels; 1: thresholds of Section 4.2, k16 / k4 are capacities
    tau16: float = math.inf       # policy 1: A_d > tau16 -> fp16 tier
    tau4: float = math.inf        # policy 1: tau4 < A_d <= tau16 -> 4-bit tier
    sink: int = 0                 # the first `sink` tokens of a sequence stay in full precision for good (Appendix E)
    in_dtype: int = 0             # mirrors the library's field; the oracle itself always takes binary16 arrays (a
                                  # bfloat16 input is converted with bf16_bits_to_f16 before it is handed over)

    @property
    def g(self):
        return self.Hq // self.Hkv

    @property
    def ks(self):
        return self.k4 + self.k16


# --------------------------------------------------------------------------
# input precision
# --------------------------------------------------------------------------
def bf16_bits_to_f16(bits: np.ndarray) -> np.ndarray:
    """The cache works on binary16 values.  A bfloat16 input (the precision of the paper's models, Section 5)
    enters it as the nearest binary16 (ties to even), saturated at +-65504: exact wherever binary16 has the range
    (bfloat16 carries 8 significant bits, binary16 11), rounded only inside the binary16 subnormals.
    `bits`: uint16 bfloat16 patterns (finite)."""
    x32 = (np.asarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)
    return np.clip(x32, np.float32(-65504.0), np.float32(65504.0)).astype(np.float16)


# --------------------------------------------------------------------------
# Eq. 2-3: asymmetric B-bit min/max quantizer
# --------------------------------------------------------------------------
def group_params(x16: np.ndarray, bits: int, axis: int):
    """Scale and zero-point of Eq. 2-3 for groups laid along `axis`.

    z = min(X) (stored as fp16; a -0 minimum or maximum is taken as +0),
    s = (max(X) - min(X)) / (2^B - 1): binary32 subtract, binary32 divide,
    then round-to-nearest-even to fp16 (the stored value)."""
    assert x16.dtype == np.float16
    mn = x16.min(axis=axis).astype(np.float32) + np.float32(0.0)   # "+ 0" turns -0 into +0
    mx = x16.max(axis=axis).astype(np.float32) + np.float32(0.0)
    z16 = mn.astype(np.float16)
    d32 = mx - mn
    s32 = d32 / np.float32((1 << bits) - 1)
    s16 = s32.astype(np.float16)
    return s16, z16


def encode(x16: np.ndarray, s16: np.ndarray, z16: np.ndarray, bits: int) -> np.ndarray:
    """Eq. 2: round((x - z) / s) in binary32 with round-half-to-even, clamped to
    [0, 2^B - 1].  s, z broadcast against x.  A group whose stored scale is 0
    (constant group, or a range that underflows fp16) gets code 0 everywhere."""
    x = x16.astype(np.float32)
    z = z16.astype(np.float32)
    s = s16.astype(np.float32)
    safe = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    y = ((x - z) / safe).astype(np.float32)
    c = np.clip(np.rint(y), 0, (1 << bits) - 1)
    c = np.where(s > 0, c, 0)
    return c.astype(np.uint8)


def decode(c: np.ndarray, s16: np.ndarray, z16: np.ndarray) -> np.ndarray:
    """Eq. 3 in binary64: x~ = c * s + z with the STORED fp16 s and z."""
    return c.astype(np.float64) * s16.astype(np.float64) + z16.astype(np.float64)


def quantize_keys(K16: np.ndarray, chans: np.ndarray, bits: int, Gk: int):
    """Per-channel quantization of keys (Section 4.2: keys are quantized per
    channel; the group is Gk consecutive tokens of one channel).
    K16: [L, D] with L % Gk == 0.  Returns codes [L, n], s16, z16 [L/Gk, n] for
    the n channels listed in `chans` (in that order)."""
    L = K16.shape[0]
    n = len(chans)
    X = K16[:, chans].reshape(L // Gk, Gk, n)
    s16, z16 = group_params(X, bits, axis=1)
    codes = encode(X, s16[:, None, :], z16[:, None, :], bits).reshape(L, n)
    return codes, s16, z16


def quantize_values(V16: np.ndarray, Gv: int):
    """Per-token 2-bit quantization of values (Section 4.2): the group is Gv
    consecutive channels of one token.  V16: [L, D].  Returns codes [L, D],
    s16, z16 [L, D/Gv]."""
    L, D = V16.shape
    X = V16.reshape(L, D // Gv, Gv)
    s16, z16 = group_params(X, 2, axis=2)
    codes = encode(X, s16[..., None], z16[..., None], 2).reshape(L, D)
    return codes, s16, z16


# --------------------------------------------------------------------------
# Eq. 6-8: salience score and channel selection
# --------------------------------------------------------------------------
def fix24(x16: np.ndarray) -> np.ndarray:
    """x * 2^24 as an exact int64 (x is fp16)."""
    return np.rint(x16.astype(np.float64) * float(1 << FIX_SHIFT)).astype(np.int64)


def abs_query_sum(Q16: np.ndarray) -> np.ndarray:
    """Sum of |q| over every axis but the last, in units of 2^-24 (exact).
    Eq. 6 is this sum divided by the number of summed query vectors; with
    grouped-query attention the sum also runs over the query heads that share
    the KV head (Appendix D, first paragraph)."""
    D = Q16.shape[-1]
    return np.abs(fix24(Q16)).reshape(-1, D).sum(axis=0, dtype=np.int64).astype(np.uint64)


def key_range(K16: np.ndarray) -> np.ndarray:
    """max(k_d) - min(k_d) over the tokens of K16 [L, D], in units of 2^-24
    (exact).  Eq. 7 is this divided by (2^B - 1)."""
    f = fix24(K16)
    return (f.max(axis=0) - f.min(axis=0)).astype(np.int64)


def salience(qacc: np.ndarray, rng: np.ndarray, score_mode: int = 0) -> np.ndarray:
    """Eq. 8 up to positive constants common to all channels of the head:
    A_d = (sum|q|_d) * (range_d), one binary64 multiply of the two integers
    converted to binary64.  score_mode 1 is the error-only ablation A_d = S_d."""
    if score_mode == 1:
        return rng.astype(np.float64)
    return qacc.astype(np.float64) * rng.astype(np.float64)


def select_channels(A: np.ndarray, k16: int, k4: int) -> np.ndarray:
    """Top-(k16+k4) channels of the score; ties go to the lower channel index.
    The k16 best go to the fp16 tier, the next k4 to the 4-bit tier; each tier
    is stored in ascending channel order.  Returns uint8 [k16 + k4]."""
    D = A.shape[0]
    order = sorted(range(D), key=lambda d: (-float(A[d]), d))
    hi16 = sorted(order[:k16])
    hi4 = sorted(order[k16:k16 + k4])
    return np.array(hi16 + hi4, dtype=np.uint8)


NO_CHANNEL = 255  # an unused entry of a channel list (threshold policy)


def threshold_in_score_units(tau: float, qcnt: int, score_mode: int = 0) -> float:
    """The threshold of Section 4.2 carried over to the units of `salience`.

    In real units A_d = I_d * S_d with I_d = (sum|q|_d 2^-24) / count (Eq. 6) and
    S_d = (range_d 2^-24) / (2^2 - 1) (Eq. 7 for the two-bit quantizer a channel
    gets unless it is promoted), so  A_d > tau  <=>  sum|q|_d * range_d > tau * 3 * 2^48 * count.
    The right-hand side is formed in binary64, left to right: (tau * 3) * 2^48
    (exact) * count.  With the error-only score, S_d > tau <=> range_d > tau * 3 * 2^24."""
    if score_mode == 1:
        return (float(tau) * 3.0) * float(1 << FIX_SHIFT)
    return ((float(tau) * 3.0) * float(1 << (2 * FIX_SHIFT))) * float(int(qcnt))


def select_channels_threshold(A: np.ndarray, thr16: float, thr4: float, cap16: int, cap4: int) -> np.ndarray:
    """The three-tier rule of Section 4.2 on the scores A (thresholds already in
    the units of A): A_d > thr16 -> fp16, thr4 < A_d <= thr16 -> 4 bit, else 2 bit.
    The record has room for cap16 fp16 channels and cap4 four-bit channels per
    block: when more pass a threshold the best by (score, lower index) keep
    the tier and the others fall to the next one down.  Returns uint8
    [cap16 + cap4]: the fp16 tier ascending, filled up with NO_CHANNEL, then the
    4-bit tier likewise."""
    D = A.shape[0]
    order = sorted(range(D), key=lambda d: (-float(A[d]), d))
    hi16 = [d for d in order if float(A[d]) > thr16][:cap16]
    # candidates of the 4-bit tier: channels between the thresholds, and channels above thr16 that found no fp16 place
    cand4 = [d for d in order if d not in hi16 and (float(A[d]) > thr4 or float(A[d]) > thr16)]
    hi4 = cand4[:cap4]
    out = np.full(cap16 + cap4, NO_CHANNEL, dtype=np.uint8)
    out[:len(hi16)] = sorted(hi16)
    out[cap16:cap16 + len(hi4)] = sorted(hi4)
    return out


def tier_lists(sel: np.ndarray, k16: int):
    """(fp16-tier channels, 4-bit-tier channels) of a stored selection, unused entries dropped."""
    sel = np.asarray(sel, dtype=np.uint8)
    hi16 = sel[:k16]
    hi4 = sel[k16:]
    return hi16[hi16 != NO_CHANNEL].astype(np.int64), hi4[hi4 != NO_CHANNEL].astype(np.int64)


def lo_channels(sel: np.ndarray, D: int) -> np.ndarray:
    """The non-salient channels in ascending order."""
    mask = np.ones(D, dtype=bool)
    sel = np.asarray(sel).astype(np.int64)
    mask[sel[sel != NO_CHANNEL]] = False
    return np.nonzero(mask)[0]


# --------------------------------------------------------------------------
# physical layout of one quantized block of R tokens ("block record")
# --------------------------------------------------------------------------
def _al16(n: int) -> int:
    return (n + 15) // 16 * 16


@dataclasses.dataclass(frozen=True)
class BlockLayout:
    NL: int      # 2-bit key channels
    Wlo: int     # u32 words per token for the 2-bit key plane
    NLp: int     # 16 * Wlo
    NG: int      # key groups per block
    NVG: int     # value groups per token
    W4: int      # u32 words per token for the 4-bit key plane
    off_idx: int
    off_kmax: int
    off_klo_s: int
    off_klo_z: int
    off_k4_s: int
    off_k4_z: int
    off_klo: int
    off_k4: int
    off_k16: int
    off_v: int
    off_v_s: int
    off_v_z: int
    rec_bytes: int
    v_interleave: int   # 1: value words take their 16 tokens from both 32-token halves of a 64-token span


MAX_REC_TOKENS = 128


def rec_tokens(cfg: OracleConfig) -> int:
    """Tokens one stored record holds.  A flushed block of R tokens is stored as R / rec_tokens records, all with
    the block's channel selection: R = 256 as two records of 128 tokens, R = 96 with key groups that divide 32 as
    three records of 32 tokens, every other R as one record.  (A storage choice: quantization groups never straddle
    a record.)"""
    if cfg.R > MAX_REC_TOKENS:
        return MAX_REC_TOKENS
    if cfg.R == 96 and 32 % cfg.Gk == 0:
        return 32
    return cfg.R


def block_layout(cfg: OracleConfig) -> BlockLayout:
    """Byte offsets of the planes inside one block record (R below: rec_tokens(cfg)).  Every plane starts
    on a 16-byte boundary; padding bytes are zero.
      idx    u8  [ks]               fp16-tier channels ascending, then 4-bit tier ascending (threshold policy:
                                    each tier filled up to its capacity with NO_CHANNEL)
      kmax   f16 [NG + 1]           [NG]: largest stored value scale of the block; [g < NG]:
                                    largest stored scale of the group's 2-bit and 4-bit channels (derived
                                    metadata: lets a reader normalise the scales without scanning them)
      klo_s  f16 [NG][NLp]          scales of the 2-bit key channels (ascending non-salient channels)
      klo_z  f16 [NG][NLp]          zero-points
      k4_s   f16 [NG][k4]           scales of the 4-bit tier (tier order)
      k4_z   f16 [NG][k4]
      klo    u32 [R][Wlo]           16 two-bit codes per word along channels; even codes fill the low half-word,
                                    odd codes the high one: code i in bits [16(i&1) + 2(i>>1), +2)
      k4     u32 [R][k4/8]          8 four-bit codes per word, code i in bits [16(i&1) + 4(i>>1), +4)
      k16    f16 [R][k16]           raw fp16 values of the fp16 tier
      v      u32 [R/16][D]          16 two-bit codes per word along TOKENS for one channel, same bit order as klo;
                                    code i of word tg belongs to token value_word_token(tg, i)
      v_s    f16 [R][D/Gv]          value scales per (token, channel group)
      v_z    f16 [R][D/Gv]
    """
    D, R = cfg.D, rec_tokens(cfg)
    NL = D if cfg.policy == 1 else D - cfg.ks     # threshold policy: room for every channel (tier sizes vary per block)
    Wlo = (NL + 15) // 16
    NLp = 16 * Wlo
    NG = R // cfg.Gk
    NVG = D // cfg.Gv
    W4 = cfg.k4 // 8
    off = 0
    offs = {}
    for name, size in (("idx", cfg.ks), ("kmax", (NG + 1) * 2), ("klo_s", NG * NLp * 2), ("klo_z", NG * NLp * 2),
                       ("k4_s", NG * cfg.k4 * 2), ("k4_z", NG * cfg.k4 * 2),
                       ("klo", R * Wlo * 4), ("k4", R * W4 * 4), ("k16", R * cfg.k16 * 2),
                       ("v", (R // 16) * D * 4), ("v_s", R * NVG * 2), ("v_z", R * NVG * 2)):
        offs["off_" + name] = off
        off += _al16(size)
    return BlockLayout(NL=NL, Wlo=Wlo, NLp=NLp, NG=NG, NVG=NVG, W4=W4, rec_bytes=off,
                       v_interleave=int(cfg.Gk == 32 and R % 64 == 0), **offs)


def value_word_token(tg: int, i: int, interleave: int) -> int:
    """Token (inside the block) of code i of value word tg.  Plain: the 16 consecutive tokens 16 tg + i.
    Interleaved (key groups of 32 tokens, R a multiple of 64): word j of a 64-token span holds the j-th 8 tokens
    of the span's first key group (codes 0..7) and the j-th 8 tokens of its second key group (codes 8..15), so
    that a reader that walks key group by key group consumes half a word per group."""
    if not interleave:
        return 16 * tg + i
    return 64 * (tg // 4) + 8 * (tg % 4) + (i % 8) + 32 * (i // 8)


@dataclasses.dataclass
class QuantBlock:
    """One flushed block of R tokens of one (batch, KV head) pair."""
    sel: np.ndarray        # u8 [ks]
    lo_codes: np.ndarray   # u8 [R, n_lo]   (n_lo = D - n16 - n4 channels at 2 bit)
    lo_s: np.ndarray       # f16 [NG, n_lo]
    lo_z: np.ndarray
    k4_codes: np.ndarray   # u8 [R, n4]     (n4 = k4, n16 = k16 under the top-k policy)
    k4_s: np.ndarray       # f16 [NG, n4]
    k4_z: np.ndarray
    k16: np.ndarray        # f16 [R, n16]
    v_codes: np.ndarray    # u8 [R, D]
    v_s: np.ndarray        # f16 [R, NVG]
    v_z: np.ndarray


def quantize_block(cfg: OracleConfig, K16: np.ndarray, V16: np.ndarray, sel: np.ndarray) -> QuantBlock:
    """The KeyQuant step of Appendix D.1 on one R-token block: split channels by
    tier, group-quantize each tier, keep the fp16 tier raw; per-token 2-bit values."""
    sel = np.asarray(sel, dtype=np.uint8)
    hi16, hi4 = tier_lists(sel, cfg.k16)
    lo = lo_channels(sel, cfg.D)
    lo_codes, lo_s, lo_z = quantize_keys(K16, lo, 2, cfg.Gk)
    k4_codes, k4_s, k4_z = quantize_keys(K16, hi4, 4, cfg.Gk)
    v_codes, v_s, v_z = quantize_values(V16, cfg.Gv)
    return QuantBlock(sel=sel, lo_codes=lo_codes, lo_s=lo_s, lo_z=lo_z, k4_codes=k4_codes, k4_s=k4_s,
                      k4_z=k4_z, k16=K16[:, hi16].copy(), v_codes=v_codes, v_s=v_s, v_z=v_z)


def _pack_along_last(codes: np.ndarray, bits: int) -> np.ndarray:
    """Pack codes [..., n] (n a multiple of 32/bits) into u32 [..., n*bits/32].
    Code i of a word goes to bits [16*(i&1) + bits*(i>>1), + bits): even codes in
    the low half-word, odd codes in the high half-word (an adjacent pair of
    codes then sits at the same position of the two halves)."""
    per = 32 // bits
    c = codes.astype(np.uint32).reshape(codes.shape[:-1] + (codes.shape[-1] // per, per))
    i = np.arange(per, dtype=np.uint32)
    shifts = np.uint32(16) * (i & 1) + np.uint32(bits) * (i >> 1)
    return np.bitwise_or.reduce(c << shifts, axis=-1).astype(np.uint32)


def sub_block(cfg: OracleConfig, blk: QuantBlock, j: int) -> QuantBlock:
    """Tokens [j * rec_tokens, (j + 1) * rec_tokens) of a block, with their groups."""
    Rr = rec_tokens(cfg)
    t = slice(j * Rr, (j + 1) * Rr)
    g = slice(j * Rr // cfg.Gk, (j + 1) * Rr // cfg.Gk)
    return QuantBlock(sel=blk.sel, lo_codes=blk.lo_codes[t], lo_s=blk.lo_s[g], lo_z=blk.lo_z[g], k4_codes=blk.k4_codes[t],
                      k4_s=blk.k4_s[g], k4_z=blk.k4_z[g], k16=blk.k16[t], v_codes=blk.v_codes[t], v_s=blk.v_s[t],
                      v_z=blk.v_z[t])


def pack_block(cfg: OracleConfig, blk: QuantBlock) -> np.ndarray:
    """Serialise one block into its records (uint8 [R / rec_tokens, rec_bytes])."""
    n_rec = cfg.R // rec_tokens(cfg)
    return np.stack([pack_record(cfg, sub_block(cfg, blk, j) if n_rec > 1 else blk) for j in range(n_rec)])


def pack_record(cfg: OracleConfig, blk: QuantBlock) -> np.ndarray:
    """Serialise rec_tokens tokens of a block into one record (uint8 [rec_bytes])."""
    lay = block_layout(cfg)
    rec = np.zeros(lay.rec_bytes, dtype=np.uint8)

    def put(off, arr):
        b = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
        rec[off:off + b.size] = b

    # Planes are sized for the capacity of each tier; entries past a tier's actual size are zero.
    put(lay.off_idx, blk.sel)
    allscales = np.concatenate([blk.lo_s, blk.k4_s], axis=1)          # [NG, n_lo + n4] fp16, all >= 0
    put(lay.off_kmax, np.concatenate([allscales.max(axis=1), [blk.v_s.max()]]).astype(np.float16))
    pad = lay.NLp - blk.lo_codes.shape[1]
    pad4 = cfg.k4 - blk.k4_codes.shape[1]
    pad16 = cfg.k16 - blk.k16.shape[1]
    s = np.pad(blk.lo_s, ((0, 0), (0, pad)))
    z = np.pad(blk.lo_z, ((0, 0), (0, pad)))
    put(lay.off_klo_s, s.astype(np.float16))
    put(lay.off_klo_z, z.astype(np.float16))
    put(lay.off_k4_s, np.pad(blk.k4_s, ((0, 0), (0, pad4))))
    put(lay.off_k4_z, np.pad(blk.k4_z, ((0, 0), (0, pad4))))
    put(lay.off_klo, _pack_along_last(np.pad(blk.lo_codes, ((0, 0), (0, pad))), 2))
    if cfg.k4:
        put(lay.off_k4, _pack_along_last(np.pad(blk.k4_codes, ((0, 0), (0, pad4))), 4))
    if cfg.k16:
        put(lay.off_k16, np.pad(blk.k16, ((0, 0), (0, pad16))))
    # values: 16 codes per word along tokens, one word per (token group, channel)
    tok = np.array([[value_word_token(tg, i, lay.v_interleave) for i in range(16)] for tg in range(rec_tokens(cfg) // 16)])
    vc = blk.v_codes[tok].transpose(0, 2, 1)                              # [tg, d, 16]
    put(lay.off_v, _pack_along_last(vc, 2))
    put(lay.off_v_s, blk.v_s)
    put(lay.off_v_z, blk.v_z)
    return rec


def dequant_block_keys(cfg: OracleConfig, blk: QuantBlock) -> np.ndarray:
    """K^ of one block in binary64, [R, D]: fp16 tier raw, other tiers by Eq. 3."""
    R, D, Gk = cfg.R, cfg.D, cfg.Gk
    out = np.empty((R, D), dtype=np.float64)
    hi16, hi4 = tier_lists(blk.sel, cfg.k16)
    lo = lo_channels(blk.sel, D)
    rep = lambda a: np.repeat(a, Gk, axis=0)
    out[:, lo] = decode(blk.lo_codes, rep(blk.lo_s), rep(blk.lo_z))
    if len(hi4):
        out[:, hi4] = decode(blk.k4_codes, rep(blk.k4_s), rep(blk.k4_z))
    if len(hi16):
        out[:, hi16] = blk.k16.astype(np.float64)
    return out


def dequant_block_values(cfg: OracleConfig, blk: QuantBlock) -> np.ndarray:
    rep = lambda a: np.repeat(a, cfg.Gv, axis=1)
    return decode(blk.v_codes, rep(blk.v_s), rep(blk.v_z))


# --------------------------------------------------------------------------
# cache state machine (Appendix D.1, D.2)
# --------------------------------------------------------------------------
class OracleCache:
    """All sequences of the batch advance in lock-step.  Per (b, KV head) pair:
    a list of quantized blocks, an fp16 residual window, an exact |q| sum."""

    def __init__(self, cfg: OracleConfig):
        assert cfg.Hq % cfg.Hkv == 0 and cfg.R % cfg.Gk == 0 and cfg.D % cfg.Gv == 0
        assert cfg.R % 16 == 0 and cfg.k4 % 8 == 0 and cfg.ks <= cfg.D and cfg.T_max % cfg.R == 0
        self.cfg = cfg
        P = cfg.B * cfg.Hkv
        self.blocks = [[] for _ in range(P)]                       # QuantBlock lists
        self.res_k = np.zeros((P, cfg.R, cfg.D), dtype=np.float16)
        self.res_v = np.zeros((P, cfg.R, cfg.D), dtype=np.float16)
        self.sink_k = np.zeros((P, cfg.sink, cfg.D), dtype=np.float16)
        self.sink_v = np.zeros((P, cfg.sink, cfg.D), dtype=np.float16)
        self.n_sink = 0
        self.n_res = 0
        self.n_quant = 0
        self.qacc = np.zeros((P, cfg.D), dtype=np.uint64)
        self.qcnt = np.zeros(P, dtype=np.uint64)
        self.n_flush_calls = 0

    # -- Eq. 6 accumulator -------------------------------------------------
    def accumulate_queries(self, Q16: np.ndarray):
        """Q16: [B, Hq, Lq, D] (or [B, Hq, D] for one decode step)."""
        cfg = self.cfg
        if Q16.ndim == 3:
            Q16 = Q16[:, :, None, :]
        B, Hq, Lq, D = Q16.shape
        Qg = Q16.reshape(B, cfg.Hkv, cfg.g, Lq, D)
        for b in range(B):
            for j in range(cfg.Hkv):
                p = b * cfg.Hkv + j
                self.qacc[p] += abs_query_sum(Qg[b, j])
                self.qcnt[p] += np.uint64(cfg.g * Lq)

    # -- selection ---------------------------------------------------------
    def select(self, K16: np.ndarray) -> np.ndarray:
        """Selection for keys K16 [B, Hkv, L, D] with the current accumulator.
        Returns u8 [B, Hkv, ks]."""
        cfg = self.cfg
        B, Hkv, L, D = K16.shape
        sel = np.zeros((B, Hkv, cfg.ks), dtype=np.uint8)
        for b in range(B):
            for j in range(Hkv):
                p = b * Hkv + j
                sel[b, j] = self.score_and_select(p, K16[b, j])
        return sel

    def score_and_select(self, p: int, Kb: np.ndarray) -> np.ndarray:
        """Channel tiers of pair p for the keys Kb [L, D]: Eq. 6-8 with the current
        accumulator, then the top-k budget or the thresholds of Section 4.2."""
        cfg = self.cfg
        A = salience(self.qacc[p], key_range(Kb), cfg.score_mode)
        if cfg.policy == 1:
            t16 = threshold_in_score_units(cfg.tau16, int(self.qcnt[p]), cfg.score_mode)
            t4 = threshold_in_score_units(cfg.tau4, int(self.qcnt[p]), cfg.score_mode)
            return select_channels_threshold(A, t16, t4, cfg.k16, cfg.k4)
        return select_channels(A, cfg.k16, cfg.k4)

    def select_channels(self, Q16, K16):
        """The library's select call: add the queries (if any) to the
        accumulator, then select for K16."""
        if Q16 is not None:
            self.accumulate_queries(Q16)
        return self.select(K16)

    # -- append / flush ----------------------------------------------------
    def flush_count(self, n_new: int) -> int:
        total = self.n_res + n_new
        R = self.cfg.R
        if self.cfg.flush_mode == 0:
            return max(0, -(-total // R) - 1)
        return total // R

    def append(self, k_new: np.ndarray, v_new: np.ndarray, sel: np.ndarray | None = None):
        """k_new, v_new: [B, Hkv, n, D] fp16.  Tokens enter the residual window one
        by one; in deferred mode a full window is flushed just before the next
        token enters, in eager mode as soon as it is full.  `sel` (u8
        [B, Hkv, ks]) fixes the channel choice of every block flushed by this
        call; with sel None each block is scored from the accumulator and its
        own R tokens."""
        cfg = self.cfg
        B, Hkv, n, D = k_new.shape
        R = cfg.R
        # the first cfg.sink tokens of the sequence go to the sink and never leave it
        take = min(n, cfg.sink - self.n_sink)
        F = self.flush_count(n - take)
        if self.n_quant + F * R > cfg.T_max:
            raise OverflowError("cache capacity exceeded")
        if take:
            for p in range(B * Hkv):
                self.sink_k[p, self.n_sink:self.n_sink + take] = k_new[p // Hkv, p % Hkv, :take]
                self.sink_v[p, self.n_sink:self.n_sink + take] = v_new[p // Hkv, p % Hkv, :take]
            self.n_sink += take
            k_new, v_new, n = k_new[:, :, take:], v_new[:, :, take:], n - take
            if n == 0:
                return
        for b in range(B):
            for j in range(Hkv):
                p = b * Hkv + j
                ks = np.concatenate([self.res_k[p, :self.n_res], k_new[b, j]], axis=0)
                vs = np.concatenate([self.res_v[p, :self.n_res], v_new[b, j]], axis=0)
                for f in range(F):
                    Kb = ks[f * R:(f + 1) * R]
                    Vb = vs[f * R:(f + 1) * R]
                    if sel is not None:
                        s = sel[b, j]
                    else:
                        s = self.score_and_select(p, Kb)
                    self.blocks[p].append(quantize_block(cfg, Kb, Vb, s))
                rest_k, rest_v = ks[F * R:], vs[F * R:]
                self.res_k[p, :len(rest_k)] = rest_k
                self.res_v[p, :len(rest_v)] = rest_v
        self.n_res = self.n_res + n - F * R
        self.n_quant += F * R
        self.n_flush_calls += F
        if F and cfg.qacc_reset_on_flush:
            self.qacc[:] = 0
            self.qcnt[:] = 0

    # -- bytes ---------------------------------------------------------------
    def packed_blocks(self) -> np.ndarray:
        """uint8 [P, n_records, rec_bytes]: the records of every flushed block, oldest first."""
        lay = block_layout(self.cfg)
        P = len(self.blocks)
        per = self.cfg.R // rec_tokens(self.cfg)
        nb = self.n_quant // self.cfg.R
        out = np.zeros((P, nb * per, lay.rec_bytes), dtype=np.uint8)
        for p in range(P):
            for i, blk in enumerate(self.blocks[p]):
                out[p, i * per:(i + 1) * per] = pack_block(self.cfg, blk)
        return out

    # -- Eq. 1 over the mixed-precision cache ----------------------------------
    def dequantized(self, p: int):
        """(K^, V^) in binary64 for pair p, [T, D] each: sink tokens as stored,
        quantized tokens by Eq. 3, residual tokens as stored."""
        cfg = self.cfg
        Ks = [self.sink_k[p, :self.n_sink].astype(np.float64)] + [dequant_block_keys(cfg, blk) for blk in self.blocks[p]]
        Vs = [self.sink_v[p, :self.n_sink].astype(np.float64)] + [dequant_block_values(cfg, blk) for blk in self.blocks[p]]
        Ks.append(self.res_k[p, :self.n_res].astype(np.float64))
        Vs.append(self.res_v[p, :self.n_res].astype(np.float64))
        return np.concatenate(Ks, axis=0), np.concatenate(Vs, axis=0)

    def decode_attention(self, q16: np.ndarray, scale: float | None = None, accumulate_q: bool = False):
        """q16: [B, Hq, D] fp16.  Returns (out [B, Hq, D], lse [B, Hq]) in binary64.
        Query head h attends through KV head h // g."""
        cfg = self.cfg
        B, Hq, D = q16.shape
        if scale is None or scale <= 0:
            scale = 1.0 / math.sqrt(D)
        if accumulate_q:
            self.accumulate_queries(q16)
        out = np.zeros((B, Hq, D), dtype=np.float64)
        lse = np.zeros((B, Hq), dtype=np.float64)
        for b in range(B):
            for j in range(cfg.Hkv):
                Kh, Vh = self.dequantized(b * cfg.Hkv + j)
                qs = q16[b, j * cfg.g:(j + 1) * cfg.g].astype(np.float64)      # [g, D]
                logits = (qs @ Kh.T) * scale                                   # [g, T]
                m = logits.max(axis=1, keepdims=True)
                e = np.exp(logits - m)
                l = e.sum(axis=1, keepdims=True)
                out[b, j * cfg.g:(j + 1) * cfg.g] = (e / l) @ Vh
                lse[b, j * cfg.g:(j + 1) * cfg.g] = (m + np.log(l))[:, 0]
        return out, lse


# --------------------------------------------------------------------------
# closed forms used for reporting
# --------------------------------------------------------------------------
def effective_key_bits(D: int, k16: int, k4: int) -> float:
    """B_eff of Appendix C: mean bit-width over the key channels."""
    return (16 * k16 + 4 * k4 + 2 * (D - k16 - k4)) / D


def algorithmic_bytes_per_pair(cfg: OracleConfig, n_q: int, r: int) -> int:
    """Bytes one decode step must move for one (batch, KV head) pair in the
    minimal representation of the method: packed codes, fp16 scale and
    zero-point per group, fp16-tier values, one index byte per salient channel
    and block, the fp16 residual window, and q in / out."""
    D, ks = cfg.D, cfg.ks
    nb = n_q // cfg.R
    ng = n_q // cfg.Gk
    b = n_q * (D - ks) // 4 + ng * (D - ks) * 4
    b += n_q * cfg.k4 // 2 + ng * cfg.k4 * 4
    b += n_q * cfg.k16 * 2
    b += nb * ks
    b += n_q * D // 4 + n_q * (D // cfg.Gv) * 4
    b += r * D * 4
    b += cfg.g * D * 4
    return b
