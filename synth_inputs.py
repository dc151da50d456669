"""Seeded synthetic inputs for the MixKVQ hot path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
bench.  It holds NO arithmetic of the method (no quantizer, no score, no
attention): only shapes and random tensors.

The tensors stand in for the paper's long chain-of-thought decoding workloads
(Section 5, "Experiments"), which need model weights and datasets that are not
available here.  Their structure follows what the paper reports about real
key/value/query activations:
  * a few key channels carry outliers of much larger magnitude than the rest
    (Section 4.1, "Key Cache is Generally More Important", Figure 2);
  * the value cache has no such channel structure (same passage);
  * query magnitude per channel is only weakly related to key scale
    (Section 4.1, Figure 3(a): Pearson coefficient 0.16), so the query outlier
    channels are drawn independently of the key outlier channels.
"""
from __future__ import annotations

import dataclasses
import numpy as np

SEED_BASE = 0x4D4B5651  # ASCII "MKVQ"


@dataclasses.dataclass(frozen=True)
class Workload:
    """Resolved shape of one benchmark configuration."""
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    T: int          # cached tokens at the timed decode step (prompt length)
    Gk: int         # key group size along tokens
    Gv: int         # value group size along channels
    R: int          # residual window length == flush unit
    k4: int         # salient key channels stored at 4 bit
    k16: int        # salient key channels stored as fp16
    steps: int = 1  # consecutive decode steps the configuration times

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv


WORKLOADS = {
    0: Workload("cfg0_1head_1k", B=1, Hq=1, Hkv=1, D=128, T=1024, Gk=32, Gv=32, R=32, k4=8, k16=0),
    1: Workload("cfg1_gqa7b_b8_32k", B=8, Hq=28, Hkv=4, D=128, T=32768, Gk=128, Gv=128, R=128, k4=16, k16=0),
    2: Workload("cfg2_gqa32b_b64_32k", B=64, Hq=40, Hkv=8, D=128, T=32768, Gk=128, Gv=128, R=128, k4=0, k16=12),
    3: Workload("cfg3_longcot_b4_128k", B=4, Hq=40, Hkv=8, D=128, T=131072, Gk=128, Gv=128, R=128, k4=16, k16=0,
                steps=512),
    4: Workload("cfg4_prefill_b16_32k", B=16, Hq=40, Hkv=8, D=128, T=32768, Gk=128, Gv=128, R=128, k4=16, k16=0),
}


def _rng(cfg_id: int, stream: int) -> np.random.Generator:
    root = np.random.SeedSequence(SEED_BASE + cfg_id)
    return np.random.Generator(np.random.PCG64(root.spawn(stream + 1)[stream]))


def cfg0_tensors(T: int = 1024, D: int = 128, Lq: int = 1024):
    """Single head, batch 1: K, V, q ~ N(0,1) in fp16; four fixed key channels
    scaled by 15.  Returns K[1,1,T,D], V[1,1,T,D], Qprompt[1,1,Lq,D], q[1,1,D]."""
    rk, rv, rq, rd = (_rng(0, i) for i in range(4))
    K = rk.standard_normal((1, 1, T, D), dtype=np.float32)
    K[..., [5, 37, 70, 101]] *= 15.0
    V = rv.standard_normal((1, 1, T, D), dtype=np.float32)
    Qp = rq.standard_normal((1, 1, Lq, D), dtype=np.float32)
    q = rd.standard_normal((1, 1, D), dtype=np.float32)
    return K.astype(np.float16), V.astype(np.float16), Qp.astype(np.float16), q.astype(np.float16)


def _student_t3_magnitude(rng: np.random.Generator, shape) -> np.ndarray:
    """|t| with 3 degrees of freedom, normalised to unit mean (E|t_3| = 1.1027)."""
    return (np.abs(rng.standard_t(3.0, size=shape)) / 1.1027).astype(np.float32)


def heavy_tailed_kv(cfg_id: int, B: int, Hkv: int, T: int, D: int = 128, n_outlier: int = 4):
    """Keys with outlier channels and heavy-tailed per-token magnitudes, values
    with heavy-tailed per-token magnitudes only.  Returns fp16 K, V of shape
    [B, Hkv, T, D] and the key outlier channel ids [B, Hkv, n_outlier]."""
    rk, rv, _, ro = (_rng(cfg_id, i) for i in range(4))
    K = np.empty((B, Hkv, T, D), dtype=np.float16)
    V = np.empty((B, Hkv, T, D), dtype=np.float16)
    out_ids = np.empty((B, Hkv, n_outlier), dtype=np.int64)
    for b in range(B):
        for h in range(Hkv):
            c = np.ones(D, dtype=np.float32)
            ids = ro.choice(D, size=n_outlier, replace=False)
            c[ids] = ro.uniform(10.0, 20.0, size=n_outlier).astype(np.float32)
            out_ids[b, h] = np.sort(ids)
            m = _student_t3_magnitude(rk, (T, 1))
            eps = rk.standard_normal((T, D), dtype=np.float32)
            K[b, h] = np.clip(eps * m * c, -32768.0, 32768.0).astype(np.float16)
            mv = _student_t3_magnitude(rv, (T, 1))
            epsv = rv.standard_normal((T, D), dtype=np.float32)
            V[b, h] = np.clip(epsv * mv, -32768.0, 32768.0).astype(np.float16)
    return K, V, out_ids


def outlier_queries(cfg_id: int, B: int, Hq: int, L: int, D: int = 128, n_outlier: int = 4,
                    stream: int = 2) -> np.ndarray:
    """Queries [B, Hq, L, D] fp16 ~ a_d * N(0,1); each query head has its own,
    independently drawn outlier channels (a_d ~ U(10,20) on 4 channels)."""
    rq = _rng(cfg_id, stream)
    Q = np.empty((B, Hq, L, D), dtype=np.float16)
    for b in range(B):
        for h in range(Hq):
            a = np.ones(D, dtype=np.float32)
            ids = rq.choice(D, size=n_outlier, replace=False)
            a[ids] = rq.uniform(10.0, 20.0, size=n_outlier).astype(np.float32)
            Q[b, h] = (rq.standard_normal((L, D), dtype=np.float32) * a).astype(np.float16)
    return Q


def scaled_workload(cfg_id: int, B: int | None = None, T: int | None = None, Hq: int | None = None,
                    Hkv: int | None = None) -> Workload:
    """A configuration with some dimensions overridden (parity slices of the
    full-size configurations)."""
    w = WORKLOADS[cfg_id]
    kw = {}
    if B is not None:
        kw["B"] = B
    if T is not None:
        kw["T"] = T
    if Hq is not None:
        kw["Hq"] = Hq
    if Hkv is not None:
        kw["Hkv"] = Hkv
    return dataclasses.replace(w, **kw)
