"""Helpers for the GPU parity tests: build the oracle cache and the library's
cache from the same seeded fp16 inputs and compare them."""
import numpy as np
import torch

import paper_2512_19206_amd as M
from oracle import mixkvq_oracle as O

ATOL, RTOL = 2e-3, 1e-2   # |gpu - oracle| <= ATOL + RTOL * |oracle| on attention outputs (fp32 accumulate vs fp64)
LSE_ATOL = 2e-3


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_pair(**kw):
    """(oracle cache, library cache) for one configuration."""
    return O.OracleCache(O.OracleConfig(**kw)), M.Cache(M.make_config(**kw))


def check_state(oc: O.OracleCache, gc: M.Cache, check_qacc=True):
    """Bit-exact comparison of everything the cache stores."""
    torch.cuda.synchronize()
    nq, r = gc.state()
    assert (nq, r) == (oc.n_quant, oc.n_res)
    nb = nq // O.rec_tokens(oc.cfg)      # records
    if nb:
        got = gc.block_records()[:, :nb].cpu().numpy()
        ref = oc.packed_blocks()
        if not np.array_equal(got, ref):
            lay = O.block_layout(oc.cfg)
            bad = np.argwhere(got != ref)
            p, b, off = bad[0]
            planes = [(n, getattr(lay, n)) for n in dir(lay) if n.startswith("off_")]
            plane = max((o, n) for n, o in planes if o <= off)[1]
            raise AssertionError(f"{len(bad)} record bytes differ; first at pair {p} block {b} byte {off} ({plane}): "
                                 f"gpu {got[p, b, off]} oracle {ref[p, b, off]}")
    ns = gc.sink_count()
    assert ns == oc.n_sink
    if ns:
        sk, sv = gc.sink()
        assert np.array_equal(sk[:, :ns].cpu().numpy().view(np.uint16), oc.sink_k[:, :ns].view(np.uint16))
        assert np.array_equal(sv[:, :ns].cpu().numpy().view(np.uint16), oc.sink_v[:, :ns].view(np.uint16))
    if r:
        rk, rv = gc.residual()
        assert np.array_equal(rk[:, :r].cpu().numpy().view(np.uint16), oc.res_k[:, :r].view(np.uint16))
        assert np.array_equal(rv[:, :r].cpu().numpy().view(np.uint16), oc.res_v[:, :r].view(np.uint16))
    if check_qacc:
        acc, cnt = gc.query_accumulator()
        assert np.array_equal(acc.cpu().numpy().astype(np.uint64), oc.qacc)
        assert np.array_equal(cnt.cpu().numpy().astype(np.uint64), oc.qcnt)


def check_attention(oc: O.OracleCache, gc: M.Cache, q16: np.ndarray, accumulate_q=False, scale=0.0, atol=ATOL):
    """atol: the absolute term of the bar; ATOL unless the cache holds values beyond 512 (see value_atol)."""
    out, lse = gc.decode_attention(dev(q16), scale=scale, accumulate_q=accumulate_q)
    torch.cuda.synchronize()
    ro, rl = oc.decode_attention(q16, scale=scale if scale > 0 else None, accumulate_q=accumulate_q)
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    err = np.abs(go - ro)
    tol = atol + RTOL * np.abs(ro)
    assert np.all(err <= tol), f"attention out of tolerance: max excess {(err - tol).max():.3e}, max abs err {err.max():.3e}"
    assert np.all(np.abs(gl - rl) <= LSE_ATOL + 1e-4 * np.abs(rl)), f"lse max err {np.abs(gl - rl).max():.3e}"
    return float(err.max()), float(np.linalg.norm(go - ro) / max(np.linalg.norm(ro), 1e-30))


def value_atol(max_abs_value: float) -> float:
    """Absolute term of the attention bar for a cache whose dequantized values reach max_abs_value.  The kernel
    accumulates sum (p s) c and sum p z of Eq. 3 in binary32 and adds them at the end; where a value group has |z| far
    above its dequantized values the two sums cancel, and what remains carries the rounding of binary32 sums of
    magnitude |z| (2^-24 each, a few dozen roundings per wavefront).  The documented bar: ATOL up to |value| = 512,
    2^-18 of the largest magnitude beyond."""
    return max(ATOL, float(max_abs_value) * 2.0 ** -18)
