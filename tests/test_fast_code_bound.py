"""Host-side check of the error analysis behind the quantize-and-pack kernel's shortcut for Eq. 2.

The kernel forms q0 = x * r + nz (one fused multiply-add; r = rcp(s) good to one ulp, nz = fl(-z * r)) and takes
rint(q0) as the code whenever q0 is further than EPS from every half-integer, provided the stored scale is a normal
binary16 and |z r| <= 32; all other codes are redone with the division.  This test replays that arithmetic in numpy
(with the reciprocal pushed one ulp either way) on random and adversarial groups and checks, against the oracle's
Eq. 2, that every code the shortcut would keep is the right one and that |q0 - q| stays inside the bound the kernel's
comment states.  It pins the analysis, not the kernel: the kernel itself is compared bit for bit on the GPU."""
import numpy as np
import pytest

from oracle import mixkvq_oracle as O

EPS = {2: 2.0 ** -18, 4: 2.0 ** -16}
BOUND = {2: 2.9e-6, 4: 6.5e-6}
MAX_ZR = 32.0
MIN_NORMAL_F16 = 2.0 ** -14


def _groups(rng, n_groups, n, bits):
    """fp16 groups [n_groups, n] with a spread of offsets, scales and tie-prone integer grids."""
    top = (1 << bits) - 1
    kind = rng.integers(0, 4, n_groups)
    scale = 2.0 ** rng.uniform(-10, 8, (n_groups, 1))
    offs = rng.uniform(-10, 10, (n_groups, 1)) * scale
    X = rng.standard_normal((n_groups, n)) * scale + offs
    # integer grids: range = top * step makes every quotient an exact multiple of 1/2 or 1/4
    step = 2.0 ** rng.integers(-6, 6, (n_groups, 1))
    grid = (rng.integers(0, 2 * top + 1, (n_groups, n)) * 0.5 + rng.integers(-8, 9, (n_groups, 1)) * top) * step
    grid[:, 0] = grid.min(1)
    grid[:, 1] = grid[:, 0] + (top * step)[:, 0]
    grid = np.minimum(grid, grid[:, 1:2])
    X = np.where((kind == 0)[:, None], grid, X)
    # heavy tail: one large element stretches the scale
    X[kind == 1, 2] *= 30.0
    return np.clip(X, -60000.0, 60000.0).astype(np.float16)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("ulp_shift", [-1, 0, 1])
def test_shortcut_codes_equal_eq2_wherever_the_kernel_keeps_them(bits, ulp_shift):
    rng = np.random.default_rng(100 + 10 * bits + ulp_shift)
    X = _groups(rng, 6000, 64, bits)
    s16, z16 = O.group_params(X, bits, axis=1)
    ref = O.encode(X, s16[:, None], z16[:, None], bits)
    s = s16.astype(np.float32)
    z = z16.astype(np.float32)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        r = np.where(s > 0, np.float32(1.0) / np.where(s > 0, s, np.float32(1.0)), np.float32(0.0)).astype(np.float32)
        if ulp_shift:
            r = np.where(s > 0, np.nextafter(r, np.float32(np.inf if ulp_shift > 0 else 0.0)), r).astype(np.float32)
        nz = (-z * r).astype(np.float32)
    fast = (s >= MIN_NORMAL_F16) & (np.abs(nz) <= MAX_ZR)       # the groups the shortcut serves
    assert fast.sum() > 3000
    q0 = (X.astype(np.longdouble) * r[:, None].astype(np.longdouble) + nz[:, None].astype(np.longdouble)).astype(np.float32)
    c = np.rint(q0)
    dev = np.abs(q0 - c)
    keep = fast[:, None] & (dev <= np.float32(0.5) - np.float32(EPS[bits]))
    assert keep.mean() > 0.5
    assert np.array_equal(c[keep].astype(np.int64), ref[keep].astype(np.int64))
    # no kept code needs a clamp
    assert c[keep].min() >= 0 and c[keep].max() <= (1 << bits) - 1
    # the distance to Eq. 2's own quotient is inside the stated bound
    q = ((X.astype(np.float32) - z[:, None]) / np.where(s > 0, s, np.float32(1.0))[:, None]).astype(np.float32)
    err = np.abs(q0.astype(np.float64) - q.astype(np.float64))[fast]
    assert err.max() <= BOUND[bits], err.max()
    assert BOUND[bits] < EPS[bits]


def test_ties_are_common_in_fp16_data():
    """Exact ties (x - z)/s = k + 1/2 are what the correction pass is for: on gaussian fp16 data they are roughly
    1e-4 of all codes, far more than the width of the EPS band alone would give."""
    rng = np.random.default_rng(7)
    X = rng.standard_normal((4096, 128)).astype(np.float16)
    s16, z16 = O.group_params(X, 2, axis=1)
    q = (X.astype(np.float64) - z16.astype(np.float64)[:, None]) / s16.astype(np.float64)[:, None]
    ties = np.abs(np.abs(q - np.rint(q)) - 0.5) < 1e-12
    assert 1e-5 < ties.mean() < 1e-3
