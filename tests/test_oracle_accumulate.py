"""Pins for the oracle's accumulation (Alg. 1/2 accumulation line + the DGC momentum
correction of Sec. V-A).  CPU only."""
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "accumulate_closed_form.txt")


def test_closed_form_golden(oracle):
    # m = 1/2, g = 2^-10: exact rational values from tests/golden (written without the oracle)
    rows = [l.split() for l in open(GOLD) if not l.startswith("#")]
    n = 37
    g = np.full(n, 2.0 ** -10, np.float32)
    u = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    for t, ub, vb in rows:
        oracle.accumulate(g, u, v, 0.5)
        assert (u.view(np.uint32) == int(ub, 16)).all(), t
        assert (v.view(np.uint32) == int(vb, 16)).all(), t


def test_zero_momentum_is_plain_residual_sum(oracle):
    # m = 0: v_t = v_{t-1} + g_t, the paper's g_l = grad + g_acc; small integers are exact
    rng = np.random.default_rng(1)
    n = 1000
    u = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    tot = np.zeros(n, np.int64)
    for _ in range(20):
        gi = rng.integers(-1000, 1000, n)
        oracle.accumulate(gi.astype(np.float32), u, v, 0.0)
        tot += gi
        assert (u == gi.astype(np.float32)).all()
        assert (v == tot.astype(np.float32)).all()


def _two_roundings(g, u, v, m):
    # independent route: fp64 holds the fp32 product exactly and the fp64 sum of two fp32
    # numbers rounds to fp32 like a direct fp32 sum (53 >= 2*24+2), so each step rounds once
    with np.errstate(over="ignore"):
        prod = (np.float64(np.float32(m)) * u.astype(np.float64)).astype(np.float32)
        un = (prod.astype(np.float64) + g.astype(np.float64)).astype(np.float32)
        vn = (v.astype(np.float64) + un.astype(np.float64)).astype(np.float32)
    return un, vn


def test_random_bitwise_vs_second_implementation(oracle):
    rng = np.random.default_rng(2)
    n = 50_000
    u = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    # denormals, zeros and huge values must pass through unchanged in kind
    u[:4] = [1e-42, -1e-45, 0.0, -0.0]
    v[:4] = [1e-40, 3e-39, -0.0, 1e38]
    for t in range(5):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        g[:4] = [1e-44, 1e-45, -0.0, 3e38]
        eu, ev = _two_roundings(g, u, v, 0.9)
        oracle.accumulate(g, u, v, 0.9)
        assert (u.view(np.uint32) == eu.view(np.uint32)).all()
        assert (v.view(np.uint32) == ev.view(np.uint32)).all()


def test_no_fused_multiply_add(oracle):
    # inputs where fl(m*u + g) with one rounding differs from fl(fl(m*u) + g):
    # the oracle must give the two-rounding value
    rng = np.random.default_rng(3)
    n = 200_000
    m = np.float32(0.9)
    u = rng.standard_normal(n).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    fused = (np.float64(m) * u.astype(np.float64) + g.astype(np.float64)).astype(np.float32)
    two, _ = _two_roundings(g, u, np.zeros(n, np.float32), m)
    differ = fused.view(np.uint32) != two.view(np.uint32)
    assert differ.sum() > 100  # the case exists in the sample
    uu, vv = u.copy(), np.zeros(n, np.float32)
    oracle.accumulate(g, uu, vv, float(m))
    assert (uu.view(np.uint32) == two.view(np.uint32)).all()
    assert (uu.view(np.uint32)[differ] != fused.view(np.uint32)[differ]).all()
