"""Pins for the oracle's exact top-k with residual update (Alg. 1/2: threshold, mask, g~,
residual; Sec. V-A: exactly mu values per vector).  CPU only."""
import numpy as np
import pytest


def key(x):
    return x.view(np.uint32) & np.uint32(0x7FFFFFFF)


def brute_force(v, k):
    """k rounds of arg-max over the magnitude keys; np.argmax returns the lowest index among
    equal maxima, which is the tie rule."""
    kk = key(v).astype(np.int64)
    sel = []
    for _ in range(k):
        i = int(np.argmax(kk))
        sel.append(i)
        kk[i] = -1
    return np.array(sorted(sel), dtype=np.uint32)


def check_invariants(v0, u0, v1, u1, vals, idx, k):
    n = v0.size
    assert idx.size == k and vals.size == k
    assert (np.diff(idx.astype(np.int64)) > 0).all()          # strictly ascending => distinct
    assert (idx < n).all() if k else True
    sel = np.zeros(n, bool)
    sel[idx] = True
    # partition, bit for bit: selected -> value sent and residual +0; unselected -> untouched
    assert (vals.view(np.uint32) == v0[idx].view(np.uint32)).all()
    assert (v1[sel].view(np.uint32) == 0).all()
    assert (v1[~sel].view(np.uint32) == v0[~sel].view(np.uint32)).all()
    if u0 is not None:
        assert (u1[sel].view(np.uint32) == 0).all()
        assert (u1[~sel].view(np.uint32) == u0[~sel].view(np.uint32)).all()
    if 0 < k < n:
        ks, kc = key(v0)[sel], key(v0)[~sel]
        thr = ks.min()
        assert thr >= kc.max()
        tied_sel = np.nonzero(sel & (key(v0) == thr))[0]
        tied_uns = np.nonzero(~sel & (key(v0) == thr))[0]
        if tied_uns.size:
            assert tied_sel.max() < tied_uns.min()             # lower index wins a tie


def run(oracle, v0, k, with_u=True):
    rng = np.random.default_rng(k + v0.size)
    u0 = rng.standard_normal(v0.size).astype(np.float32) if with_u else None
    v1 = v0.copy()
    u1 = u0.copy() if with_u else None
    vals, idx = oracle.topk(v1, u1, k)
    check_invariants(v0, u0, v1, u1, vals, idx, k)
    return vals, idx, v1


@pytest.mark.parametrize("n", [1, 2, 7, 64, 1000, 4096])
def test_brute_force_small(oracle, n):
    rng = np.random.default_rng(n)
    # few distinct magnitudes => many ties, mixed signs
    v0 = (rng.integers(-6, 7, n)).astype(np.float32) * np.float32(0.25)
    ks = sorted({0, 1, 2, n // 3, n - 1, n} & set(range(n + 1)))
    for k in ks:
        _, idx, _ = run(oracle, v0, k, with_u=(k % 2 == 0))
        assert (idx == brute_force(v0, k)).all(), (n, k)
    v0 = rng.standard_normal(n).astype(np.float32)
    for k in ks:
        _, idx, _ = run(oracle, v0, k)
        assert (idx == brute_force(v0, k)).all(), (n, k)


def test_signed_permutation_known_answer(oracle):
    n, k = 5000, 137
    rng = np.random.default_rng(5)
    perm = rng.permutation(n) + 1                      # magnitudes 1..n, all distinct
    v0 = (perm * rng.choice([-1, 1], n)).astype(np.float32)
    vals, idx, _ = run(oracle, v0, k)
    assert (idx == np.sort(np.nonzero(perm > n - k)[0])).all()
    assert set(np.abs(vals).astype(int)) == set(range(n - k + 1, n + 1))


def test_all_equal_magnitudes_take_lowest_indices(oracle):
    n, k = 3000, 777
    v0 = np.full(n, 0.125, np.float32)
    v0[::3] *= -1
    _, idx, _ = run(oracle, v0, k)
    assert (idx == np.arange(k)).all()


def test_duplicates_straddling_the_cut(oracle):
    # 10 values above the threshold value, t = 50 copies of it, of which r = 7 must be taken
    n = 2000
    rng = np.random.default_rng(9)
    v0 = (rng.random(n) * 0.5).astype(np.float32)
    big = rng.choice(n, 60, replace=False)
    v0[big[:10]] = 2.0 + rng.random(10).astype(np.float32)
    tied = np.sort(big[10:])
    v0[tied] = 1.0
    v0[tied[::2]] = -1.0
    _, idx, _ = run(oracle, v0, 17)
    assert (idx == np.sort(np.concatenate([big[:10], tied[:7]]))).all()


def test_special_values(oracle):
    # +-0 only: all keys equal -> first k indices; values keep their sign bit
    v0 = np.array([0.0, -0.0, -0.0, 0.0, -0.0], np.float32)
    vals, idx, v1 = run(oracle, v0, 3)
    assert (idx == [0, 1, 2]).all()
    assert (vals.view(np.uint32) == v0[:3].view(np.uint32)).all()
    # denormals order by magnitude
    v0 = np.array([1e-45, -3e-45, 2e-45, 0.0, 1e-44], np.float32)
    _, idx, _ = run(oracle, v0, 2)
    assert (idx == [1, 4]).all()
    # NaN has the largest key, then Inf
    v0 = np.array([1.0, np.inf, -5.0, np.nan, 3.0], np.float32)
    vals, idx, _ = run(oracle, v0, 2)
    assert (idx == [1, 3]).all() and np.isnan(vals[1]) and np.isinf(vals[0])


def test_no_ties_equals_threshold_mask(oracle):
    # Alg. 1/2 as printed: threshold = min(top-k |g|), mask = |g| >= threshold
    rng = np.random.default_rng(11)
    v0 = np.unique(rng.standard_normal(40_000).astype(np.float32))
    v0 = v0[np.unique(np.abs(v0), return_index=True)[1]]       # distinct magnitudes
    rng.shuffle(v0)
    k = v0.size // 1000 * 7 + 3
    vals, idx, v1 = run(oracle, v0, k)
    thr = np.sort(np.abs(v0))[-k]
    mask = np.abs(v0) >= thr
    assert mask.sum() == k
    assert (np.nonzero(mask)[0] == idx).all()
    assert (v1 == np.where(mask, 0, v0)).all() and (vals == v0[mask]).all()


def test_large_random_against_partition(oracle):
    # n big enough for the benchmark's shapes in miniature; np.partition is a different routine
    rng = np.random.default_rng(13)
    n, k = 1_000_003, 1000
    v0 = (rng.laplace(0, 1e-3, n)).astype(np.float32)
    vals, idx, _ = run(oracle, v0, k)
    kth = np.partition(key(v0), n - k)[n - k]
    assert key(vals).min() == kth
    assert (key(v0) > kth).sum() <= k <= (key(v0) >= kth).sum()


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.topk(np.zeros(4, np.float32), None, 5)
