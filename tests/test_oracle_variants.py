"""Pins for the oracle's per-layer selection (Sec. V-A, layer loop of Alg. 1 / Alg. 2), the
ring-allreduce helpers (Sec. V-A: shared positions; Alg. 2: average of the compressed
representations) and the innovation component (Alg. 1, Sec. IV-C).  CPU only.  Everything is
checked against something other than the oracle's own code: known answers, brute force written
with different primitives, invariants, and the special cases that reduce to the flat selection."""
import numpy as np
import pytest

from test_oracle_topk import brute_force, check_invariants, key


def random_layout(rng, n, n_seg):
    cuts = np.sort(rng.choice(np.arange(1, n), n_seg - 1, replace=False)) if n_seg > 1 else np.array([], int)
    return np.concatenate([[0], cuts, [n]]).astype(np.uint64)


# ------------------------------------------------------------------ per-layer top-k

def test_segmented_known_answer_scales(oracle):
    # three layers whose magnitudes differ by orders of magnitude: a flat top-k would take
    # everything from the last layer; per-layer selection takes the largest of EACH layer
    n_l, k_l = 100, 3
    rng = np.random.default_rng(0)
    v, expect = [], []
    for l, scale in enumerate([1e-6, 1e-3, 1.0]):
        perm = rng.permutation(n_l) + 1                       # magnitudes 1..n_l, each once
        sign = rng.choice([-1.0, 1.0], n_l)
        v.append((perm * sign * scale).astype(np.float32))
        expect.append(np.sort(np.nonzero(perm > n_l - k_l)[0]) + l * n_l)
    v = np.concatenate(v)
    v0 = v.copy()
    vals, idx = oracle.topk_segmented(v, None, [0, 100, 200, 300], [k_l] * 3)
    assert (idx == np.concatenate(expect)).all()
    assert (vals.view(np.uint32) == v0[idx].view(np.uint32)).all()
    assert (v[idx] == 0).all() and np.count_nonzero(v) == 300 - 9
    # the flat selection of 9 differs: all from the last layer
    _, flat = oracle.topk(v0.copy(), None, 9)
    assert (flat >= 200).all()


@pytest.mark.parametrize("n,n_seg", [(50, 1), (64, 5), (1000, 17), (4096, 40)])
def test_segmented_brute_force_and_invariants(oracle, n, n_seg):
    rng = np.random.default_rng(n + n_seg)
    off = random_layout(rng, n, n_seg)
    lens = np.diff(off).astype(int)
    ks = np.array([rng.integers(0, m + 1) for m in lens], dtype=np.uint64)
    ks[0] = min(1, lens[0]); ks[-1] = lens[-1]                # k_l = 1 and k_l = n_l both occur
    v0 = (rng.integers(-6, 7, n) * 0.25).astype(np.float32)   # few magnitudes: ties in every layer
    u0 = rng.standard_normal(n).astype(np.float32)
    v1, u1 = v0.copy(), u0.copy()
    vals, idx = oracle.topk_segmented(v1, u1, off, ks)
    assert idx.size == int(ks.sum())
    assert (np.diff(idx.astype(np.int64)) > 0).all()
    o = 0
    for l in range(n_seg):
        lo, hi, k = int(off[l]), int(off[l + 1]), int(ks[l])
        seg_idx = idx[o:o + k]
        assert ((seg_idx >= lo) & (seg_idx < hi)).all()       # exactly k_l from layer l
        assert (seg_idx - lo == brute_force(v0[lo:hi], k)).all()
        check_invariants(v0[lo:hi], u0[lo:hi], v1[lo:hi], u1[lo:hi], vals[o:o + k],
                         (seg_idx - lo).astype(np.uint32), k)
        o += k


def test_segmented_one_layer_is_the_flat_selection(oracle):
    rng = np.random.default_rng(5)
    v = rng.standard_normal(3000).astype(np.float32)
    a, b = v.copy(), v.copy()
    vals_s, idx_s = oracle.topk_segmented(a, None, [0, 3000], [77])
    vals_f, idx_f = oracle.topk(b, None, 77)
    assert (idx_s == idx_f).all() and (vals_s.view(np.uint32) == vals_f.view(np.uint32)).all()
    assert (a.view(np.uint32) == b.view(np.uint32)).all()


def test_segmented_every_element_its_own_layer(oracle):
    # n layers of one element with k_l = 1: everything is sent, in order
    v = np.arange(1, 21, dtype=np.float32) * np.float32(-0.5)
    v0 = v.copy()
    vals, idx = oracle.topk_segmented(v, None, np.arange(21), np.ones(20))
    assert (idx == np.arange(20)).all() and (vals == v0).all() and not v.any()


def test_segmented_rejects_bad_layouts(oracle):
    v = np.ones(10, np.float32)
    with pytest.raises(ValueError):
        oracle.topk_segmented(v, None, [0, 5, 9], [1, 1])     # does not cover the vector
    with pytest.raises(ValueError):
        oracle.topk_segmented(v, None, [0, 5, 10], [6, 1])    # k_l > n_l


# ------------------------------------------------------------------ shared positions (ring-allreduce)

def test_gather_takes_values_and_clears_state(oracle):
    rng = np.random.default_rng(1)
    n = 500
    v0 = rng.standard_normal(n).astype(np.float32)
    u0 = rng.standard_normal(n).astype(np.float32)
    idx = np.sort(rng.choice(n, 60, replace=False)).astype(np.uint32)
    v, u = v0.copy(), u0.copy()
    vals = oracle.gather(v, u, idx)
    assert (vals.view(np.uint32) == v0[idx].view(np.uint32)).all()
    rest = np.ones(n, bool); rest[idx] = False
    assert (v[idx].view(np.uint32) == 0).all() and (u[idx].view(np.uint32) == 0).all()
    assert (v[rest] == v0[rest]).all() and (u[rest] == u0[rest]).all()
    # what is sent plus what is kept is the accumulated gradient, position by position
    back = v.copy(); back[idx] = vals
    assert (back.view(np.uint32) == v0.view(np.uint32)).all()


def test_gather_at_own_topk_positions_equals_topk(oracle):
    # a node that "gathers" at the positions its own selection would pick ends in the same state
    rng = np.random.default_rng(2)
    v0 = rng.laplace(0, 1, 2000).astype(np.float32)
    u0 = rng.standard_normal(2000).astype(np.float32)
    a_v, a_u = v0.copy(), u0.copy()
    vals_t, idx_t = oracle.topk(a_v, a_u, 40)
    b_v, b_u = v0.copy(), u0.copy()
    vals_g = oracle.gather(b_v, b_u, idx_t)
    assert (vals_g.view(np.uint32) == vals_t.view(np.uint32)).all()
    assert (a_v.view(np.uint32) == b_v.view(np.uint32)).all() and (a_u.view(np.uint32) == b_u.view(np.uint32)).all()


def test_gather_rejects_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.gather(np.zeros(4, np.float32), None, np.array([1, 4], np.uint32))


def test_average_exact_cases(oracle):
    rng = np.random.default_rng(3)
    x = rng.integers(-1000, 1000, (1, 64)).astype(np.float32)
    # K equal copies, K a power of two: the average is the copy itself, bit for bit
    for K in (1, 2, 4, 8):
        out = oracle.average(np.repeat(x, K, axis=0), 1.0 / K)
        assert (out.view(np.uint32) == x[0].view(np.uint32)).all()
    # small integers, scale 1: the plain integer sum
    y = rng.integers(-50, 50, (5, 33)).astype(np.float32)
    assert (oracle.average(y, 1.0) == y.astype(np.int64).sum(axis=0)).all()


def test_average_rounds_each_step_in_node_order(oracle):
    # fp32: (1 + 2^-24) rounds to 1, so adding 2^-24 twice to 1 gives 1, while 2^-24 + 2^-24 + 1
    # gives 1 + 2^-23: the result depends on the order, and the order is the node order
    t = np.float32(2.0 ** -24)
    a = oracle.average(np.array([[1.0], [t], [t]], np.float32), 1.0)
    b = oracle.average(np.array([[t], [t], [1.0]], np.float32), 1.0)
    assert a[0] == np.float32(1.0) and b[0] == np.float32(1.0) + np.float32(2.0 ** -23)
    # the product is rounded before the sum: 3 * (1/3 rounded) is not 1 in one fused step
    third = np.float32(1.0 / 3.0)
    s = np.float32(np.float32(third * np.float32(3.0)))
    assert oracle.average(np.array([[3.0]], np.float32), third)[0] == s


# ------------------------------------------------------------------ innovation component

def test_innovation_known_answer(oracle):
    vals = np.array([0.5, -4.0, 3.0, -0.25, 4.0, 1.0, -6.0, 2.0], np.float32)
    out = oracle.innovation(vals, [0, 8], [3])
    # top three magnitudes: 6, then the two 4s (both fit)
    assert (out == np.array([0, -4.0, 0, 0, 4.0, 0, -6.0, 0], np.float32)).all()
    out = oracle.innovation(vals, [0, 8], [2])
    # cut inside the tie: the lower position wins
    assert (out == np.array([0, -4.0, 0, 0, 0, 0, -6.0, 0], np.float32)).all()
    # per layer: two layers of four, one value each
    out = oracle.innovation(vals, [0, 4, 8], [1, 1])
    assert (out == np.array([0, -4.0, 0, 0, 0, 0, -6.0, 0], np.float32)).all()
    assert (vals == np.array([0.5, -4.0, 3.0, -0.25, 4.0, 1.0, -6.0, 2.0], np.float32)).all()   # input untouched


@pytest.mark.parametrize("k,n_seg", [(40, 1), (300, 7), (2048, 30)])
def test_innovation_is_the_selection_written_in_place(oracle, k, n_seg):
    rng = np.random.default_rng(k)
    off = random_layout(rng, k, n_seg)
    lens = np.diff(off).astype(int)
    ks = np.maximum(1, lens // 10).astype(np.uint64)           # "top 10 %" of Alg. 1
    vals = (rng.integers(-9, 10, k) * 0.5).astype(np.float32)
    out = oracle.innovation(vals, off, ks)
    for l in range(n_seg):
        lo, hi = int(off[l]), int(off[l + 1])
        keep = brute_force(vals[lo:hi], int(ks[l]))
        expect = np.zeros(hi - lo, np.float32)
        expect[keep] = vals[lo:hi][keep]
        assert (out[lo:hi].view(np.uint32) == expect.view(np.uint32)).all()
    # invariants: kept entries equal the input, the rest is +0, exactly sum(ks) kept when no zeros are kept
    kept = out.view(np.uint32) != 0
    assert (out[kept] == vals[kept]).all()
    assert kept.sum() <= int(ks.sum())


def test_decoder_with_innovation_channel(oracle):
    # delta weights: the last layer passes the innovation channel through, the rest is ignored
    from paper_2103_08870_amd import synth
    k = 37
    enc = [(1, 4, 3, 2), (4, 2, 3, 2)]
    dec = [(2, 4, 3, 2), (4, 3, 3, 2), (4, 1, 1, 1)]           # last: 3 + 1 innovation channel -> 1
    rng = np.random.default_rng(0)
    w = [rng.standard_normal((ci, co, ks)).astype(np.float32) for ci, co, ks, _ in dec]
    b = [rng.standard_normal(co).astype(np.float32) for _, co, _, _ in dec]
    lat_len = oracle.encoder_lengths(k, enc)[-1]
    latent = rng.standard_normal((2, lat_len)).astype(np.float32)
    innov = rng.standard_normal(k).astype(np.float32)
    w[-1][:] = 0; w[-1][3, 0, 0] = 1.0; b[-1][:] = 0
    out = oracle.decode_with_innovation(latent, innov, k, enc, dec, w, b)
    assert (out == innov).all()
    # general weights: equals the plain decoder of the first layers followed by an explicit
    # weighted sum of its channels and the innovation
    w[-1] = rng.standard_normal((4, 1, 1)).astype(np.float32)
    b[-1] = rng.standard_normal(1).astype(np.float32)
    out = oracle.decode_with_innovation(latent, innov, k, enc, dec, w, b)
    x = latent
    lens = oracle.decoder_lengths(k, enc, dec)
    for (ci, co, ks, st), wl, bl, lo in zip(dec[:-1], w[:-1], b[:-1], lens[:-1]):
        x = oracle.conv_transpose1d(x, wl, bl, ks, st, lo, True)
    ref = b[-1][0] + (w[-1][:3, 0, 0].astype(np.float64)[:, None] * x).sum(axis=0) + float(w[-1][3, 0, 0]) * innov
    assert np.allclose(out, ref, rtol=1e-6, atol=1e-6)
