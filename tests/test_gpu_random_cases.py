"""GPU parity on seeded random cases: shapes, batch sizes, paddings, base alignments, value distributions and
layer stacks drawn at random (fixed seeds), each compared with the oracle as in the hand-picked parity tests:
bit for bit for selection, gathering, scattering and averaging, within 1e-4 relative L2 for the autoencoder.
The hand-picked tests aim at the boundaries someone thought of; these are for the ones nobody did."""
import numpy as np
import pytest
import torch

from paper_2103_08870_amd import synth
from test_gpu_parity import B, ELEM_TOL_DEEP, assert_close  # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


def bits(t, a):
    """Bit for bit, except that where the oracle holds a NaN any NaN will do: a NaN that went through the
    accumulation keeps its NaN-ness, but its sign and payload follow the processor's propagation rule."""
    h = t.detach().cpu().numpy()
    if h.shape != a.shape:
        return False
    same = h.view(np.uint32) == a.view(np.uint32)
    return bool((same | (np.isnan(h) & np.isnan(a))).all())


def values(rng, shape, kind):
    if kind == 0:
        return rng.standard_normal(shape).astype(np.float32)
    if kind == 1:
        return rng.laplace(0, 1e-3, shape).astype(np.float32)
    if kind == 2:   # few distinct magnitudes
        return (rng.integers(-6, 7, shape) * 0.25).astype(np.float32)
    if kind == 3:   # mostly zeros
        x = rng.standard_normal(shape).astype(np.float32)
        x[rng.random(shape) < 0.97] = 0.0
        return x
    if kind == 4:   # heavy tail with a tie plateau at the top
        x = (rng.standard_normal(shape) * 10.0 ** rng.integers(-6, 3, shape)).astype(np.float32)
        x[rng.random(shape) < 0.01] = np.float32(1234.5)
        return x
    if kind == 5:   # magnitudes growing / falling along the index
        n = shape[-1]
        ramp = np.linspace(0, 1, n, dtype=np.float32)
        x = rng.standard_normal(shape).astype(np.float32) * (ramp if rng.random() < 0.5 else ramp[::-1])
        return x.astype(np.float32)
    x = rng.standard_normal(shape).astype(np.float32)   # special values mixed in
    sp = np.array([np.inf, -np.inf, np.nan, 1e-45, -1e-45, 0.0, -0.0, 3.4e38], np.float32)
    m = rng.random(shape) < 0.001
    x[m] = sp[rng.integers(0, sp.size, int(m.sum()))]
    return x


def rand_n(rng):
    r = rng.random()
    if r < 0.25:
        return int(rng.integers(1, 5000))
    if r < 0.5:
        return int(rng.integers(5000, 300_000))
    if r < 0.8:
        return int(rng.integers(262_144, 1_500_000))
    return int(rng.integers(1_500_000, 6_000_000))


def rand_k(rng, n):
    r = rng.random()
    if r < 0.1:
        return int(rng.integers(0, min(n, 3) + 1))
    if r < 0.6:
        return max(1, int(n * 10.0 ** rng.uniform(-4, -2)))
    if r < 0.9:
        return max(1, int(n * 10.0 ** rng.uniform(-2, -0.7)))
    return int(rng.integers(max(1, n // 2), n + 1))


def case_flat(B, O, rng, desc):
    n = rand_n(rng); k = rand_k(rng, n); batch = int(rng.integers(1, 5))
    pad = int(rng.choice([0, 0, 1, 3, 4, 64])); shift = int(rng.choice([0, 0, 0, 1, 2, 4]))
    kind = int(rng.integers(0, 7)); fused = bool(rng.random() < 0.6); with_u = fused or bool(rng.random() < 0.6)
    force = bool(rng.random() < 0.2); iters = int(rng.integers(1, 4)); m = float(rng.choice([0.0, 0.5, 0.9]))
    desc.append(f"flat n={n} k={k} batch={batch} pad={pad} shift={shift} kind={kind} fused={fused} u={with_u} force={force} iters={iters} m={m}")
    stride = n + pad
    ctx = B.Context(max(n, 16), max(k, 1), batch)
    if force:
        B.lgc_set_option(ctx, B.LGC_OPT_SELECT_PATH, 1)
    u = values(rng, (batch, stride), 0) * np.float32(1e-3)
    v = values(rng, (batch, stride), kind)
    flat = lambda a: torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), a.ravel()])).cuda()
    du_f, dv_f = flat(u), flat(v)
    view = lambda t: t[shift:].view(batch, stride)[:, :n]
    for it in range(iters):
        g = values(rng, (batch, stride), kind if it % 2 == 0 else 1)
        dg_f = flat(g)
        ovals = torch.full((batch, k), 7.0, device="cuda"); oidx = torch.full((batch, k), -1, device="cuda", dtype=torch.int32)
        if fused:
            B.lgc_accumulate_topk(ctx, view(dg_f), view(du_f), view(dv_f), m, k, ovals, oidx)
        else:
            B.lgc_topk(ctx, view(dv_f), view(du_f) if with_u else None, k, ovals, oidx)
        assert B.lgc_stats(ctx)[2] == 0, "device-side errors"
        for b in range(batch):
            ub, vb = u[b, :n].copy(), v[b, :n].copy()
            if fused:
                O.accumulate(g[b, :n].copy(), ub, vb, m)
            vals, idx = O.topk(vb, ub if with_u else None, k)
            u[b, :n], v[b, :n] = ub, vb
            assert (oidx[b].cpu().numpy().astype(np.uint32) == idx).all(), ("idx", it, b)
            assert bits(ovals[b], vals), ("vals", it, b)
        assert bits(dv_f[shift:].view(batch, stride), v), ("v", it)
        assert bits(du_f[shift:].view(batch, stride), u), ("u", it)
    ctx.close()


def case_seg(B, O, rng, desc):
    n = rand_n(rng) + 64; batch = int(rng.integers(1, 4)); kind = int(rng.integers(0, 7))
    n_seg = int(rng.integers(1, min(400, n // 8) + 1))
    cuts = np.sort(rng.choice(np.arange(1, n), size=n_seg - 1, replace=False)) if n_seg > 1 else np.array([], np.int64)
    off = [0] + [int(c) for c in cuts] + [n]
    ratio = 10.0 ** rng.uniform(-4, -0.5)
    ks = [min(off[i + 1] - off[i], max(1, int(ratio * (off[i + 1] - off[i])))) for i in range(n_seg)]
    if rng.random() < 0.3:
        for i in rng.integers(0, n_seg, 3):
            ks[i] = int(rng.integers(0, off[i + 1] - off[i] + 1))
    fused = bool(rng.random() < 0.6); iters = int(rng.integers(1, 3))
    desc.append(f"seg n={n} n_seg={n_seg} total_k={sum(ks)} batch={batch} kind={kind} fused={fused} iters={iters}")
    total = sum(ks)
    ctx = B.Context(n, max(total, 1), batch)
    seg = B.Segments(off, ks)
    B.lgc_reserve(ctx, seg=seg)
    u = values(rng, (batch, n), 0) * np.float32(1e-3); v = values(rng, (batch, n), kind)
    du, dv = torch.from_numpy(u.copy()).cuda(), torch.from_numpy(v.copy()).cuda()
    for it in range(iters):
        g = values(rng, (batch, n), 1)
        dg = torch.from_numpy(g).cuda()
        ovals = torch.full((batch, total), 7.0, device="cuda"); oidx = torch.full((batch, total), -1, device="cuda", dtype=torch.int32)
        if fused:
            B.lgc_accumulate_topk_segmented(ctx, seg, dg, du, dv, 0.9, ovals, oidx)
        else:
            B.lgc_topk_segmented(ctx, seg, dv, du, ovals, oidx)
        assert B.lgc_stats(ctx)[2] == 0
        for b in range(batch):
            ub, vb = u[b].copy(), v[b].copy()
            if fused:
                O.accumulate(g[b].copy(), ub, vb, 0.9)
            vals, idx = O.topk_segmented(vb, ub, off, ks)
            u[b], v[b] = ub, vb
            assert (oidx[b].cpu().numpy().astype(np.uint32) == idx).all(), ("idx", it, b)
            assert bits(ovals[b], vals), ("vals", it, b)
        assert bits(dv, v) and bits(du, u), ("uv", it)
    seg.close(); ctx.close()


def case_scatter(B, O, rng, desc):
    n = rand_n(rng); batch = int(rng.integers(1, 9)); k = min(n, max(1, rand_k(rng, n)))
    mode = int(rng.integers(0, 3))
    desc.append(f"scatter n={n} k={k} batch={batch} mode={mode}")
    ctx = B.Context(max(n, 16), k, batch)
    idx = np.zeros((batch, k), np.uint32)
    for b in range(batch):
        if mode == 0:
            idx[b] = np.sort(rng.choice(n, k, replace=False)).astype(np.uint32)
        elif mode == 1:   # same positions in all nodes
            idx[b] = idx[0] if b else np.sort(rng.choice(n, k, replace=False)).astype(np.uint32)
        else:             # clustered
            lo = int(rng.integers(0, n - k + 1)); idx[b] = np.arange(lo, lo + k, dtype=np.uint32)
    vals = values(rng, (batch, k), 0)
    dense = values(rng, (n,), 1)
    dd = torch.from_numpy(dense.copy()).cuda()
    B.lgc_scatter(ctx, torch.from_numpy(vals).cuda(), torch.from_numpy(idx.view(np.int32)).cuda(), 1.0 / batch, dd)
    for b in range(batch):
        O.scatter(vals[b], idx[b], 1.0 / batch, dense)
    assert bits(dd, dense)
    ctx.close()


CH = [1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 48, 64, 128]


def rand_stack(rng):
    n_enc = int(rng.integers(1, 6)); n_dec = int(rng.integers(1, 6))
    es = [int(rng.random() < 0.55) + 1 for _ in range(n_enc)]
    twos = sum(1 for x in es if x == 2)
    if twos > n_dec:
        n_dec = twos
    pos = set(rng.choice(n_dec, twos, replace=False).tolist()) if twos else set()
    ds = [2 if i in pos else 1 for i in range(n_dec)]
    ec = [1] + [int(rng.choice(CH)) for _ in range(n_enc)]
    dc = [ec[-1]] + [int(rng.choice(CH)) for _ in range(n_dec - 1)] + [1]
    ks = lambda: 3 if rng.random() < 0.8 else 1
    enc = [(ec[i], ec[i + 1], ks(), es[i]) for i in range(n_enc)]
    dec = [(dc[i], dc[i + 1], ks(), ds[i]) for i in range(n_dec)]
    return enc, dec


def case_ae(B, O, rng, desc):
    r = rng.random()
    if r < 0.15:
        enc, dec = synth.paper_ae()
    elif r < 0.3:
        enc, dec = synth.mirrored_ae((1, int(rng.choice([4, 8, 16])), int(rng.choice([2, 4, 8]))))
    else:
        enc, dec = rand_stack(rng)
    cost = sum(a * b * c for a, b, c, _ in list(enc) + list(dec))
    kmax = max(1, min(60_000, int(3e8 / cost)))
    k = int(rng.integers(1, kmax + 1)) if rng.random() < 0.7 else int(rng.integers(1, min(kmax, 300) + 1))
    batch = int(rng.integers(1, 5)); slope = float(rng.choice([0.0, 0.01, 0.2]))
    seed = int(rng.integers(0, 1 << 30))
    desc.append(f"ae enc={list(enc)} dec={list(dec)} k={k} batch={batch} slope={slope} wseed={seed}")
    ew, eb, dw, db = synth.ae_weights(enc, dec, device="cuda", seed=seed)
    ae = B.Autoencoder(enc, dec, ew, eb, dw, db, slope=slope)
    hw = [[t.cpu().numpy() for t in xs] for xs in (ew, eb, dw, db)]
    ctx = B.Context(1 << 16, 1 << 16, batch)
    B.lgc_reserve(ctx, ae, k, batch)
    x = rng.laplace(0, 1e-2, (batch, k)).astype(np.float32)
    lat = torch.zeros((batch, B.lgc_latent_len(ae, k)), device="cuda")
    B.lgc_encode(ctx, ae, torch.from_numpy(x).cuda(), lat)
    ols = [O.encode(x[b], enc, hw[0], hw[1], slope=slope) for b in range(batch)]
    rec = torch.zeros((batch, k), device="cuda")
    B.lgc_decode(ctx, ae, torch.from_numpy(np.stack([o.ravel() for o in ols])).cuda(), rec)
    for b in range(batch):
        assert_close(lat[b], ols[b], elem=ELEM_TOL_DEEP, what=("latent", b))
        assert_close(rec[b], O.decode(ols[b], k, enc, dec, hw[2], hw[3], slope=slope), elem=ELEM_TOL_DEEP,
                     what=("reconstruction", b))
    ctx.close(); ae.close()


def case_gather(B, O, rng, desc):
    n = rand_n(rng); batch = int(rng.integers(1, 9)); k = min(n, max(1, rand_k(rng, n)))
    fused = bool(rng.random() < 0.5); with_u = fused or bool(rng.random() < 0.5); pad = int(rng.choice([0, 1, 4]))
    desc.append(f"gather n={n} k={k} batch={batch} fused={fused} u={with_u} pad={pad}")
    stride = n + pad
    ctx = B.Context(max(n, 16), k, batch)
    idx = np.sort(rng.choice(n, k, replace=False)).astype(np.uint32)
    u = values(rng, (batch, stride), 1); v = values(rng, (batch, stride), 0); g = values(rng, (batch, stride), 1)
    du, dv, dg = (torch.from_numpy(a.copy()).cuda() for a in (u, v, g))
    out = torch.full((batch, k), 7.0, device="cuda")
    di = torch.from_numpy(idx.view(np.int32)).cuda()
    if fused:
        B.lgc_accumulate_gather(ctx, dg[:, :n], du[:, :n], dv[:, :n], 0.9, di, out)
    else:
        B.lgc_gather(ctx, dv[:, :n], du[:, :n] if with_u else None, di, out)
    ref = np.zeros((batch, k), np.float32)
    for b in range(batch):
        ub, vb = u[b, :n].copy(), v[b, :n].copy()
        if fused:
            O.accumulate(g[b, :n].copy(), ub, vb, 0.9)
        ref[b] = O.gather(vb, ub if with_u else None, idx)
        u[b, :n], v[b, :n] = ub, vb
    assert bits(out, ref) and bits(dv, v) and bits(du, u)
    L = int(rng.integers(1, 200_000)); xs = values(rng, (batch, L), 0)
    avg = torch.zeros(L, device="cuda")
    B.lgc_average(ctx, torch.from_numpy(xs).cuda(), 1.0 / batch, avg)
    assert bits(avg, O.average(xs, 1.0 / batch))
    ctx.close()


def case_innovation(B, O, rng, desc):
    k = int(rng.integers(1, 200_000)); batch = int(rng.integers(1, 5)); kind = int(rng.integers(0, 7))
    n_seg = int(rng.integers(1, min(400, k) + 1))
    cuts = np.sort(rng.choice(np.arange(1, k), size=n_seg - 1, replace=False)) if n_seg > 1 else np.array([], np.int64)
    off = [0] + [int(c) for c in cuts] + [k]
    ks = [int(rng.integers(0, max(1, (off[i + 1] - off[i]) // 3) + 1)) for i in range(n_seg)]
    desc.append(f"innovation k={k} n_seg={n_seg} kept={sum(ks)} batch={batch} kind={kind}")
    ctx = B.Context(max(k, 16), max(k, 1), batch)
    seg = B.Segments(off, ks)
    vals = values(rng, (batch, k), kind)
    out = torch.full((batch, k), 7.0, device="cuda")
    B.lgc_innovation(ctx, seg, torch.from_numpy(vals).cuda(), out)
    assert B.lgc_stats(ctx)[2] == 0
    for b in range(batch):
        assert bits(out[b], O.innovation(vals[b], off, ks)), b
    seg.close(); ctx.close()

def case_reuse(B, O, rng, desc):
    """One context, many calls of different n, k, batch, path and entry point."""
    max_n = int(rng.choice([300_000, 1_200_000, 3_000_000])); max_k = max_n // int(rng.choice([3, 10, 100])); max_b = int(rng.integers(1, 5))
    calls = int(rng.integers(4, 12))
    desc.append(f"reuse max_n={max_n} max_k={max_k} max_b={max_b} calls={calls}")
    ctx = B.Context(max_n, max_k, max_b)
    for c in range(calls):
        n = int(rng.integers(1, max_n + 1)) if rng.random() < 0.7 else max_n
        k = min(n, max_k, rand_k(rng, n)); batch = int(rng.integers(1, max_b + 1)); kind = int(rng.integers(0, 6))
        mode = int(rng.integers(0, 4)); force = int(rng.random() < 0.25)
        desc.append(f"  call {c}: n={n} k={k} batch={batch} kind={kind} mode={mode} force={force}")
        B.lgc_set_option(ctx, B.LGC_OPT_SELECT_PATH, force)
        u = values(rng, (batch, n), 1); v = values(rng, (batch, n), kind); g = values(rng, (batch, n), 1)
        du, dv, dg = (torch.from_numpy(a.copy()).cuda() for a in (u, v, g))
        if mode == 3:   # per-layer plan over the same vector
            n_seg = int(rng.integers(1, min(100, n) + 1))
            cuts = np.sort(rng.choice(np.arange(1, n), size=n_seg - 1, replace=False)) if n_seg > 1 else np.array([], np.int64)
            off = [0] + [int(x) for x in cuts] + [n]
            ks = [min(off[i + 1] - off[i], max(1, int((k / n) * (off[i + 1] - off[i])))) for i in range(n_seg)]
            while sum(ks) > max_k:
                ks[int(np.argmax(ks))] //= 2
            total = sum(ks)
            seg = B.Segments(off, ks)
            B.lgc_reserve(ctx, seg=seg)
            ovals = torch.full((batch, total), 7.0, device="cuda"); oidx = torch.full((batch, total), -1, device="cuda", dtype=torch.int32)
            B.lgc_accumulate_topk_segmented(ctx, seg, dg, du, dv, 0.9, ovals, oidx)
            seg.close()
        else:
            ovals = torch.full((batch, k), 7.0, device="cuda"); oidx = torch.full((batch, k), -1, device="cuda", dtype=torch.int32)
            if mode == 0:
                B.lgc_accumulate_topk(ctx, dg, du, dv, 0.9, k, ovals, oidx)
            elif mode == 1:
                B.lgc_topk(ctx, dv, du, k, ovals, oidx)
            else:
                B.lgc_accumulate(ctx, dg, du, dv, 0.9)
                B.lgc_topk(ctx, dv, None, k, ovals, oidx)
        assert B.lgc_stats(ctx)[2] == 0
        for b in range(batch):
            ub, vb = u[b].copy(), v[b].copy()
            if mode != 1:
                O.accumulate(g[b].copy(), ub, vb, 0.9)
            if mode == 3:
                vals, idx = O.topk_segmented(vb, ub, off, ks)
            else:
                vals, idx = O.topk(vb, ub if mode != 2 else None, k)
            u[b], v[b] = ub, vb
            assert (oidx[b].cpu().numpy().astype(np.uint32) == idx).all(), ("idx", c, b)
            assert bits(ovals[b], vals), ("vals", c, b)
        assert bits(dv, v) and bits(du, u), ("uv", c)
    ctx.close()


def run_cases(B, oracle, fn, family, block, count):
    for i in range(count):
        rng = np.random.default_rng([20210308, family, block, i])
        desc = []
        try:
            fn(B, oracle, rng, desc)
        except AssertionError as e:
            raise AssertionError(f"case {i} of block {block}: {desc}: {e}") from e


@pytest.mark.parametrize("block", range(6))
def test_random_flat_selection(B, oracle, block):
    run_cases(B, oracle, case_flat, 0, block, 10)


@pytest.mark.parametrize("block", range(3))
def test_random_per_layer_selection(B, oracle, block):
    run_cases(B, oracle, case_seg, 1, block, 10)


@pytest.mark.parametrize("block", range(2))
def test_random_scatter(B, oracle, block):
    run_cases(B, oracle, case_scatter, 2, block, 15)


@pytest.mark.parametrize("block", range(4))
def test_random_autoencoder_stacks(B, oracle, block):
    run_cases(B, oracle, case_ae, 3, block, 20)


@pytest.mark.parametrize("block", range(2))
def test_random_gather_and_average(B, oracle, block):
    run_cases(B, oracle, case_gather, 4, block, 15)


@pytest.mark.parametrize("block", range(2))
def test_random_innovation(B, oracle, block):
    run_cases(B, oracle, case_innovation, 5, block, 20)


@pytest.mark.parametrize("block", range(2))
def test_random_calls_on_one_context(B, oracle, block):
    run_cases(B, oracle, case_reuse, 6, block, 6)
