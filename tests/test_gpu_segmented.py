"""GPU parity of the per-layer (segmented) top-k, through the C ABI, against the CPU oracle:
positions, values, residual v and momentum buffer u bit for bit."""
import numpy as np
import pytest
import torch

from paper_2103_08870_amd import synth
from test_gpu_parity import B, dev, same_bits  # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


def run_segmented(B, oracle, ctx, seg, offsets, ks, v0, u0, g=None, momentum=0.9, pad=0):
    """v0, u0, g: [batch][n] numpy.  Runs the library and the oracle and compares everything;
    returns the (fast, fallback) counters."""
    batch, n = v0.shape
    K = int(np.sum(ks))

    def padded(a):
        if a is None:
            return None, None
        full = np.zeros((batch, n + pad), np.float32)
        full[:, :n] = a
        d = dev(full)
        return d, d[:, :n]
    dvf, dv = padded(v0)
    duf, du = padded(u0)
    ovals = torch.full((batch, K), 7.0, device="cuda")
    oidx = torch.full((batch, K), -1, device="cuda", dtype=torch.int32)
    if g is not None:
        _, dg = padded(g)
        B.lgc_accumulate_topk_segmented(ctx, seg, dg, du, dv, momentum, ovals, oidx)
    else:
        B.lgc_topk_segmented(ctx, seg, dv, du, ovals, oidx)
    fast, fallback, errors = B.lgc_stats(ctx)
    assert errors == 0
    for b in range(batch):
        v1 = v0[b].copy()
        u1 = u0[b].copy() if u0 is not None else None
        if g is not None:
            oracle.accumulate(g[b].copy(), u1, v1, momentum)
        vals, idx = oracle.topk_segmented(v1, u1, offsets, ks)
        got = oidx[b].cpu().numpy().astype(np.uint32)
        assert (got == idx).all(), (b, int(np.argmax(got != idx)))
        assert same_bits(ovals[b], vals)
        assert same_bits(dv[b], v1)
        if u0 is not None:
            assert same_bits(du[b], u1)
    if pad:
        assert (dvf[:, n:] == 0).all()
    return fast, fallback


def random_layout(rng, n, n_seg):
    cuts = np.sort(rng.choice(np.arange(1, n), n_seg - 1, replace=False)) if n_seg > 1 else np.array([], int)
    return np.concatenate([[0], cuts, [n]]).astype(np.int64)


@pytest.mark.parametrize("n,n_seg,batch,pad", [(1, 1, 1, 0), (77, 5, 2, 0), (10_000, 40, 2, 3), (15_001, 3, 1, 0),
                                               (200_000, 400, 3, 4)])
def test_small_segments_selected_from_v(B, oracle, n, n_seg, batch, pad):
    # every segment is below the sampling size (16 K elements): one block per (segment, node) works on v itself
    rng = np.random.default_rng(n + n_seg)
    off = random_layout(rng, n, n_seg)
    lens = np.diff(off)
    ks = np.array([rng.integers(0, min(m, 50) + 1) for m in lens])
    ks[0] = min(1, lens[0]); ks[-1] = lens[-1] if lens[-1] < 3000 else 7       # k_l = 1, k_l = n_l
    ctx = B.Context(n, max(int(ks.sum()), 1), batch)
    seg = B.Segments(off.tolist(), ks.tolist())
    B.lgc_reserve(ctx, seg=seg)
    assert seg.total_k == int(ks.sum())
    for trial in range(2):
        if trial == 0:
            v0 = rng.standard_normal((batch, n)).astype(np.float32)
        else:       # few distinct magnitudes: ties at every cut, mixed signs
            v0 = (rng.integers(-4, 5, (batch, n)) * 0.25).astype(np.float32)
        u0 = rng.standard_normal((batch, n)).astype(np.float32)
        assert run_segmented(B, oracle, ctx, seg, off, ks, v0, u0 if trial == 0 else None, pad=pad) == (0, 0)
    seg.close(); ctx.close()


def mixed_layout():
    """Sampled and direct segments side by side, boundaries at odd places (rows of 1024 elements
    that hold several segments, segments that start and end inside a row)."""
    sizes = [100, 70_001, 5, 200_000, 65_536, 999_999, 3_000, 64, 64, 64, 300_000, 1, 131_073, 450_000, 8_191, 777,
             8_192, 33]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    ks = [max(1, s // 1000) for s in sizes]
    ks[2] = 5            # whole segment
    ks[8] = 0            # nothing from this one
    ks[10] = 100_000     # a third of a large segment: too dense for sampling, selected from v
    ks[13] = 4_500       # 1 %
    return off, np.array(ks)


@pytest.mark.parametrize("fused,aligned_base", [(False, True), (True, True), (True, False)])
def test_mixed_segments(B, oracle, fused, aligned_base):
    off, ks = mixed_layout()
    n = int(off[-1])
    batch = 2
    rng = np.random.default_rng(11 + fused)
    ctx = B.Context(n + 1, int(ks.sum()), batch)
    seg = B.Segments(off.tolist(), ks.tolist())
    B.lgc_reserve(ctx, seg=seg)
    scale = np.repeat(np.exp(rng.uniform(np.log(1e-5), np.log(1e-2), len(ks))), np.diff(off)).astype(np.float32)
    v0 = (rng.laplace(0, 1, (batch, n)) * scale).astype(np.float32)
    u0 = (rng.standard_normal((batch, n)) * scale).astype(np.float32)
    g = (rng.laplace(0, 1, (batch, n)) * scale).astype(np.float32) if fused else None
    if aligned_base:
        fast, fallback = run_segmented(B, oracle, ctx, seg, off, ks, v0, u0, g)
    else:
        # base pointers 4 bytes off a 16-byte boundary: the scalar-load variants of every kernel
        dv, du = dev(np.concatenate([[0], v0[0]]).astype(np.float32)), dev(np.concatenate([[0], u0[0]]).astype(np.float32))
        dg = dev(np.concatenate([[0], g[0]]).astype(np.float32))
        K = int(ks.sum())
        ovals = torch.zeros((1, K), device="cuda"); oidx = torch.zeros((1, K), device="cuda", dtype=torch.int32)
        B.lgc_accumulate_topk_segmented(ctx, seg, dg[1:], du[1:], dv[1:], 0.9, ovals, oidx)
        fast, fallback, errors = B.lgc_stats(ctx)
        assert errors == 0
        v1, u1 = v0[0].copy(), u0[0].copy()
        oracle.accumulate(g[0].copy(), u1, v1, 0.9)
        vals, idx = oracle.topk_segmented(v1, u1, off, ks)
        assert (oidx[0].cpu().numpy().astype(np.uint32) == idx).all() and same_bits(ovals[0], vals)
        assert same_bits(dv[1:], v1) and same_bits(du[1:], u1)
        batch = 1
    # sampled: 70 001, 200 000, 65 536, 999 999, 131 073, 450 000, 8 192 (not the dense one, not 8 191)
    assert fast == 7 * batch and fallback == 0
    seg.close(); ctx.close()


def test_candidate_overflow_falls_back_to_v(B, oracle):
    # one large segment of equal magnitudes: its estimate flags every element, the candidate list
    # overflows, and every sampled segment is then selected from v itself (the slow, exact way)
    sizes = [100_000, 400_000, 80_000, 30_000]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    ks = np.array([100, 400, 80, 30])
    n = int(off[-1])
    rng = np.random.default_rng(4)
    v0 = rng.standard_normal((1, n)).astype(np.float32)
    v0[0, off[1]:off[2]] = 0.5
    v0[0, off[1]:off[2]:3] = -0.5
    ctx = B.Context(n, int(ks.sum()), 1)
    seg = B.Segments(off.tolist(), ks.tolist())
    B.lgc_reserve(ctx, seg=seg)
    assert run_segmented(B, oracle, ctx, seg, off, ks, v0, None) == (0, 4)
    seg.close(); ctx.close()


def test_fused_equals_accumulate_then_segmented(B):
    w = synth.workload(2, n=1_500_000)
    off, ks = synth.layer_plan(w)
    K = sum(ks)
    ctx = B.Context(w.n, K, w.nodes)
    seg = B.Segments(off, ks)
    B.lgc_reserve(ctx, seg=seg)
    g = synth.gradients(w, 0, device="cuda")
    u1 = torch.randn((w.nodes, w.n), device="cuda") * 1e-4
    v1 = torch.randn((w.nodes, w.n), device="cuda") * 1e-4
    u2, v2 = u1.clone(), v1.clone()
    va, ia = torch.zeros((w.nodes, K), device="cuda"), torch.zeros((w.nodes, K), device="cuda", dtype=torch.int32)
    vb, ib = torch.zeros_like(va), torch.zeros_like(ia)
    B.lgc_accumulate_topk_segmented(ctx, seg, g, u1, v1, 0.9, va, ia)
    B.lgc_accumulate(ctx, g, u2, v2, 0.9)
    B.lgc_topk_segmented(ctx, seg, v2, u2, vb, ib)
    assert B.lgc_stats(ctx)[2] == 0
    assert torch.equal(ia, ib) and torch.equal(va.view(torch.int32), vb.view(torch.int32))
    assert torch.equal(u1.view(torch.int32), u2.view(torch.int32)) and torch.equal(v1.view(torch.int32), v2.view(torch.int32))
    seg.close(); ctx.close()


@pytest.mark.parametrize("cfg,n", [(2, 2_000_003), (3, 1_500_000), (4, 2_100_000)])
def test_workload_iterations(B, oracle, cfg, n):
    # the workloads' own layers (161 / 314 / 400 segments, mu_l = max(1, floor(ratio n_l))), state carried
    w = synth.workload(cfg, n=n, nodes=2)
    off, ks = synth.layer_plan(w)
    ctx = B.Context(n, sum(ks), w.nodes)
    seg = B.Segments(off, ks)
    B.lgc_reserve(ctx, seg=seg)
    u = np.zeros((w.nodes, n), np.float32); v = np.zeros((w.nodes, n), np.float32)
    for t in range(3):
        g = synth.gradients(w, t, device="cpu").numpy()
        u0, v0 = u.copy(), v.copy()
        run_segmented(B, oracle, ctx, seg, np.array(off), np.array(ks), v0, u0, g, w.momentum)
        for b in range(w.nodes):
            oracle.accumulate(g[b], u[b], v[b], w.momentum)
            oracle.topk_segmented(v[b], u[b], off, ks)
    seg.close(); ctx.close()


def test_full_size_resnet50_layers(B, oracle):
    # the benchmark's launch configuration: all 4 nodes x 25.6 M, 161 layers; two nodes checked in full
    w = synth.workload(2)
    off, ks = synth.layer_plan(w)
    K = sum(ks)
    sampled = sum(1 for a, b in zip(off, off[1:]) if b - a >= 8_192)
    ctx = B.Context(w.n, K, w.nodes)
    seg = B.Segments(off, ks)
    B.lgc_reserve(ctx, seg=seg)
    u = torch.zeros((w.nodes, w.n), device="cuda"); v = torch.zeros((w.nodes, w.n), device="cuda")
    vals = torch.zeros((w.nodes, K), device="cuda"); idx = torch.zeros((w.nodes, K), device="cuda", dtype=torch.int32)
    hu = np.zeros((2, w.n), np.float32); hv = np.zeros((2, w.n), np.float32)
    for t in range(2):
        g = synth.gradients(w, t, device="cuda")
        B.lgc_accumulate_topk_segmented(ctx, seg, g, u, v, w.momentum, vals, idx)
        fast, fallback, errors = B.lgc_stats(ctx)
        assert errors == 0 and fallback == 0 and fast == sampled * w.nodes
        for j, b in enumerate((0, w.nodes - 1)):
            oracle.accumulate(g[b].cpu().numpy(), hu[j], hv[j], w.momentum)
            ovals, oidx = oracle.topk_segmented(hv[j], hu[j], off, ks)
            assert (idx[b].cpu().numpy().astype(np.uint32) == oidx).all()
            assert same_bits(vals[b], ovals) and same_bits(v[b], hv[j]) and same_bits(u[b], hu[j])
    seg.close(); ctx.close()


def test_layer_thresholds_carried_at_full_size(B, oracle):
    """Alg. 1 / Alg. 2 at the benchmark's size for 24 iterations: once a layer's k-th magnitude moves smoothly its
    candidate threshold is taken from the trend of the layer's earlier selections instead of a sample
    (lgc_stats_carried counts layers and nodes); node 0 is compared with the oracle in full in every iteration,
    then the gradients are scaled by 5 for one more, which puts every carried threshold far off."""
    w = synth.workload(2)
    off, ks = synth.layer_plan(w)
    K = sum(ks)
    sampled = sum(1 for a, b in zip(off, off[1:]) if b - a >= 8_192)
    ctx = B.Context(w.n, K, w.nodes)
    seg = B.Segments(off, ks)
    B.lgc_reserve(ctx, seg=seg)
    u = torch.zeros((w.nodes, w.n), device="cuda"); v = torch.zeros((w.nodes, w.n), device="cuda")
    vals = torch.zeros((w.nodes, K), device="cuda"); idx = torch.zeros((w.nodes, K), device="cuda", dtype=torch.int32)
    hu = np.zeros(w.n, np.float32); hv = np.zeros(w.n, np.float32)
    carried, fell_back = [], []
    for t in range(25):
        g = synth.gradients(w, t % 10, device="cuda") * (5.0 if t == 24 else 1.0)
        B.lgc_accumulate_topk_segmented(ctx, seg, g, u, v, w.momentum, vals, idx)
        fast, fallback, errors = B.lgc_stats(ctx)
        assert errors == 0 and fast + fallback == sampled * w.nodes
        carried.append(B.lgc_stats_carried(ctx)); fell_back.append(fallback)
        oracle.accumulate(g[0].cpu().numpy(), hu, hv, w.momentum)
        ovals, oidx = oracle.topk_segmented(hv, hu, off, ks)
        assert (idx[0].cpu().numpy().astype(np.uint32) == oidx).all(), t
        assert same_bits(vals[0], ovals) and same_bits(v[0], hv) and same_bits(u[0], hu), t
    print("layers x nodes with a carried threshold per iteration:", carried, "fell back:", fell_back)
    assert sum(carried[:4]) == 0 and carried[23] > sampled * w.nodes // 4
    assert sum(fell_back) <= sum(carried) // 100        # a carried threshold that fails sends its layer to the exact path: rare
    seg.close(); ctx.close()


def test_argument_errors(B):
    with pytest.raises(B.LgcError):
        B.Segments([0, 5, 5, 10], [1, 0, 1])          # empty segment
    with pytest.raises(B.LgcError):
        B.Segments([0, 5, 10], [6, 1])                # k_l > n_l
    with pytest.raises(B.LgcError):
        B.Segments([1, 5, 10], [1, 1])                # does not start at 0
    ctx = B.Context(100, 4, 1)
    seg = B.Segments([0, 50, 100], [3, 3])            # 6 outputs > max_k
    v = torch.zeros(100, device="cuda")
    with pytest.raises(B.LgcError):
        B.lgc_topk_segmented(ctx, seg, v, None, torch.zeros(6, device="cuda"), torch.zeros(6, device="cuda", dtype=torch.int32))
    seg.close(); ctx.close()


def test_adversarial_layouts_per_layer(B, oracle):
    """The magnitude layouts of test_topk_adversarial_layouts under a per-layer plan of large (sampled) and
    small layers: ramps, a cut inside a tie group, mostly zeros, one hot stretch, infinities and NaNs."""
    from test_gpu_parity import adversarial_inputs
    n = 2_300_000
    rng = np.random.default_rng(9)
    off = np.unique(np.concatenate([[0, n], rng.choice(np.arange(1, n), 11, replace=False),
                                    900_000 + np.arange(1, 30) * 500]))      # 12 large layers, 29 of 500 elements
    lens = np.diff(off)
    ks = np.maximum(1, lens // 60)
    ctx = B.Context(n, int(ks.sum()), 1)
    seg = B.Segments(off.tolist(), ks.tolist())
    B.lgc_reserve(ctx, seg=seg)
    u0 = rng.standard_normal((1, n)).astype(np.float32)
    for name, v in adversarial_inputs(n, int(ks.sum()), rng):
        run_segmented(B, oracle, ctx, seg, off, ks, v[None, :].copy(), u0)
    seg.close(); ctx.close()
