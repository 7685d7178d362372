"""GPU parity of the ring-allreduce pattern's calls (values at shared positions, average of the
compressed representations) and of the whole ring-allreduce iteration, through the C ABI, against
the CPU oracle: bit-exact for values, residual, momentum buffer and average; autoencoder outputs
within 1e-4 relative L2."""
import numpy as np
import pytest
import torch

from paper_2103_08870_amd import synth
from test_gpu_parity import B, REL_L2_TOL, assert_close, dev, make_ae, rel_l2, same_bits  # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,batch,pad,k", [(5, 1, 0, 2), (4097, 2, 3, 100), (1_000_003, 3, 1, 5000), (2_000_000, 4, 0, 0)])
def test_gather_and_accumulate_gather(B, oracle, n, batch, pad, k):
    rng = np.random.default_rng(n + k)
    stride = n + pad
    ctx = B.Context(n, max(k, 1), batch)
    u = rng.standard_normal((batch, stride)).astype(np.float32)
    v = rng.standard_normal((batch, stride)).astype(np.float32)
    du, dv = dev(u), dev(v)
    for t in range(3):
        idx = np.sort(rng.choice(n, k, replace=False)).astype(np.uint32)
        didx = dev(idx.astype(np.int32))
        out = torch.full((batch, k), 7.0, device="cuda")
        if t == 1:      # plain gather, without the momentum buffer on the odd iteration
            B.lgc_gather(ctx, dv[:, :n], None, didx, out)
            ref = [oracle.gather(v[b, :n], None, idx) for b in range(batch)]
        else:
            g = (rng.standard_normal((batch, stride)) * 0.1).astype(np.float32)
            B.lgc_accumulate_gather(ctx, dev(g)[:, :n], du[:, :n], dv[:, :n], 0.9, didx, out)
            ref = []
            for b in range(batch):
                oracle.accumulate(g[b, :n].copy(), u[b, :n], v[b, :n], 0.9)
                ref.append(oracle.gather(v[b, :n], u[b, :n], idx))
        assert B.lgc_stats(ctx)[2] == 0
        for b in range(batch):
            assert same_bits(out[b], ref[b])
        assert same_bits(dv, v) and same_bits(du, u)          # padding untouched too
    ctx.close()


def test_gather_position_out_of_range_is_counted(B, oracle):
    n, k = 1000, 10
    ctx = B.Context(n, k, 1)
    v = np.arange(n, dtype=np.float32)
    dv = dev(v)
    idx = np.arange(0, 100, 10).astype(np.int64)
    idx[3] = n + 5
    out = torch.full((1, k), 7.0, device="cuda")
    B.lgc_gather(ctx, dv, None, dev(idx.astype(np.int32)), out)
    assert B.lgc_stats(ctx, check=False)[2] == 1
    keep = np.arange(k) != 3
    ref = oracle.gather(v, None, idx[keep].astype(np.uint32))
    o = out[0].cpu().numpy()
    assert (o[keep] == ref).all() and o[3] == 0.0
    assert same_bits(dv, v)
    ctx.close()


@pytest.mark.parametrize("K,length", [(1, 1), (3, 1000), (4, 25_600), (8, 89_001)])
def test_average(B, oracle, K, length):
    rng = np.random.default_rng(K + length)
    ctx = B.Context(16, 1, K)
    x = rng.standard_normal((K, length)).astype(np.float32)
    out = torch.zeros(length, device="cuda")
    for scale in (1.0 / K, 1.0 / 3.0):
        B.lgc_average(ctx, dev(x), scale, out)
        assert same_bits(out, oracle.average(x, scale))
    ctx.close()


@pytest.mark.parametrize("cfg,n", [(2, 1_300_000), (3, 1_100_000)])
def test_ring_allreduce_iterations(B, oracle, cfg, n):
    """Alg. 2 with the selecting node rotating: the selecting node runs accumulate + top-k, the
    others accumulate and take the values at its positions; all encode, the compressed
    representations are averaged, decoded once and placed once.  Every stage is compared."""
    w = synth.workload(cfg, n=n)
    K, k = w.nodes, w.k
    ae, enc, dec, (ew, eb, dw, db) = make_ae(B, w.ae_channels)
    ctx = B.Context(n, k, K)
    u = np.zeros((K, n), np.float32); v = np.zeros((K, n), np.float32)
    du, dv = dev(u), dev(v)
    vals = torch.zeros((K, k), device="cuda")
    idx = torch.zeros(k, device="cuda", dtype=torch.int32)
    lat_len = B.lgc_latent_len(ae, k)
    lat = torch.zeros((K, lat_len), device="cuda")
    avg = torch.zeros((1, lat_len), device="cuda")
    rec = torch.zeros((1, k), device="cuda")
    for t in range(4):
        g = synth.gradients(w, t, device="cpu").numpy()
        dg = dev(g)
        L = (t * 3 + 1) % K                                   # the selecting node of this iteration
        B.lgc_accumulate_topk(ctx, dg[L], du[L], dv[L], w.momentum, k, vals[L], idx)
        for lo, hi in ((0, L), (L + 1, K)):
            if hi > lo:
                B.lgc_accumulate_gather(ctx, dg[lo:hi], du[lo:hi], dv[lo:hi], w.momentum, idx, vals[lo:hi])
        B.lgc_encode(ctx, ae, vals, lat)
        B.lgc_average(ctx, lat, 1.0 / K, avg[0])
        B.lgc_decode(ctx, ae, avg, rec)
        dense = torch.zeros(n, device="cuda")
        B.lgc_scatter(ctx, rec, idx.view(1, k), 1.0, dense)
        assert B.lgc_stats(ctx)[2] == 0
        # oracle
        for b in range(K):
            oracle.accumulate(g[b], u[b], v[b], w.momentum)
        ovals = np.zeros((K, k), np.float32)
        ovals[L], oidx = oracle.topk(v[L], u[L], k)
        for b in range(K):
            if b != L:
                ovals[b] = oracle.gather(v[b], u[b], oidx)
        assert (idx.cpu().numpy().astype(np.uint32) == oidx).all()
        assert same_bits(vals, ovals) and same_bits(dv, v) and same_bits(du, u)
        olat = np.stack([oracle.encode(ovals[b], enc, ew, eb).ravel() for b in range(K)])
        for b in range(K):
            assert_close(lat[b], olat[b], what=("latent", b))
        lat_h = lat.cpu().numpy()
        assert same_bits(avg[0], oracle.average(lat_h, 1.0 / K))              # exact on the same input
        oavg = oracle.average(olat, 1.0 / K)
        orec = oracle.decode(oavg.reshape(w.ae_channels[-1], -1), k, enc, dec, dw, db)
        assert_close(rec[0], orec, factor=2.0, what="reconstruction of the average")
        ref = np.zeros(n, np.float32)
        oracle.scatter(rec[0].cpu().numpy(), oidx, 1.0, ref)
        assert same_bits(dense, ref)
    ctx.close(); ae.close()


def test_ring_allreduce_full_size_resnet50(B, oracle):
    """The benchmark's launch configuration of the ring-allreduce pattern (4 nodes x 25.6 M, k = 25 600):
    selected values, positions and the state of the selecting node and of one other node, bit for bit."""
    w = synth.workload(2)
    K, n, k = w.nodes, w.n, w.k
    ctx = B.Context(n, k, K)
    u = torch.zeros((K, n), device="cuda"); v = torch.zeros((K, n), device="cuda")
    vals = torch.zeros((K, k), device="cuda"); idx = torch.zeros(k, device="cuda", dtype=torch.int32)
    hu = np.zeros((K, n), np.float32); hv = np.zeros((K, n), np.float32)
    for t in range(2):
        g = synth.gradients(w, t, device="cuda")
        L = (t + 1) % K
        B.lgc_accumulate_topk(ctx, g[L], u[L], v[L], w.momentum, k, vals[L], idx)
        for lo, hi in ((0, L), (L + 1, K)):
            if hi > lo:
                B.lgc_accumulate_gather(ctx, g[lo:hi], u[lo:hi], v[lo:hi], w.momentum, idx, vals[lo:hi])
        assert B.lgc_stats(ctx)[2] == 0
        gh = g.cpu().numpy()
        for b in range(K):
            oracle.accumulate(gh[b], hu[b], hv[b], w.momentum)
        ovals, oidx = oracle.topk(hv[L], hu[L], k)
        assert (idx.cpu().numpy().astype(np.uint32) == oidx).all() and same_bits(vals[L], ovals)
        for b in range(K):
            if b != L:
                assert same_bits(vals[b], oracle.gather(hv[b], hu[b], oidx))
        other = (L + 2) % K
        for b in (L, other):
            assert same_bits(v[b], hv[b]) and same_bits(u[b], hu[b])
    ctx.close()


def test_two_steps_in_a_hip_graph_replay_like_eager_calls(B, oracle):
    """The calls only enqueue kernels (no allocation, no host synchronisation, no memset once the
    scratch exists), so a stream capture of the path replays correctly.  The selection scratch
    alternates between two state sets from call to call, so a graph must hold an even number of
    selection calls.  Every replay is compared with the same steps made eagerly; there are enough replays for the
    selections to start taking their thresholds from the trend of the earlier ones (the record of those is kept
    on the device, so a replayed graph carries thresholds like eager calls do)."""
    w = synth.workload(2, n=1 << 21, nodes=2)
    K, n, k = w.nodes, w.n, w.k
    ae, enc, dec, _ = make_ae(B, w.ae_channels)
    gs = [synth.gradients(w, t, device="cuda") for t in range(2)]

    def make_state():
        return dict(u=torch.zeros((K, n), device="cuda"), v=torch.zeros((K, n), device="cuda"),
                    vals=torch.zeros((K, k), device="cuda"), idx=torch.zeros((K, k), device="cuda", dtype=torch.int32),
                    lat=torch.zeros((K, B.lgc_latent_len(ae, k)), device="cuda"), rec=torch.zeros((K, k), device="cuda"),
                    dense=torch.zeros((2, n), device="cuda"))

    def two_steps(ctx, s):
        for t in range(2):
            B.lgc_accumulate_topk(ctx, gs[t], s["u"], s["v"], w.momentum, k, s["vals"], s["idx"])
            B.lgc_encode(ctx, ae, s["vals"], s["lat"])
            B.lgc_decode(ctx, ae, s["lat"], s["rec"])
            B.lgc_scatter(ctx, s["rec"], s["idx"], 1.0 / K, s["dense"][t])

    ctx_e, ctx_g = B.Context(n, k, K), B.Context(n, k, K)
    eager, graphed = make_state(), make_state()
    two_steps(ctx_g, graphed)                 # warm-up outside the capture: grows the activation scratch
    for key in graphed:
        graphed[key].zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        two_steps(ctx_g, graphed)             # recorded, not run
    replays = 20
    for replay in range(replays):
        graph.replay()
        two_steps(ctx_e, eager)
        torch.cuda.synchronize()
        for key in eager:                     # u, v carry over from replay to replay; dense accumulates
            assert torch.equal(eager[key].view(torch.int32), graphed[key].view(torch.int32)), (replay, key)
    assert B.lgc_stats(ctx_g)[2] == 0 and B.lgc_stats(ctx_e)[2] == 0
    carried_e, carried_g = B.lgc_stats_carried(ctx_e), B.lgc_stats_carried(ctx_g)
    print(f"selections with a carried threshold: eager {carried_e}, replayed graph {carried_g}, of {2 * replays * K} each")
    assert carried_e > 0 and carried_g > 0, (carried_e, carried_g)   # the counts differ at most by what the warm-up's two records change
    # and the eager side agrees with the oracle on the last selection (so both do)
    hu = np.zeros((K, n), np.float32); hv = np.zeros((K, n), np.float32)
    ghs = [g.cpu().numpy() for g in gs]
    for rep in range(replays):
        for t in range(2):
            for b in (K - 1,):
                oracle.accumulate(ghs[t][b], hu[b], hv[b], w.momentum)
                ovals, oidx = oracle.topk(hv[b], hu[b], k)
    assert (graphed["idx"][K - 1].cpu().numpy().astype(np.uint32) == oidx).all() and same_bits(graphed["vals"][K - 1], ovals)
    ctx_e.close(); ctx_g.close(); ae.close()


def test_timing_of_the_streaming_launches(B):
    """LGC_OPT_PROFILE: the streaming launches of a call are timed by events that the launches stamp themselves;
    lgc_profile_read returns their summed duration and count and starts over."""
    n, k, K = 3_000_000, 3000, 2
    ctx = B.Context(n, k, K)
    g = torch.randn((K, n), device="cuda") * 1e-3
    u = torch.zeros((K, n), device="cuda"); v = torch.zeros((K, n), device="cuda")
    vals = torch.zeros((K, k), device="cuda"); idx = torch.zeros((K, k), device="cuda", dtype=torch.int32)
    B.lgc_accumulate_topk(ctx, g, u, v, 0.9, k, vals, idx)          # not timed: the option is off
    assert B.lgc_profile_read(ctx) == (0.0, 0)
    B.lgc_set_option(ctx, B.LGC_OPT_PROFILE, 1)
    B.lgc_accumulate(ctx, g, u, v, 0.9)
    B.lgc_topk(ctx, v, u, k, vals, idx)
    B.lgc_accumulate_topk(ctx, g, u, v, 0.9, k, vals, idx)
    ms, calls = B.lgc_profile_read(ctx)
    # 24 MB read and 48 MB read + written per pass: between a few microseconds and a few milliseconds in all
    assert calls == 3 and 0.005 < ms < 20.0, (ms, calls)
    assert B.lgc_profile_read(ctx) == (0.0, 0)
    B.lgc_set_option(ctx, B.LGC_OPT_PROFILE, 0)
    B.lgc_accumulate(ctx, g, u, v, 0.9)
    assert B.lgc_profile_read(ctx) == (0.0, 0)
    assert B.lgc_stats(ctx)[2] == 0
    ctx.close()
