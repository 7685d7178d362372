"""GPU parity of the parameter-server pattern's extra steps (Alg. 1, Sec. IV-C, Sec. V-B): the
innovation component (bit-exact) and the decoder that takes it as one more channel (1e-4 relative
L2), through the C ABI, against the CPU oracle; then Alg. 1 end to end."""
import numpy as np
import pytest
import torch

from paper_2103_08870_amd import synth
from test_gpu_parity import B, REL_L2_TOL, assert_close, dev, rel_l2, same_bits  # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


def random_layout(rng, n, n_seg):
    cuts = np.sort(rng.choice(np.arange(1, n), n_seg - 1, replace=False)) if n_seg > 1 else np.array([], int)
    return np.concatenate([[0], cuts, [n]]).astype(np.int64)


@pytest.mark.parametrize("k,n_seg,batch", [(1, 1, 1), (40, 1, 2), (2048, 30, 1), (25_532, 161, 4), (44_501, 314, 3),
                                           (300_000, 3, 1)])
def test_innovation(B, oracle, k, n_seg, batch):
    rng = np.random.default_rng(k + n_seg)
    off = random_layout(rng, k, n_seg)
    lens = np.diff(off)
    ks = np.maximum(1, lens // 10)                              # "top 10 %" of Alg. 1
    if n_seg >= 3:
        ks[1] = 0; ks[2] = lens[2]                              # nothing / everything kept
    ctx = B.Context(max(k, 16), max(k, 16), batch)
    seg = B.Segments(off.tolist(), ks.tolist())
    for trial in range(2):
        if trial == 0:
            vals = rng.laplace(0, 1e-2, (batch, k)).astype(np.float32)
        else:   # few distinct magnitudes: the cut falls inside a tie group in most layers
            vals = (rng.integers(-5, 6, (batch, k)) * 0.125).astype(np.float32)
        dvals = dev(vals)
        out = torch.full((batch, k), 7.0, device="cuda")
        B.lgc_innovation(ctx, seg, dvals, out)
        assert B.lgc_stats(ctx)[2] == 0
        assert same_bits(dvals, vals)                           # input untouched
        for b in range(batch):
            assert same_bits(out[b], oracle.innovation(vals[b], off, ks)), (trial, b)
    seg.close(); ctx.close()


def make_innovation_ae(B, channels, slope=0.0):
    enc, dec = synth.innovation_ae(channels)
    ew, eb, dw, db = synth.ae_weights(enc, dec, device="cuda")
    ae = B.Autoencoder(enc, dec, ew, eb, dw, db, slope=slope)
    host = [[t.cpu().numpy() for t in xs] for xs in (ew, eb, dw, db)]
    return ae, enc, dec, host


@pytest.mark.parametrize("channels,k,batch,slope", [((1, 8, 4), 1024, 1, 0.0), ((1, 8, 4), 25_532, 4, 0.0),
                                                    ((1, 16, 8), 44_501, 2, 0.01), ((1, 16, 8), 5, 2, 0.0),
                                                    # not one of the shapes with a kernel of their own: layer by layer
                                                    ((1, 6, 3), 777, 2, 0.01), ((1, 16, 8), 4099, 3, 0.2)])
def test_decode_with_innovation(B, oracle, channels, k, batch, slope):
    ae, enc, dec, (ew, eb, dw, db) = make_innovation_ae(B, channels, slope)
    ctx = B.Context(1 << 20, 1 << 20, 4)
    B.lgc_reserve(ctx, ae, k, batch)
    rng = np.random.default_rng(k)
    lat_len = B.lgc_latent_len(ae, k)
    latent = rng.standard_normal((batch, lat_len)).astype(np.float32)
    innov = np.where(rng.random((batch, k)) < 0.1, rng.laplace(0, 1e-2, (batch, k)), 0.0).astype(np.float32)
    rec = torch.zeros((batch, k), device="cuda")
    B.lgc_decode_innovation(ctx, ae, dev(latent), dev(innov), rec)
    for b in range(batch):
        ref = oracle.decode_with_innovation(latent[b].reshape(channels[-1], -1), innov[b], k, enc, dec, dw, db, slope)
        assert_close(rec[b], ref, what=("reconstruction", b))
    # the two decoders do not take each other's autoencoders
    with pytest.raises(B.LgcError):
        B.lgc_decode(ctx, ae, dev(latent), rec)
    plain_enc, plain_dec = synth.mirrored_ae(channels)
    pw = synth.ae_weights(plain_enc, plain_dec, device="cuda")
    plain = B.Autoencoder(plain_enc, plain_dec, *pw)
    with pytest.raises(B.LgcError):
        B.lgc_decode_innovation(ctx, plain, dev(latent), dev(innov), rec)
    plain.close(); ctx.close(); ae.close()


def test_parameter_server_iteration_per_layer(B, oracle):
    """Alg. 1 on every node: accumulate, per-layer top-k, per-layer innovation (top 10 % of each layer's
    selected values), encoder, decoder with the innovation channel; then the master's average (Sec. V-B)."""
    w = synth.workload(2, n=1_800_000, nodes=3)
    K, n = w.nodes, w.n
    off, ks = synth.layer_plan(w)
    mu = sum(ks)
    out_off = np.concatenate([[0], np.cumsum(ks)])
    inv_ks = [max(1, k_l // 10) for k_l in ks]
    ctx = B.Context(n, mu, K)
    seg = B.Segments(off, ks)
    inv_seg = B.Segments(out_off.tolist(), inv_ks)
    ae, enc, dec, (ew, eb, dw, db) = make_innovation_ae(B, w.ae_channels)
    B.lgc_reserve(ctx, ae, mu, K, seg)
    u = np.zeros((K, n), np.float32); v = np.zeros((K, n), np.float32)
    du, dv = dev(u), dev(v)
    vals = torch.zeros((K, mu), device="cuda"); idx = torch.zeros((K, mu), device="cuda", dtype=torch.int32)
    innov = torch.zeros((K, mu), device="cuda")
    lat = torch.zeros((K, B.lgc_latent_len(ae, mu)), device="cuda")
    rec = torch.zeros((K, mu), device="cuda")
    for t in range(3):
        g = synth.gradients(w, t, device="cpu").numpy()
        B.lgc_accumulate_topk_segmented(ctx, seg, dev(g), du, dv, w.momentum, vals, idx)
        B.lgc_innovation(ctx, inv_seg, vals, innov)
        B.lgc_encode(ctx, ae, vals, lat)
        B.lgc_decode_innovation(ctx, ae, lat, innov, rec)
        dense = torch.zeros(n, device="cuda")
        B.lgc_scatter(ctx, rec, idx, 1.0 / K, dense)
        assert B.lgc_stats(ctx)[2] == 0
        ref_dense = np.zeros(n, np.float32)
        rec_h = rec.cpu().numpy()
        for b in range(K):
            oracle.accumulate(g[b], u[b], v[b], w.momentum)
            ovals, oidx = oracle.topk_segmented(v[b], u[b], off, ks)
            assert (idx[b].cpu().numpy().astype(np.uint32) == oidx).all() and same_bits(vals[b], ovals)
            oinv = oracle.innovation(ovals, out_off, inv_ks)
            assert same_bits(innov[b], oinv)
            assert np.count_nonzero(oinv) <= sum(inv_ks)
            olat = oracle.encode(ovals, enc, ew, eb)
            assert_close(lat[b], olat, what=("latent", b))
            orec = oracle.decode_with_innovation(olat, oinv, mu, enc, dec, dw, db)
            assert_close(rec[b], orec, factor=2.0, what=("reconstruction", b))
            oracle.scatter(rec_h[b], oidx, 1.0 / K, ref_dense)      # exact on the library's own reconstruction
        assert same_bits(dv, v) and same_bits(du, u)
        assert same_bits(dense, ref_dense)
    inv_seg.close(); seg.close(); ctx.close(); ae.close()
