"""The seeded generators give the stated shapes, are reproducible, and hold the structure the
workloads are described with.  CPU only, reduced sizes."""
import torch

from paper_2103_08870_amd import synth


def test_workload_table():
    assert synth.workload(2).n == 25_600_000 and synth.workload(2).k == 25_600 and synth.workload(2).nodes == 4
    assert synth.workload(3).ks == (44_500,) and synth.workload(4).ks == (6_700, 67_000)
    assert synth.workload(5).ks == (268_435, 2_684_354) and synth.workload(5).n == 1 << 28
    w = synth.workload(4, n=1_000_000)
    assert w.ks == (100, 1000)


def test_segments_cover_n():
    for cfg in (2, 3, 4):
        for n in (None, 300_000):
            w = synth.workload(cfg, n=n)
            sizes, scales = synth.segment_layout(w)
            assert sizes.numel() == w.segments and int(sizes.sum()) == w.n and int(sizes.min()) >= 64
            assert float(scales.min()) >= 1e-5 and float(scales.max()) <= 1e-2


def test_reproducible_and_correlated():
    w = synth.workload(2, n=400_000)
    a, b = synth.gradients(w, 3), synth.gradients(w, 3)
    assert torch.equal(a, b) and a.shape == (4, 400_000) and a.dtype == torch.float32
    assert not torch.equal(a, synth.gradients(w, 4))
    c = torch.corrcoef(a[:, :200_000].double())
    assert float(c[0, 1]) > 0.5                         # common part dominates the innovation


def test_stress_has_ties_at_the_cut():
    w = synth.workload(5, n=1 << 20)
    g = synth.gradients(w, 0)[0]
    for k in w.ks:
        kth = torch.topk(g.abs(), k).values[-1]
        assert int((g.abs() == kth).sum()) >= 60       # the cut falls inside a group of equals
    assert g.abs().unique().numel() < 0.9 * g.numel()


def test_ae_weights_bounds():
    enc, dec = synth.mirrored_ae((1, 16, 8))
    ew, eb, dw, db = synth.ae_weights(enc, dec)
    assert ew[1].shape == (8, 16, 3) and dw[0].shape == (8, 16, 3) and dw[1].shape == (16, 1, 3)
    assert float(ew[1].abs().max()) <= 1 / (48 ** 0.5) and db[1].shape == (1,)
