"""End-to-end pin of the oracle over a carried run (Alg. 1 / Alg. 2, the loop over iterations: the residual
g_acc of one iteration is the accumulator of the next): at EVERY iteration of a 10-iteration run what is sent and
what is kept partition the accumulated gradient exactly.  The check is made by selection, not by addition
(-0 + +0 would give +0 and raise a false alarm): at a selected position the sent value has the accumulated
value's bits and the residual is +0; at any other position the residual has the accumulated value's bits and
nothing was placed.  CPU only."""
import numpy as np
import pytest

from paper_2103_08870_amd import synth


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


@pytest.mark.parametrize("cfg,n,ratio_index,momentum", [(4, 60_000, 0, 0.9), (4, 60_000, 1, 0.9), (2, 41_003, 0, 0.0),
                                                         (5, 1 << 16, 1, 0.9)])
def test_sent_plus_kept_is_the_accumulated_gradient_at_every_iteration(oracle, cfg, n, ratio_index, momentum):
    w = synth.workload(cfg, n=n, nodes=2)
    k = w.ks[ratio_index]
    u = np.zeros((w.nodes, n), np.float32)
    v = np.zeros((w.nodes, n), np.float32)
    sent_total = 0
    for t in range(10):
        g = synth.gradients(w, t, k_for_ties=(k,)).numpy()
        if t == 3:
            g[0, 5] = -0.0; v[0, 5] = -0.0; u[0, 5] = -0.0     # a negative zero that stays unselected
        for b in range(w.nodes):
            u_before, v_before = u[b].copy(), v[b].copy()
            oracle.accumulate(g[b], u[b], v[b], momentum)
            v_acc, u_acc = v[b].copy(), u[b].copy()
            if momentum == 0.0:
                # Alg. 1 / Alg. 2 as printed: g_l = grad + g_acc (the momentum buffer is the fresh gradient)
                assert (bits(v_acc) == bits((v_before + g[b]).astype(np.float32))).all()
            vals, idx = oracle.topk(v[b], u[b], k)
            sel = np.zeros(n, bool)
            sel[idx] = True
            assert sel.sum() == k and (np.diff(idx.astype(np.int64)) > 0).all()
            # the partition, by selection
            assert (bits(vals) == bits(v_acc)[idx]).all()
            assert (bits(v[b])[sel] == 0).all() and (bits(u[b])[sel] == 0).all()
            assert (bits(v[b])[~sel] == bits(v_acc)[~sel]).all()
            assert (bits(u[b])[~sel] == bits(u_acc)[~sel]).all()
            # placed back at scale 1 (scatter into zeros) and added to the residual it gives the accumulated
            # gradient again: equal as numbers everywhere, equal in bits wherever the value is not a zero
            dense = np.zeros(n, np.float32)
            oracle.scatter(vals, idx, 1.0, dense)
            assert (bits(dense)[~sel] == 0).all()
            total = (dense + v[b]).astype(np.float32)
            assert (total == v_acc).all()
            nz = v_acc != 0
            assert (bits(total)[nz] == bits(v_acc)[nz]).all()
            sent_total += k
            if b == 0:
                idx0 = idx
        if t == 3:
            assert bits(v[0])[5] == 0x80000000 or 5 in idx0      # -0 + -0 = -0 survives where it was not sent
    assert sent_total == 10 * w.nodes * k
