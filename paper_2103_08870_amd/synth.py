"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws random inputs (gradients, autoencoder weights).  It
holds none of the method's arithmetic and is the one place that both the CPU
oracle's tests and the GPU library's tests / benchmark take their inputs from,
so that both sides always see the same bytes.

The paper's workloads are real training gradients of ResNet50 / ResNet101 /
PSPNet (Sec. VI); those are not available, so synthetic gradients of the same
sizes stand in for them.  Their structure follows the paper's model of a
gradient as a common part plus a per-node innovation (Sec. IV-A,
g_k = g_cp + g_I) and its per-layer layout (Sec. V: one vector per layer, here
"segments" with their own scale).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

import torch

SEED_BASE = 20210308

Layer = Tuple[int, int, int, int]  # (c_in, c_out, ksize, stride)


def mirrored_ae(channels: Sequence[int]) -> Tuple[List[Layer], List[Layer]]:
    """Encoder 1 -> c1 -> ... (kernel 3, stride 2 each) and the mirrored
    transposed decoder."""
    enc = [(channels[i], channels[i + 1], 3, 2) for i in range(len(channels) - 1)]
    rev = list(channels)[::-1]
    dec = [(rev[i], rev[i + 1], 3, 2) for i in range(len(rev) - 1)]
    return enc, dec


def innovation_ae(channels: Sequence[int]) -> Tuple[List[Layer], List[Layer]]:
    """Autoencoder of the parameter-server pattern (Sec. IV-C) at the benchmark's encoder shape:
    the mirrored transposed layers bring the latent back to length k with channels[1] // 2
    channels, then the innovation component joins as one more channel and a final kernel-1,
    stride-1 layer maps them to the one output channel (the structure of Table II's last rows)."""
    enc = [(channels[i], channels[i + 1], 3, 2) for i in range(len(channels) - 1)]
    rev = list(channels)[::-1]
    mid = max(1, channels[1] // 2)
    dec = [(rev[i], rev[i + 1], 3, 2) for i in range(len(rev) - 2)]
    dec.append((rev[-2], mid, 3, 2))
    dec.append((mid + 1, 1, 1, 1))
    return enc, dec


def paper_ae() -> Tuple[List[Layer], List[Layer]]:
    """Layer shapes of Table I (encoder) and Table II (decoder).  Table II lists
    five stride-2 transposed layers against four stride-2 encoder layers, which
    cannot restore the input length; its first transposed layer is taken with
    stride 1."""
    enc = [(1, 64, 3, 2), (64, 128, 3, 2), (128, 256, 3, 2), (256, 64, 3, 2), (64, 4, 1, 1)]
    dec = [(4, 4, 3, 1), (4, 32, 3, 2), (32, 64, 3, 2), (64, 128, 3, 2), (128, 32, 3, 2),
           (32, 1, 1, 1)]
    return enc, dec


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int                      # 1..5
    nodes: int                    # K simulated nodes
    n: int                        # elements per node
    ks: Tuple[int, ...]           # selected per node (one entry per ratio)
    momentum: float
    ae_channels: Tuple[int, ...]
    iters: int
    kind: str                     # "normal" | "laplace_segments" | "mixture_ties"
    segments: int = 0
    innovation_weight: float = 0.0
    ratios: Tuple[float, ...] = ()

    @property
    def k(self) -> int:
        return self.ks[-1]


_FULL = {
    1: Workload("tiny", 1, 1, 1 << 20, (1024,), 0.9, (1, 8, 4), 3, "normal"),
    2: Workload("resnet50", 2, 4, 25_600_000, (25_600,), 0.9, (1, 8, 4), 10, "laplace_segments",
                segments=161, innovation_weight=0.3, ratios=(0.001,)),
    3: Workload("resnet101", 3, 8, 44_500_000, (44_500,), 0.9, (1, 16, 8), 10, "laplace_segments",
                segments=314, innovation_weight=0.3, ratios=(0.001,)),
    4: Workload("pspnet", 4, 8, 67_000_000, (6_700, 67_000), 0.9, (1, 16, 8), 10,
                "laplace_segments", segments=400, innovation_weight=0.5, ratios=(0.0001, 0.001)),
    5: Workload("stress", 5, 1, 1 << 28, (268_435, 2_684_354), 0.9, (1, 16, 8), 3, "mixture_ties",
                ratios=(0.001, 0.01)),
}


def workload(cfg: int, n: Optional[int] = None, nodes: Optional[int] = None) -> Workload:
    """Workload `cfg` (1..5).  `n` / `nodes` shrink it for tests while keeping
    its structure; k follows the same ratios (floor)."""
    w = _FULL[cfg]
    if nodes is not None:
        w = replace(w, nodes=nodes)
    if n is not None and n != w.n:
        if w.ratios:
            ks = tuple(max(1, int(math.floor(r * n))) for r in w.ratios)
        else:
            ks = tuple(max(1, (k * n) // w.n) for k in w.ks)
        w = replace(w, n=n, ks=ks)
    return w


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def segment_layout(w: Workload) -> Tuple[torch.Tensor, torch.Tensor]:
    """(sizes[int64], scales b_s[float64]) of the Laplace segments, on CPU.
    Sizes are log-uniform weights normalised to n (at least 64 each, the last
    one absorbs the remainder); scales are log-uniform in [1e-5, 1e-2]."""
    gen = _gen("cpu", SEED_BASE + 1000 * w.cfg + 500)
    s = w.segments
    lw = torch.empty(s, dtype=torch.float64).uniform_(math.log(1e3), math.log(2.4e6), generator=gen)
    wts = torch.exp(lw)
    sizes = torch.clamp(torch.round(w.n * wts / wts.sum()), min=64).to(torch.int64)
    # last segment absorbs the remainder; if the floor of 64 overshoots, shrink the largest
    while int(sizes[:-1].sum()) + 64 > w.n:
        j = int(torch.argmax(sizes[:-1]))
        sizes[j] = max(64, int(sizes[j]) - (int(sizes[:-1].sum()) + 64 - w.n))
    sizes[-1] = w.n - int(sizes[:-1].sum())
    lb = torch.empty(s, dtype=torch.float64).uniform_(math.log(1e-5), math.log(1e-2), generator=gen)
    return sizes, torch.exp(lb)


def layer_plan(w: Workload, ratio: Optional[float] = None) -> Tuple[List[int], List[int]]:
    """The workload's layers as a segment plan for per-layer selection (Sec. V-A):
    (offsets [segments + 1], ks [segments]) with mu_l = max(1, floor(ratio * n_l))."""
    sizes, _ = segment_layout(w)
    r = w.ratios[-1] if ratio is None else ratio
    offsets = [0]
    for sz in sizes.tolist():
        offsets.append(offsets[-1] + int(sz))
    ks = [max(1, int(math.floor(r * int(sz)))) for sz in sizes.tolist()]
    return offsets, ks


def _laplace(shape, scale: torch.Tensor, gen: torch.Generator, device) -> torch.Tensor:
    u = torch.rand(shape, generator=gen, device=device, dtype=torch.float32) - 0.5
    return -scale * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))


def gradients(w: Workload, t: int, device="cpu", k_for_ties: Optional[Sequence[int]] = None) -> torch.Tensor:
    """Fresh gradients of iteration t for all nodes: fp32 tensor [nodes][n]."""
    gen = _gen(device, SEED_BASE + 1000 * w.cfg + t)
    if w.kind == "normal":
        return torch.randn((w.nodes, w.n), generator=gen, device=device, dtype=torch.float32) * 1e-3
    if w.kind == "laplace_segments":
        sizes, scales = segment_layout(w)
        b = torch.repeat_interleave(scales.to(torch.float32), sizes).to(device)
        c = _laplace((w.n,), b, gen, device)
        out = torch.empty((w.nodes, w.n), device=device, dtype=torch.float32)
        for i in range(w.nodes):
            e = _laplace((w.n,), b, gen, device)
            out[i] = c + w.innovation_weight * e
        return out
    if w.kind == "mixture_ties":
        out = torch.empty((w.nodes, w.n), device=device, dtype=torch.float32)
        ks = tuple(k_for_ties) if k_for_ties is not None else w.ks
        for i in range(w.nodes):
            z = torch.randn(w.n, generator=gen, device=device, dtype=torch.float32)
            big = torch.rand(w.n, generator=gen, device=device) < 0.001
            g = z * torch.where(big, 1e-1, 1e-4).to(torch.float32)
            del z, big
            # a quarter of the positions snap to one of 4096 log-spaced magnitudes in [1e-5, 1]
            snap = torch.rand(w.n, generator=gen, device=device) < 0.25
            levels = torch.logspace(-5.0, 0.0, 4096, device=device, dtype=torch.float32)
            mag = g.abs().clamp(min=1e-5, max=1.0)
            pos = torch.round((torch.log10(mag) + 5.0) * (4095.0 / 5.0)).to(torch.int64).clamp(0, 4095)
            g = torch.where(snap, torch.copysign(levels[pos], g), g)
            del snap, mag, pos
            # copies of the would-be k-th magnitude, spread over the whole index range,
            # so that the cut falls inside a group of equal magnitudes
            for k in ks:
                if 0 < k <= w.n:
                    kth = torch.topk(g.abs(), k, sorted=True).values[-1]
                    copies = min(64, w.n)
                    where = (torch.arange(copies, device=device, dtype=torch.int64) * (w.n // copies)
                             + torch.randint(0, max(1, w.n // copies), (copies,), generator=gen,
                                             device=device))
                    g[where] = torch.copysign(kth, g[where])
            out[i] = g
        return out
    raise ValueError(w.kind)


def ae_weights(enc: Sequence[Layer], dec: Sequence[Layer], device="cpu", seed: int = SEED_BASE + 7):
    """Weights and biases ~ U(+-1/sqrt(ksize*c_in)).  Returns
    (enc_w, enc_b, dec_w, dec_b): conv weights [c_out][c_in][ksize],
    transposed-conv weights [c_in][c_out][ksize]."""
    gen = _gen("cpu", seed)

    def uni(shape, bound):
        return ((torch.rand(shape, generator=gen, dtype=torch.float32) * 2.0 - 1.0) * bound).to(device)

    enc_w, enc_b, dec_w, dec_b = [], [], [], []
    for (ci, co, ks, _) in enc:
        bound = 1.0 / math.sqrt(ks * ci)
        enc_w.append(uni((co, ci, ks), bound))
        enc_b.append(uni((co,), bound))
    for (ci, co, ks, _) in dec:
        bound = 1.0 / math.sqrt(ks * ci)
        dec_w.append(uni((ci, co, ks), bound))
        dec_b.append(uni((co,), bound))
    return enc_w, enc_b, dec_w, dec_b
