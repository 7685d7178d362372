"""ctypes front-end of the CPU oracle (``lgc_oracle.c``).

TEST INFRASTRUCTURE ONLY: the oracle is what the GPU library is checked
against.  Nothing in the product package may import this module; it is used by
the tests, by the smoke check and by the benchmark's ``cpu_baseline`` leg.
It imports nothing from the product package either.

All arrays are numpy, fp32 / uint32, C-contiguous.  State arrays (``u``, ``v``,
``dense``) are updated in place, like the paper's ``g_acc``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lgc_oracle.c")
_LIB = os.path.join(_HERE, "liblgc_oracle.so")

Layer = Tuple[int, int, int, int]  # (c_in, c_out, ksize, stride)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  FMA contraction is off so that each fp32
    operation rounds on its own."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = C.CDLL(_LIB)
        fp = C.POINTER(C.c_float)
        u32p = C.POINTER(C.c_uint32)
        ip = C.POINTER(C.c_int)
        lib.oracle_accumulate.argtypes = [fp, fp, fp, C.c_size_t, C.c_float]
        lib.oracle_accumulate.restype = None
        lib.oracle_topk.argtypes = [fp, fp, C.c_size_t, C.c_size_t, fp, u32p]
        lib.oracle_topk.restype = C.c_int
        lib.oracle_conv_len.argtypes = [C.c_size_t, C.c_int, C.c_int]
        lib.oracle_conv_len.restype = C.c_size_t
        lib.oracle_conv1d.argtypes = [fp, C.c_int, C.c_size_t, fp, fp, C.c_int, C.c_int, C.c_int,
                                      C.c_int, C.c_float, fp]
        lib.oracle_conv1d.restype = None
        lib.oracle_conv_transpose1d.argtypes = [fp, C.c_int, C.c_size_t, fp, fp, C.c_int, C.c_int,
                                                C.c_int, C.c_size_t, C.c_int, C.c_float, fp]
        lib.oracle_conv_transpose1d.restype = C.c_int
        lib.oracle_encode.argtypes = [fp, C.c_size_t, C.c_int, ip, ip, ip, C.POINTER(fp),
                                      C.POINTER(fp), C.c_float, fp]
        lib.oracle_encode.restype = C.c_size_t
        lib.oracle_decode.argtypes = [fp, C.c_size_t, C.c_int, ip, ip, ip,
                                      C.POINTER(C.c_size_t), C.POINTER(fp), C.POINTER(fp),
                                      C.c_float, fp]
        lib.oracle_decode.restype = C.c_int
        lib.oracle_scatter.argtypes = [fp, u32p, C.c_size_t, C.c_float, fp, C.c_size_t]
        lib.oracle_scatter.restype = C.c_int
        u64p = C.POINTER(C.c_uint64)
        lib.oracle_topk_segmented.argtypes = [fp, fp, C.c_size_t, C.c_size_t, u64p, u64p, fp, u32p]
        lib.oracle_topk_segmented.restype = C.c_int
        lib.oracle_gather.argtypes = [fp, fp, C.c_size_t, u32p, C.c_size_t, fp]
        lib.oracle_gather.restype = C.c_int
        lib.oracle_average.argtypes = [fp, C.c_size_t, C.c_size_t, C.c_float, fp]
        lib.oracle_average.restype = None
        lib.oracle_innovation.argtypes = [fp, C.c_size_t, C.c_size_t, u64p, u64p, fp]
        lib.oracle_innovation.restype = C.c_int
        _lib = lib
    return _lib


def _f(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"], (a.dtype, a.flags)
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _u(a: np.ndarray):
    assert a.dtype == np.uint32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


# --------------------------------------------------------------------------- a1
def accumulate(g: np.ndarray, u: np.ndarray, v: np.ndarray, momentum: float) -> None:
    """u <- m*u + g ; v <- v + u, in place (Alg. 1/2 first loop line with DGC's
    momentum correction, Sec. V-A)."""
    assert g.shape == u.shape == v.shape and g.ndim == 1
    _load().oracle_accumulate(_f(g), _f(u), _f(v), g.size, np.float32(momentum))


# --------------------------------------------------------------------------- a2
def topk(v: np.ndarray, u, k: int):
    """Exact top-k of |v| (ties: lower index first).  Returns (vals, idx) with
    idx ascending; zeroes v (and u, if given) at idx.  Alg. 1/2 threshold /
    mask / residual lines."""
    assert v.ndim == 1
    vals = np.zeros(k, dtype=np.float32)
    idx = np.zeros(k, dtype=np.uint32)
    rc = _load().oracle_topk(_f(v), _f(u) if u is not None else None, v.size, k, _f(vals), _u(idx))
    if rc != 0:
        raise ValueError("oracle_topk: bad arguments")
    return vals, idx


# ------------------------------------------------------------------------ a3/a4
def conv_len(l_in: int, ksize: int, stride: int) -> int:
    return int(_load().oracle_conv_len(l_in, ksize, stride))


def conv1d(x: np.ndarray, w: np.ndarray, b: np.ndarray, ksize: int, stride: int,
           apply_act: bool, slope: float = 0.0) -> np.ndarray:
    """x [c_in][L] -> [c_out][L_out]; w [c_out][c_in][ksize]."""
    c_in, l_in = x.shape
    c_out = w.shape[0]
    assert w.shape == (c_out, c_in, ksize) and b.shape == (c_out,)
    out = np.zeros((c_out, conv_len(l_in, ksize, stride)), dtype=np.float32)
    _load().oracle_conv1d(_f(x), c_in, l_in, _f(w), _f(b), c_out, ksize, stride,
                          int(apply_act), np.float32(slope), _f(out))
    return out


def conv_transpose1d(x: np.ndarray, w: np.ndarray, b: np.ndarray, ksize: int, stride: int,
                     l_out: int, apply_act: bool, slope: float = 0.0) -> np.ndarray:
    """x [c_in][L] -> [c_out][l_out]; w [c_in][c_out][ksize]."""
    c_in, l_in = x.shape
    c_out = w.shape[1]
    assert w.shape == (c_in, c_out, ksize) and b.shape == (c_out,)
    out = np.zeros((c_out, l_out), dtype=np.float32)
    rc = _load().oracle_conv_transpose1d(_f(x), c_in, l_in, _f(w), _f(b), c_out, ksize, stride,
                                         l_out, int(apply_act), np.float32(slope), _f(out))
    if rc != 0:
        raise MemoryError("oracle_conv_transpose1d: out of memory")
    return out


def encoder_lengths(k: int, enc: Sequence[Layer]) -> List[int]:
    """[k, L_1, ..., L_latent]: length per channel after each encoder layer."""
    lens = [k]
    for (_, _, ks, st) in enc:
        lens.append(conv_len(lens[-1], ks, st))
    return lens


def decoder_lengths(k: int, enc: Sequence[Layer], dec: Sequence[Layer]) -> List[int]:
    """Output length of each decoder layer.  A stride-1 layer keeps the length;
    the j-th strided decoder layer restores the length that the matching
    strided encoder layer (counted from the end) consumed, so the final length
    is k again."""
    lens = encoder_lengths(k, enc)
    consumed = [lens[i] for i, (_, _, _, st) in enumerate(enc) if st != 1]
    out, cur = [], lens[-1]
    for (_, _, _, st) in dec:
        if st != 1:
            cur = consumed.pop()
        out.append(cur)
    assert not consumed, "decoder must have as many strided layers as the encoder"
    return out


def _ptr_array(arrs):
    fp = C.POINTER(C.c_float)
    return (fp * len(arrs))(*[_f(a) for a in arrs])


def encode(x: np.ndarray, enc: Sequence[Layer], w: Sequence[np.ndarray], b: Sequence[np.ndarray],
           slope: float = 0.0) -> np.ndarray:
    """x [k] (one node's selected values) -> latent [C][L].  E_c of Sec. IV."""
    k = x.size
    lens = encoder_lengths(k, enc)
    chan = [enc[0][0]] + [l[1] for l in enc]
    latent = np.zeros((chan[-1], lens[-1]), dtype=np.float32)
    n = len(enc)
    rc = _load().oracle_encode(_f(x), k, n, (C.c_int * (n + 1))(*chan),
                               (C.c_int * n)(*[l[2] for l in enc]),
                               (C.c_int * n)(*[l[3] for l in enc]),
                               _ptr_array(w), _ptr_array(b), np.float32(slope), _f(latent))
    assert rc == lens[-1]
    return latent


def decode(latent: np.ndarray, k: int, enc: Sequence[Layer], dec: Sequence[Layer],
           w: Sequence[np.ndarray], b: Sequence[np.ndarray], slope: float = 0.0) -> np.ndarray:
    """latent [C][L] -> reconstruction [k].  D_c of Sec. IV."""
    out_len = decoder_lengths(k, enc, dec)
    chan = [dec[0][0]] + [l[1] for l in dec]
    assert latent.shape[0] == chan[0] and chan[-1] == 1
    rec = np.zeros(out_len[-1], dtype=np.float32)
    n = len(dec)
    rc = _load().oracle_decode(_f(latent), latent.shape[1], n, (C.c_int * (n + 1))(*chan),
                               (C.c_int * n)(*[l[2] for l in dec]),
                               (C.c_int * n)(*[l[3] for l in dec]),
                               (C.c_size_t * n)(*out_len),
                               _ptr_array(w), _ptr_array(b), np.float32(slope), _f(rec))
    assert rc == 0
    return rec


# --------------------------------------------------------------------------- a5
def scatter(vals: np.ndarray, idx: np.ndarray, scale: float, dense: np.ndarray) -> None:
    """dense[idx[j]] += scale*vals[j] in place (node average of Sec. V-B)."""
    rc = _load().oracle_scatter(_f(vals), _u(idx), vals.size, np.float32(scale), _f(dense), dense.size)
    if rc != 0:
        raise ValueError("oracle_scatter: index out of range")


# ------------------------------------------------------ per-layer selection
def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def topk_segmented(v: np.ndarray, u, offsets, ks):
    """Per-layer top-k (Sec. V-A; layer loop of Alg. 1 / Alg. 2): segment l =
    [offsets[l], offsets[l+1]) keeps ks[l] values; results concatenated in layer
    order, positions in the flat numbering.  Zeroes v (and u) where selected."""
    off, kk = _u64(offsets), _u64(ks)
    assert off.size == kk.size + 1
    total = int(kk.sum())
    vals = np.zeros(total, dtype=np.float32)
    idx = np.zeros(total, dtype=np.uint32)
    u64p = C.POINTER(C.c_uint64)
    rc = _load().oracle_topk_segmented(_f(v), _f(u) if u is not None else None, v.size, kk.size,
                                       off.ctypes.data_as(u64p), kk.ctypes.data_as(u64p), _f(vals), _u(idx))
    if rc != 0:
        raise ValueError("oracle_topk_segmented: bad arguments")
    return vals, idx


# --------------------------------------------------- ring-allreduce variant
def gather(v: np.ndarray, u, idx: np.ndarray) -> np.ndarray:
    """Values at positions another node selected (Sec. V-A, ring-allreduce); the
    positions leave the residual v and the momentum buffer u."""
    vals = np.zeros(idx.size, dtype=np.float32)
    rc = _load().oracle_gather(_f(v), _f(u) if u is not None else None, v.size, _u(idx), idx.size, _f(vals))
    if rc != 0:
        raise ValueError("oracle_gather: index out of range")
    return vals


def average(x: np.ndarray, scale: float) -> np.ndarray:
    """x [K][len] -> sum over nodes, in node order, of scale*x_k (Alg. 2: g^avg)."""
    assert x.ndim == 2
    out = np.zeros(x.shape[1], dtype=np.float32)
    _load().oracle_average(_f(x), x.shape[0], x.shape[1], np.float32(scale), _f(out))
    return out


# ------------------------------------------------ parameter server: innovation
def innovation(vals: np.ndarray, offsets, ks) -> np.ndarray:
    """g~^I of Alg. 1: per segment of g~ the ks[l] top-magnitude values, zeros elsewhere."""
    off, kk = _u64(offsets), _u64(ks)
    out = np.zeros(vals.size, dtype=np.float32)
    u64p = C.POINTER(C.c_uint64)
    rc = _load().oracle_innovation(_f(vals), vals.size, kk.size, off.ctypes.data_as(u64p),
                                   kk.ctypes.data_as(u64p), _f(out))
    if rc != 0:
        raise ValueError("oracle_innovation: bad arguments")
    return out


def decode_with_innovation(latent: np.ndarray, innov: np.ndarray, k: int, enc: Sequence[Layer],
                           dec: Sequence[Layer], w: Sequence[np.ndarray], b: Sequence[np.ndarray],
                           slope: float = 0.0) -> np.ndarray:
    """D_c(g^c, g~^I) of Sec. IV-C / Sec. V-B: all decoder layers but the last run as in
    decode(); their output (length k) gets the innovation vector as one more
    channel, appended last; the final stride-1 layer maps the C+1 channels to 1."""
    assert dec[-1][3] == 1 and dec[-1][0] == dec[-2][1] + 1 and dec[-1][1] == 1
    out_len = decoder_lengths(k, enc, dec)
    x = np.ascontiguousarray(latent, dtype=np.float32)
    l_in = x.shape[1]
    for (ci, co, ks, st), wl, bl, lo in zip(dec[:-1], w[:-1], b[:-1], out_len[:-1]):
        x = conv_transpose1d(x, wl, bl, ks, st, lo, True, slope)
    assert x.shape[1] == k == innov.size
    x = np.concatenate([x, innov.reshape(1, k).astype(np.float32)], axis=0)
    ci, co, ks, st = dec[-1]
    return conv_transpose1d(x, w[-1], b[-1], ks, st, k, False, slope)[0]
