"""ctypes binding of liblgc.so: the same entry points as include/lgc.h, taking torch tensors.

Argument marshalling only: every step runs in the library's HIP kernels.  torch supplies
device memory (``Tensor.data_ptr()``) and the current HIP stream; nothing here computes.
There is no fall-back: if the library is missing or fails to load, import of the symbols
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblgc.so")

LGC_OK, LGC_EINVAL, LGC_ENOMEM, LGC_EHIP, LGC_EDEVICE = range(5)
LGC_OPT_SELECT_PATH, LGC_OPT_PROFILE, LGC_OPT_CARRY_THRESHOLD = 0, 1, 2

EXPORTS = [
    "lgc_create", "lgc_destroy", "lgc_last_error", "lgc_status_string",
    "lgc_accumulate", "lgc_topk", "lgc_accumulate_topk", "lgc_accumulate_topk_static",
    "lgc_ae_create", "lgc_ae_destroy", "lgc_latent_len", "lgc_encode", "lgc_decode",
    "lgc_scatter", "lgc_reserve", "lgc_set_option", "lgc_stats", "lgc_stats_carried", "lgc_profile_read",
    "lgc_gather", "lgc_accumulate_gather", "lgc_average",
    "lgc_segments_create", "lgc_segments_destroy", "lgc_segments_total_k",
    "lgc_topk_segmented", "lgc_accumulate_topk_segmented",
    "lgc_innovation", "lgc_decode_innovation",
]


class LgcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"liblgc status {status}: {message}")
        self.status = status


class _Layer(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32), ("ksize", C.c_int32), ("stride", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Loads liblgc.so (built in-tree by paper_2103_08870_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2103_08870_amd.build` "
                          "(there is no CPU fall-back)")
    l = C.CDLL(LIB_PATH)
    vp, u64, i32, f32 = C.c_void_p, C.c_uint64, C.c_int, C.c_float
    l.lgc_create.argtypes = [C.POINTER(vp), i32, u64, u64, i32]
    l.lgc_create.restype = i32
    l.lgc_destroy.argtypes = [vp]
    l.lgc_destroy.restype = None
    l.lgc_last_error.argtypes = [vp]
    l.lgc_last_error.restype = C.c_char_p
    l.lgc_status_string.argtypes = [i32]
    l.lgc_status_string.restype = C.c_char_p
    l.lgc_accumulate.argtypes = [vp, vp, vp, vp, u64, i32, u64, f32, vp]
    l.lgc_accumulate.restype = i32
    l.lgc_topk.argtypes = [vp, vp, vp, u64, i32, u64, u64, vp, vp, vp]
    l.lgc_topk.restype = i32
    l.lgc_accumulate_topk.argtypes = [vp, vp, vp, vp, u64, i32, u64, f32, u64, vp, vp, vp]
    l.lgc_accumulate_topk.restype = i32
    l.lgc_accumulate_topk_static.argtypes = [i32, vp, vp, vp, u64, i32, u64, f32, u64, vp, vp, vp]
    l.lgc_accumulate_topk_static.restype = i32
    l.lgc_ae_create.argtypes = [C.POINTER(vp), i32, i32, C.POINTER(_Layer), i32, C.POINTER(_Layer), f32,
                                C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    l.lgc_ae_create.restype = i32
    l.lgc_ae_destroy.argtypes = [vp]
    l.lgc_ae_destroy.restype = None
    l.lgc_latent_len.argtypes = [vp, u64]
    l.lgc_latent_len.restype = u64
    l.lgc_encode.argtypes = [vp, vp, vp, u64, i32, vp, vp]
    l.lgc_encode.restype = i32
    l.lgc_decode.argtypes = [vp, vp, vp, u64, i32, vp, vp]
    l.lgc_decode.restype = i32
    l.lgc_scatter.argtypes = [vp, vp, vp, u64, i32, f32, vp, u64, vp]
    l.lgc_scatter.restype = i32
    l.lgc_gather.argtypes = [vp, vp, vp, u64, i32, u64, vp, u64, vp, vp]
    l.lgc_gather.restype = i32
    l.lgc_accumulate_gather.argtypes = [vp, vp, vp, vp, u64, i32, u64, f32, vp, u64, vp, vp]
    l.lgc_accumulate_gather.restype = i32
    l.lgc_average.argtypes = [vp, vp, u64, i32, f32, vp, vp]
    l.lgc_average.restype = i32
    l.lgc_segments_create.argtypes = [C.POINTER(vp), i32, u64, u64, C.POINTER(u64), C.POINTER(u64)]
    l.lgc_segments_create.restype = i32
    l.lgc_segments_destroy.argtypes = [vp]
    l.lgc_segments_destroy.restype = None
    l.lgc_segments_total_k.argtypes = [vp]
    l.lgc_segments_total_k.restype = u64
    l.lgc_topk_segmented.argtypes = [vp, vp, vp, vp, i32, u64, vp, vp, vp]
    l.lgc_topk_segmented.restype = i32
    l.lgc_accumulate_topk_segmented.argtypes = [vp, vp, vp, vp, vp, i32, u64, f32, vp, vp, vp]
    l.lgc_accumulate_topk_segmented.restype = i32
    l.lgc_innovation.argtypes = [vp, vp, vp, i32, vp, vp]
    l.lgc_innovation.restype = i32
    l.lgc_decode_innovation.argtypes = [vp, vp, vp, vp, u64, i32, vp, vp]
    l.lgc_decode_innovation.restype = i32
    l.lgc_reserve.argtypes = [vp, vp, u64, i32, vp]
    l.lgc_reserve.restype = i32
    l.lgc_set_option.argtypes = [vp, i32, C.c_int64]
    l.lgc_set_option.restype = i32
    l.lgc_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)]
    l.lgc_stats.restype = i32
    l.lgc_stats_carried.argtypes = [vp, C.POINTER(u64)]
    l.lgc_stats_carried.restype = i32
    l.lgc_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u64)]
    l.lgc_profile_read.restype = i32
    _lib = l
    return l


def _check(status: int, ctx=None):
    if status != LGC_OK:
        msg = lib().lgc_last_error(ctx)
        raise LgcError(status, msg.decode() if msg else "")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("liblgc takes device tensors only")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _require(cond: bool, what: str) -> None:
    """Shape / layout precondition of a call: the C ABI sees raw pointers only, so a tensor that
    does not have the extent the call will touch must never reach it (also under ``python -O``)."""
    if not cond:
        raise ValueError(f"liblgc binding: {what}")


def _layout(t: torch.Tensor) -> Tuple[int, int, int]:
    """(n, batch, stride) of a [n] or [batch][n] tensor whose rows are contiguous."""
    if t.dim() == 1:
        _require(t.stride(0) == 1 or t.shape[0] <= 1, "1-D tensor must be contiguous")
        return t.shape[0], 1, t.shape[0]
    _require(t.dim() == 2 and (t.stride(1) == 1 or t.shape[1] <= 1), "expected [batch][n] with contiguous rows")
    return t.shape[1], t.shape[0], (t.stride(0) if t.shape[0] > 1 else t.shape[1])


# ------------------------------------------------------------------------------- handles

class Context:
    """lgc_ctx*: selection / autoencoder scratch on one device."""

    def __init__(self, max_n: int, max_k: int, max_batch: int = 1, device: int = 0):
        self.h = C.c_void_p()
        _check(lib().lgc_create(C.byref(self.h), device, max_n, max_k, max_batch))

    def close(self):
        if self.h:
            lib().lgc_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Autoencoder:
    """lgc_ae*: layer description plus a device copy of the weights."""

    def __init__(self, enc: Sequence[Tuple[int, int, int, int]], dec: Sequence[Tuple[int, int, int, int]],
                 enc_w, enc_b, dec_w, dec_b, slope: float = 0.0, device: int = 0):
        self.h = C.c_void_p()
        el = (_Layer * len(enc))(*[_Layer(*l) for l in enc])
        dl = (_Layer * len(dec))(*[_Layer(*l) for l in dec])
        keep = [t.contiguous() for t in list(enc_w) + list(enc_b) + list(dec_w) + list(dec_b)]
        ne, nd = len(enc), len(dec)

        def arr(ts):
            return (C.c_void_p * len(ts))(*[_ptr(t, torch.float32) for t in ts])

        _check(lib().lgc_ae_create(C.byref(self.h), device, ne, el, nd, dl, slope,
                                   arr(keep[:ne]), arr(keep[ne:2 * ne]),
                                   arr(keep[2 * ne:2 * ne + nd]), arr(keep[2 * ne + nd:])))

    def close(self):
        if self.h:
            lib().lgc_ae_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Segments:
    """lgc_segments*: the layers of the flat vector (offsets [n_seg+1]) and the values kept per layer."""

    def __init__(self, offsets: Sequence[int], ks: Sequence[int], device: int = 0):
        n_seg = len(ks)
        _require(len(offsets) == n_seg + 1, "len(offsets) == n_seg + 1")
        off = (C.c_uint64 * (n_seg + 1))(*[int(x) for x in offsets])
        kk = (C.c_uint64 * n_seg)(*[int(x) for x in ks])
        self.h = C.c_void_p()
        _check(lib().lgc_segments_create(C.byref(self.h), device, int(offsets[-1]), n_seg, off, kk), None)
        self.n = int(offsets[-1])
        self.total_k = int(lib().lgc_segments_total_k(self.h))

    def close(self):
        if getattr(self, "h", None):
            lib().lgc_segments_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------------------- entry points

def lgc_accumulate(ctx: Context, g: torch.Tensor, u: torch.Tensor, v: torch.Tensor, momentum: float) -> None:
    n, batch, stride = _layout(v)
    _require(_layout(g) == _layout(u) == (n, batch, stride), "_layout(g) == _layout(u) == (n, batch, stride)")
    _check(lib().lgc_accumulate(ctx.h, _ptr(g, torch.float32), _ptr(u, torch.float32), _ptr(v, torch.float32),
                                n, batch, stride, momentum, _stream()), ctx.h)


def lgc_topk(ctx: Context, v: torch.Tensor, u: Optional[torch.Tensor], k: int,
             out_vals: torch.Tensor, out_idx: torch.Tensor) -> None:
    n, batch, stride = _layout(v)
    _require(u is None or _layout(u) == (n, batch, stride), "u is None or _layout(u) == (n, batch, stride)")
    _require(out_vals.is_contiguous() and out_idx.is_contiguous() and out_vals.numel() == out_idx.numel() == batch * k, "out_vals.is_contiguous() and out_idx.is_contiguous() and out_vals.numel() == out_idx.numel() == batch * k")
    _check(lib().lgc_topk(ctx.h, _ptr(v, torch.float32), _ptr(u, torch.float32), n, batch, stride, k,
                          _ptr(out_vals, torch.float32), _ptr(out_idx, torch.int32), _stream()), ctx.h)


def lgc_accumulate_topk(ctx: Context, g: torch.Tensor, u: torch.Tensor, v: torch.Tensor, momentum: float, k: int,
                        out_vals: torch.Tensor, out_idx: torch.Tensor) -> None:
    n, batch, stride = _layout(v)
    _require(_layout(g) == _layout(u) == (n, batch, stride), "_layout(g) == _layout(u) == (n, batch, stride)")
    _require(out_vals.is_contiguous() and out_idx.is_contiguous() and out_vals.numel() == out_idx.numel() == batch * k, "out_vals.is_contiguous() and out_idx.is_contiguous() and out_vals.numel() == out_idx.numel() == batch * k")
    _check(lib().lgc_accumulate_topk(ctx.h, _ptr(g, torch.float32), _ptr(u, torch.float32), _ptr(v, torch.float32),
                                     n, batch, stride, momentum, k, _ptr(out_vals, torch.float32),
                                     _ptr(out_idx, torch.int32), _stream()), ctx.h)


def lgc_accumulate_topk_static(g: torch.Tensor, u: torch.Tensor, v: torch.Tensor, momentum: float, k: int,
                               out_vals: torch.Tensor, out_idx: torch.Tensor) -> None:
    """lgc_accumulate_topk without a context: the scratch is the library's fixed device array."""
    n, batch, stride = _layout(v)
    _require(_layout(g) == _layout(u) == (n, batch, stride), "g, u, v must share n, batch and row stride")
    _require(out_vals.is_contiguous() and out_idx.is_contiguous() and out_vals.numel() == out_idx.numel() == batch * k,
             "out_vals / out_idx must be contiguous with batch * k elements")
    _check(lib().lgc_accumulate_topk_static(v.device.index or 0, _ptr(g, torch.float32), _ptr(u, torch.float32),
                                            _ptr(v, torch.float32), n, batch, stride, momentum, k,
                                            _ptr(out_vals, torch.float32), _ptr(out_idx, torch.int32), _stream()), None)


def lgc_latent_len(ae: Autoencoder, k: int) -> int:
    return int(lib().lgc_latent_len(ae.h, k))


def lgc_encode(ctx: Context, ae: Autoencoder, vals: torch.Tensor, latent: torch.Tensor) -> None:
    """vals [batch][k] -> latent [batch][lgc_latent_len(ae, k)]."""
    _require(vals.dim() == 2 and vals.is_contiguous() and latent.is_contiguous(), "vals.dim() == 2 and vals.is_contiguous() and latent.is_contiguous()")
    batch, k = vals.shape
    _require(latent.numel() == batch * lgc_latent_len(ae, k), "latent.numel() == batch * lgc_latent_len(ae, k)")
    _check(lib().lgc_encode(ctx.h, ae.h, _ptr(vals, torch.float32), k, batch, _ptr(latent, torch.float32),
                            _stream()), ctx.h)


def lgc_decode(ctx: Context, ae: Autoencoder, latent: torch.Tensor, rec: torch.Tensor) -> None:
    """latent [batch][...] -> rec [batch][k]."""
    _require(rec.dim() == 2 and rec.is_contiguous() and latent.is_contiguous(), "rec.dim() == 2 and rec.is_contiguous() and latent.is_contiguous()")
    batch, k = rec.shape
    _require(latent.numel() == batch * lgc_latent_len(ae, k), "latent.numel() == batch * lgc_latent_len(ae, k)")
    _check(lib().lgc_decode(ctx.h, ae.h, _ptr(latent, torch.float32), k, batch, _ptr(rec, torch.float32),
                            _stream()), ctx.h)


def lgc_scatter(ctx: Context, vals: torch.Tensor, idx: torch.Tensor, scale: float, dense: torch.Tensor) -> None:
    """vals, idx [batch][k] (or [k]); dense [n], updated in place, nodes in order."""
    _require(vals.is_contiguous() and idx.is_contiguous() and dense.is_contiguous() and dense.dim() == 1, "vals.is_contiguous() and idx.is_contiguous() and dense.is_contiguous() and dense.dim() == 1")
    _require(vals.shape == idx.shape, "vals.shape == idx.shape")
    batch, k = (1, vals.shape[0]) if vals.dim() == 1 else vals.shape
    _check(lib().lgc_scatter(ctx.h, _ptr(vals, torch.float32), _ptr(idx, torch.int32), k, batch, scale,
                             _ptr(dense, torch.float32), dense.numel(), _stream()), ctx.h)


def lgc_topk_segmented(ctx: Context, seg: Segments, v: torch.Tensor, u: Optional[torch.Tensor],
                       out_vals: torch.Tensor, out_idx: torch.Tensor) -> None:
    n, batch, stride = _layout(v)
    _require(n == seg.n and (u is None or _layout(u) == (n, batch, stride)), "n == seg.n and (u is None or _layout(u) == (n, batch, stride))")
    _require(out_vals.is_contiguous() and out_idx.is_contiguous(), "out_vals.is_contiguous() and out_idx.is_contiguous()")
    _require(out_vals.numel() == out_idx.numel() == batch * seg.total_k, "out_vals.numel() == out_idx.numel() == batch * seg.total_k")
    _check(lib().lgc_topk_segmented(ctx.h, seg.h, _ptr(v, torch.float32), _ptr(u, torch.float32), batch, stride,
                                    _ptr(out_vals, torch.float32), _ptr(out_idx, torch.int32), _stream()), ctx.h)


def lgc_accumulate_topk_segmented(ctx: Context, seg: Segments, g: torch.Tensor, u: torch.Tensor, v: torch.Tensor,
                                  momentum: float, out_vals: torch.Tensor, out_idx: torch.Tensor) -> None:
    n, batch, stride = _layout(v)
    _require(n == seg.n and _layout(g) == _layout(u) == (n, batch, stride), "n == seg.n and _layout(g) == _layout(u) == (n, batch, stride)")
    _require(out_vals.is_contiguous() and out_idx.is_contiguous(), "out_vals.is_contiguous() and out_idx.is_contiguous()")
    _require(out_vals.numel() == out_idx.numel() == batch * seg.total_k, "out_vals.numel() == out_idx.numel() == batch * seg.total_k")
    _check(lib().lgc_accumulate_topk_segmented(ctx.h, seg.h, _ptr(g, torch.float32), _ptr(u, torch.float32),
                                               _ptr(v, torch.float32), batch, stride, momentum,
                                               _ptr(out_vals, torch.float32), _ptr(out_idx, torch.int32),
                                               _stream()), ctx.h)


def lgc_innovation(ctx: Context, seg: Segments, vals: torch.Tensor, out: torch.Tensor) -> None:
    """vals [batch][k] -> out [batch][k]: per segment of the plan the top-magnitude values, +0 elsewhere."""
    _require(vals.dim() == 2 and vals.is_contiguous() and out.is_contiguous() and out.shape == vals.shape, "vals.dim() == 2 and vals.is_contiguous() and out.is_contiguous() and out.shape == vals.shape")
    _require(vals.shape[1] == seg.n, "vals.shape[1] == seg.n")
    _check(lib().lgc_innovation(ctx.h, seg.h, _ptr(vals, torch.float32), vals.shape[0], _ptr(out, torch.float32),
                                _stream()), ctx.h)


def lgc_decode_innovation(ctx: Context, ae: Autoencoder, latent: torch.Tensor, innov: torch.Tensor,
                          rec: torch.Tensor) -> None:
    """latent [batch][...] and innovation component [batch][k] -> rec [batch][k]."""
    _require(rec.dim() == 2 and rec.is_contiguous() and latent.is_contiguous() and innov.is_contiguous(), "rec.dim() == 2 and rec.is_contiguous() and latent.is_contiguous() and innov.is_contiguous()")
    batch, k = rec.shape
    _require(innov.shape == rec.shape and latent.numel() == batch * lgc_latent_len(ae, k), "innov.shape == rec.shape and latent.numel() == batch * lgc_latent_len(ae, k)")
    _check(lib().lgc_decode_innovation(ctx.h, ae.h, _ptr(latent, torch.float32), _ptr(innov, torch.float32), k, batch,
                                       _ptr(rec, torch.float32), _stream()), ctx.h)


def lgc_gather(ctx: Context, v: torch.Tensor, u: Optional[torch.Tensor], idx: torch.Tensor,
               out_vals: torch.Tensor) -> None:
    """Values of every node at the shared positions idx [k]; v, u zeroed there.  out_vals [batch][k]."""
    n, batch, stride = _layout(v)
    _require(u is None or _layout(u) == (n, batch, stride), "u is None or _layout(u) == (n, batch, stride)")
    k = idx.numel()
    _require(idx.is_contiguous() and out_vals.is_contiguous() and out_vals.numel() == batch * k, "idx.is_contiguous() and out_vals.is_contiguous() and out_vals.numel() == batch * k")
    _check(lib().lgc_gather(ctx.h, _ptr(v, torch.float32), _ptr(u, torch.float32), n, batch, stride,
                            _ptr(idx, torch.int32), k, _ptr(out_vals, torch.float32), _stream()), ctx.h)


def lgc_accumulate_gather(ctx: Context, g: torch.Tensor, u: torch.Tensor, v: torch.Tensor, momentum: float,
                          idx: torch.Tensor, out_vals: torch.Tensor) -> None:
    n, batch, stride = _layout(v)
    _require(_layout(g) == _layout(u) == (n, batch, stride), "_layout(g) == _layout(u) == (n, batch, stride)")
    k = idx.numel()
    _require(idx.is_contiguous() and out_vals.is_contiguous() and out_vals.numel() == batch * k, "idx.is_contiguous() and out_vals.is_contiguous() and out_vals.numel() == batch * k")
    _check(lib().lgc_accumulate_gather(ctx.h, _ptr(g, torch.float32), _ptr(u, torch.float32), _ptr(v, torch.float32),
                                       n, batch, stride, momentum, _ptr(idx, torch.int32), k,
                                       _ptr(out_vals, torch.float32), _stream()), ctx.h)


def lgc_average(ctx: Context, x: torch.Tensor, scale: float, out: torch.Tensor) -> None:
    """x [batch][len] -> out [len]: sum over nodes, in order, of scale*x."""
    _require(x.dim() == 2 and x.is_contiguous() and out.is_contiguous() and out.numel() == x.shape[1], "x.dim() == 2 and x.is_contiguous() and out.is_contiguous() and out.numel() == x.shape[1]")
    _check(lib().lgc_average(ctx.h, _ptr(x, torch.float32), x.shape[1], x.shape[0], scale,
                             _ptr(out, torch.float32), _stream()), ctx.h)


def lgc_reserve(ctx: Context, ae: Optional[Autoencoder] = None, k: int = 0, batch: int = 1,
                seg: Optional[Segments] = None) -> None:
    """Reserves the context's activation scratch for (ae, k, batch) and / or the per-layer scratch for seg."""
    _check(lib().lgc_reserve(ctx.h, ae.h if ae is not None else None, k, batch,
                             seg.h if seg is not None else None), ctx.h)


def lgc_set_option(ctx: Context, opt: int, value: int) -> None:
    _check(lib().lgc_set_option(ctx.h, opt, value), ctx.h)


def lgc_stats(ctx: Context, check: bool = True) -> Tuple[int, int, int]:
    """(fast, fallback, errors) since the last call; synchronises the device."""
    a, b, c = C.c_uint64(), C.c_uint64(), C.c_uint64()
    st = lib().lgc_stats(ctx.h, C.byref(a), C.byref(b), C.byref(c))
    if check:
        _check(st, ctx.h)
    return a.value, b.value, c.value


def lgc_stats_carried(ctx: Context) -> int:
    """Selections since the last call whose candidate threshold was carried over instead of sampled; synchronises."""
    a = C.c_uint64()
    _check(lib().lgc_stats_carried(ctx.h, C.byref(a)), ctx.h)
    return a.value


def lgc_profile_read(ctx: Context) -> Tuple[float, int]:
    ms, cnt = C.c_double(), C.c_uint64()
    _check(lib().lgc_profile_read(ctx.h, C.byref(ms), C.byref(cnt)), ctx.h)
    return ms.value, cnt.value
