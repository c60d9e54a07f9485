"""Argument marshalling for ``libmxc.so`` (same names as the C entry points in include/mxc.h).

Nothing is computed here: tensors are checked for device / dtype / contiguity, outputs are
allocated with torch, and raw device pointers plus the current HIP stream are handed to the
library.  There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmxc.so")

MXC_F32, MXC_BF16 = 0, 1


class MxcError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {lib().mxc_strerror(status).decode()} (status {status})")


class _CFormat(ctypes.Structure):
    _fields_ = [("ebits", ctypes.c_int32), ("mbits", ctypes.c_int32),
                ("block", ctypes.c_int32), ("scale_bits", ctypes.c_int32)]


@dataclass(frozen=True)
class Format:
    """Element format ExMy, block size and scale format EsM0."""
    ebits: int
    mbits: int
    block: int = 32
    scale_bits: int = 8

    @property
    def bits(self) -> int:
        return 1 + self.ebits + self.mbits

    def c(self) -> _CFormat:
        return _CFormat(self.ebits, self.mbits, self.block, self.scale_bits)


def int_format(bits: int, block: int = 32, scale_bits: int = 8) -> Format:
    """INT3 / INT4 / INT5 of the paper's parameter list: a symmetric sign-magnitude integer grid
    is the 1-bit-exponent float E1M(bits-2) (its ablation table prints identical results for the
    two), so the integer types are served by that format."""
    if bits not in (3, 4, 5, 6):
        raise ValueError("integer element types of 3 to 6 bits only")
    return Format(1, bits - 2, block, scale_bits)


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load the C-ABI library; builds it first if no built library is present."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        fp = ctypes.POINTER(_CFormat)
        szp = ctypes.POINTER(ctypes.c_size_t)
        L.mxc_strerror.restype = ctypes.c_char_p
        L.mxc_strerror.argtypes = [ci]
        L.mxc_version.restype = ctypes.c_char_p
        L.mxc_version.argtypes = []
        L.mxc_packed_sizes.restype = ci
        L.mxc_packed_sizes.argtypes = [fp, i64, i64, szp, szp]
        L.mxc_effective_bits.restype = ctypes.c_double
        L.mxc_effective_bits.argtypes = [fp]
        L.mxc_quantize.restype = ci
        L.mxc_quantize.argtypes = [fp, vp, i64, i64, vp, vp, vp]
        L.mxc_quantize_batched.restype = ci
        L.mxc_quantize_batched.argtypes = [fp, ci, ctypes.POINTER(vp), i64, i64,
                                           ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
        L.mxc_dequant_reduce.restype = ci
        L.mxc_dequant_reduce.argtypes = [fp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp), i64, i64,
                                         vp, ci, vp]
        L.mxc_requantize_chunk.restype = ci
        L.mxc_requantize_chunk.argtypes = [fp, vp, ci, i64, i64, ci, ci, vp, vp, vp]
        L.mxc_dequant_reduce_own.restype = ci
        L.mxc_dequant_reduce_own.argtypes = [fp, ci, ci, vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                             i64, i64, vp, ci, vp]
        L.mxc_dequant_reduce_requantize.restype = ci
        L.mxc_dequant_reduce_requantize.argtypes = [fp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                    i64, i64, vp, vp, vp]
        L.mxc_copy_probe.restype = ci
        L.mxc_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.mxc_time_next_launch.restype = ci
        L.mxc_time_next_launch.argtypes = [vp, vp]
        _lib = L
    return _lib


def version() -> str:
    return lib().mxc_version().decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise MxcError(status, what)


def _stream(stream) -> ctypes.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _p(t: torch.Tensor) -> int:
    """Device address of a tensor; every pointer handed to the library goes through here, after
    the shape and size checks."""
    if not t.is_cuda:
        raise ValueError("the library takes device tensors only, got one on " + str(t.device))
    return t.data_ptr()


def _dev(t: torch.Tensor, dtype, what: str) -> torch.Tensor:
    if t.dtype != dtype:
        raise ValueError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _sized(t: torch.Tensor, dtype, nbytes: int, what: str) -> torch.Tensor:
    """A device tensor of ``dtype``, contiguous, holding exactly ``nbytes`` bytes: the library
    takes raw pointers, so this is the only place a short or misshapen buffer can be caught
    before a kernel reads or writes past it."""
    if t.dtype != dtype:
        raise ValueError(f"{what} must be {dtype}, got {t.dtype}")
    have = t.numel() * t.element_size()
    if have != nbytes:
        raise ValueError(f"{what} holds {have} bytes, the call needs {nbytes}")
    return _dev(t, dtype, what)


def _packed_ok(fmt: "Format", tokens: int, hidden: int, codes, scales, what: str = "") -> None:
    """Every (codes, scales) pair has the packed sizes of a [tokens, hidden] tensor."""
    cb, sb = packed_sizes(fmt, tokens, hidden)
    for c, s_ in zip(codes, scales):
        _sized(c, torch.uint8, cb, what + "codes")
        _sized(s_, torch.uint8, sb, what + "scales")


def _ptrs(ts: Sequence[torch.Tensor]):
    return (ctypes.c_void_p * len(ts))(*[_p(t) for t in ts])


def packed_sizes(fmt: Format, tokens: int, hidden: int) -> Tuple[int, int]:
    cb, sb = ctypes.c_size_t(), ctypes.c_size_t()
    f = fmt.c()
    _check(lib().mxc_packed_sizes(ctypes.byref(f), tokens, hidden, ctypes.byref(cb),
                                  ctypes.byref(sb)), "mxc_packed_sizes")
    return cb.value, sb.value


def effective_bits(fmt: Format) -> float:
    f = fmt.c()
    v = lib().mxc_effective_bits(ctypes.byref(f))
    if v < 0:
        raise MxcError(-2, "mxc_effective_bits")
    return v


def _alloc_packed(fmt: Format, tokens: int, hidden: int, device):
    """codes uint8 [tokens, hidden*b/8]; scales uint8 [tokens, hidden/block] for 8-bit scales,
    a flat bit-stream array for narrower ones."""
    cb, sb = packed_sizes(fmt, tokens, hidden)
    codes = torch.empty((tokens, cb // tokens if tokens else 0), dtype=torch.uint8, device=device)
    if fmt.scale_bits == 8:
        scales = torch.empty((tokens, sb // tokens if tokens else 0), dtype=torch.uint8, device=device)
    else:
        scales = torch.empty((sb,), dtype=torch.uint8, device=device)
    return codes, scales


def quantize(fmt: Format, x: torch.Tensor, codes: Optional[torch.Tensor] = None,
             scales: Optional[torch.Tensor] = None, stream=None):
    """bf16 [tokens, hidden] -> (packed codes uint8 [tokens, hidden*b/8], scales uint8
    [tokens, hidden/block])."""
    _dev(x, torch.bfloat16, "x")
    tokens, hidden = x.shape
    if codes is None or scales is None:
        codes, scales = _alloc_packed(fmt, tokens, hidden, x.device)
    _packed_ok(fmt, tokens, hidden, [codes], [scales])
    f = fmt.c()
    _check(lib().mxc_quantize(ctypes.byref(f), _p(x), tokens, hidden, _p(codes),
                              _p(scales), _stream(stream)), "mxc_quantize")
    return codes, scales


def _same_shape(xs: Sequence[torch.Tensor]) -> Tuple[int, int]:
    """bf16 device tensors that all have the shape of the first, which is returned."""
    if len(xs) == 0:
        raise ValueError("no tensors given")
    for x in xs:
        if x.dim() != 2 or x.shape != xs[0].shape:
            raise ValueError(f"all partials must have one 2-D shape, got {tuple(x.shape)} and "
                             f"{tuple(xs[0].shape)}")
    for x in xs:
        _dev(x, torch.bfloat16, "x")
    return int(xs[0].shape[0]), int(xs[0].shape[1])


def _lists_match(*lists) -> None:
    if len({len(l) for l in lists}) != 1:
        raise ValueError("the tensor lists of one call must have the same length")


def quantize_batched(fmt: Format, xs: Sequence[torch.Tensor],
                     codes: Optional[List[torch.Tensor]] = None,
                     scales: Optional[List[torch.Tensor]] = None, stream=None):
    """The same for several partials of one shape in a single launch."""
    tokens, hidden = _same_shape(xs)
    if codes is None or scales is None:
        pairs = [_alloc_packed(fmt, tokens, hidden, xs[0].device) for _ in xs]
        codes, scales = [p[0] for p in pairs], [p[1] for p in pairs]
    _lists_match(xs, codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    f = fmt.c()
    _check(lib().mxc_quantize_batched(ctypes.byref(f), len(xs), _ptrs(xs), tokens, hidden,
                                      _ptrs(codes), _ptrs(scales), _stream(stream)),
           "mxc_quantize_batched")
    return codes, scales


def _out_dtype(out: torch.Tensor, tokens: int, hidden: int) -> int:
    """Checks a reduction's output tensor and returns its mxc_dtype."""
    if out.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("out must be float32 or bfloat16")
    _sized(out, out.dtype, tokens * hidden * out.element_size(), "out")
    return MXC_F32 if out.dtype == torch.float32 else MXC_BF16


def dequant_reduce(fmt: Format, codes: Sequence[torch.Tensor], scales: Sequence[torch.Tensor],
                   tokens: int, hidden: int, out: Optional[torch.Tensor] = None,
                   out_dtype=torch.float32, stream=None) -> torch.Tensor:
    """Decode the partials and add them in list order with float32 adds."""
    _lists_match(codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    if out is None:
        out = torch.empty((tokens, hidden), dtype=out_dtype, device=codes[0].device)
    dt = _out_dtype(out, tokens, hidden)
    f = fmt.c()
    _check(lib().mxc_dequant_reduce(ctypes.byref(f), len(codes), _ptrs(codes), _ptrs(scales),
                                    tokens, hidden, _p(out), dt, _stream(stream)),
           "mxc_dequant_reduce")
    return out


def requantize_chunk(fmt: Format, reduced: torch.Tensor, tp: int, chunk: int,
                     codes: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
                     stream=None):
    """Quantize rows [chunk*tokens/tp, (chunk+1)*tokens/tp) of the reduced tensor."""
    if reduced.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("reduced must be float32 or bfloat16")
    _dev(reduced, reduced.dtype, "reduced")
    tokens, hidden = reduced.shape
    dt = MXC_F32 if reduced.dtype == torch.float32 else MXC_BF16
    if tp < 1 or tokens % tp:
        raise ValueError("tokens must be a multiple of tp")
    if codes is None or scales is None:
        codes, scales = _alloc_packed(fmt, tokens // tp, hidden, reduced.device)
    _packed_ok(fmt, tokens // tp, hidden, [codes], [scales])
    f = fmt.c()
    _check(lib().mxc_requantize_chunk(ctypes.byref(f), _p(reduced), dt, tokens, hidden, tp,
                                      chunk, _p(codes), _p(scales),
                                      _stream(stream)), "mxc_requantize_chunk")
    return codes, scales


def dequant_reduce_own(fmt: Format, own_rank: int, own_x: torch.Tensor,
                       codes: Sequence[Optional[torch.Tensor]],
                       scales: Sequence[Optional[torch.Tensor]], out: Optional[torch.Tensor] = None,
                       out_dtype=torch.float32, stream=None) -> torch.Tensor:
    """Reduction with rank ``own_rank`` contributing its uncompressed bf16 partial ``own_x``;
    ``codes[own_rank]`` / ``scales[own_rank]`` may be None."""
    _dev(own_x, torch.bfloat16, "own_x")
    tokens, hidden = own_x.shape
    _lists_match(codes, scales)
    others = [r for r in range(len(codes)) if r != own_rank]
    _packed_ok(fmt, tokens, hidden, [codes[r] for r in others], [scales[r] for r in others])
    if out is None:
        out = torch.empty((tokens, hidden), dtype=out_dtype, device=own_x.device)
    dt = _out_dtype(out, tokens, hidden)
    cp = (ctypes.c_void_p * len(codes))(*[None if c is None else _p(c) for c in codes])
    sp = (ctypes.c_void_p * len(codes))(*[None if s_ is None else _p(s_) for s_ in scales])
    f = fmt.c()
    _check(lib().mxc_dequant_reduce_own(ctypes.byref(f), len(codes), own_rank, _p(own_x),
                                        cp, sp, tokens, hidden, _p(out), dt,
                                        _stream(stream)), "mxc_dequant_reduce_own")
    return out


def dequant_reduce_requantize(fmt: Format, codes: Sequence[torch.Tensor],
                              scales: Sequence[torch.Tensor], tokens: int, hidden: int,
                              codes_out: Optional[torch.Tensor] = None,
                              scales_out: Optional[torch.Tensor] = None, stream=None):
    """Fused dequant-reduce + requantize of a row chunk: the tp compressed copies of a
    [tokens, hidden] chunk in, the packed arrays of the re-quantized sum out."""
    _lists_match(codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    if codes_out is None or scales_out is None:
        codes_out, scales_out = _alloc_packed(fmt, tokens, hidden, codes[0].device)
    _packed_ok(fmt, tokens, hidden, [codes_out], [scales_out], "output ")
    f = fmt.c()
    _check(lib().mxc_dequant_reduce_requantize(ctypes.byref(f), len(codes), _ptrs(codes),
                                               _ptrs(scales), tokens, hidden,
                                               _p(codes_out), _p(scales_out),
                                               _stream(stream)), "mxc_dequant_reduce_requantize")
    return codes_out, scales_out


class Launch:
    """A library call with its arguments already marshalled: for loops that issue the same call
    on the same buffers many times (serving loops, benchmarks).  Calling it enqueues the kernel
    on ``stream`` (default: torch's current stream at call time).  It keeps the tensors alive."""

    __slots__ = ("_fn", "_args", "_keep", "_what")

    def __init__(self, fn, args, keep, what):
        self._fn, self._args, self._keep, self._what = fn, args, keep, what

    def __call__(self, stream=None) -> None:
        s = stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream
        rc = self._fn(*self._args, s)
        if rc != 0:
            raise MxcError(rc, self._what)


def prepare_quantize_batched(fmt: Format, xs: Sequence[torch.Tensor],
                             codes: Sequence[torch.Tensor], scales: Sequence[torch.Tensor]) -> Launch:
    tokens, hidden = _same_shape(xs)
    _lists_match(xs, codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    f = fmt.c()
    args = (ctypes.byref(f), len(xs), _ptrs(xs), tokens, hidden, _ptrs(codes), _ptrs(scales))
    return Launch(lib().mxc_quantize_batched, args, (f, list(xs), list(codes), list(scales)),
                  "mxc_quantize_batched")


def prepare_dequant_reduce(fmt: Format, codes: Sequence[torch.Tensor],
                           scales: Sequence[torch.Tensor], tokens: int, hidden: int,
                           out: torch.Tensor) -> Launch:
    _lists_match(codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    dt = _out_dtype(out, tokens, hidden)
    f = fmt.c()
    args = (ctypes.byref(f), len(codes), _ptrs(codes), _ptrs(scales), tokens, hidden,
            _p(out), dt)
    return Launch(lib().mxc_dequant_reduce, args, (f, list(codes), list(scales), out),
                  "mxc_dequant_reduce")


def prepare_dequant_reduce_requantize(fmt: Format, codes: Sequence[torch.Tensor],
                                      scales: Sequence[torch.Tensor], tokens: int, hidden: int,
                                      codes_out: torch.Tensor, scales_out: torch.Tensor) -> Launch:
    _lists_match(codes, scales)
    _packed_ok(fmt, tokens, hidden, codes, scales)
    _packed_ok(fmt, tokens, hidden, [codes_out], [scales_out], "output ")
    f = fmt.c()
    args = (ctypes.byref(f), len(codes), _ptrs(codes), _ptrs(scales), tokens, hidden,
            _p(codes_out), _p(scales_out))
    return Launch(lib().mxc_dequant_reduce_requantize, args,
                  (f, list(codes), list(scales), codes_out, scales_out),
                  "mxc_dequant_reduce_requantize")


def prepare_requantize_chunk(fmt: Format, reduced: torch.Tensor, tp: int, chunk: int,
                             codes: torch.Tensor, scales: torch.Tensor) -> Launch:
    if reduced.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("reduced must be float32 or bfloat16")
    _dev(reduced, reduced.dtype, "reduced")
    tokens, hidden = reduced.shape
    dt = MXC_F32 if reduced.dtype == torch.float32 else MXC_BF16
    if tp < 1 or tokens % tp:
        raise ValueError("tokens must be a multiple of tp")
    _packed_ok(fmt, tokens // tp, hidden, [codes], [scales])
    f = fmt.c()
    args = (ctypes.byref(f), _p(reduced), dt, tokens, hidden, tp, chunk,
            _p(codes), _p(scales))
    return Launch(lib().mxc_requantize_chunk, args, (f, reduced, codes, scales),
                  "mxc_requantize_chunk")


def copy_probe(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    _dev(src, src.dtype, "src")
    nbytes = src.numel() * src.element_size()
    _sized(dst, dst.dtype, nbytes, "dst")
    _check(lib().mxc_copy_probe(_p(dst), _p(src), nbytes, _stream(stream)),
           "mxc_copy_probe")


def _event_handle(ev) -> ctypes.c_void_p:
    if ev is None:
        return ctypes.c_void_p(None)
    if not ev.cuda_event:
        ev.record()             # torch creates the HIP event on its first record
    return ctypes.c_void_p(ev.cuda_event)


def time_next_launch(start, stop) -> None:
    """Arm two ``torch.cuda.Event(enable_timing=True)`` (or None) for the next kernel this thread
    launches through the library: ``start.elapsed_time(stop)`` is then that kernel's own duration
    (mxc_time_next_launch).  Synchronise before reading the events."""
    _check(lib().mxc_time_next_launch(_event_handle(start), _event_handle(stop)),
           "mxc_time_next_launch")
