"""ctypes front end of the CPU oracle (``mxo.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing in the GPU product path may import this package, and this package
imports nothing from the GPU package.

Every function here only marshals numpy arrays into ``libmxo.so``; the arithmetic lives in the
C file, which states the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mxo.c")
_LIB = os.path.join(_HERE, "libmxo.so")


def build(force: bool = False) -> str:
    """Compile ``mxo.c`` with gcc (plain C, -O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-Wall", "-Wextra", _SRC, "-o", _LIB + ".tmp", "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


class _CFormat(ctypes.Structure):
    _fields_ = [("ebits", ctypes.c_int32), ("mbits", ctypes.c_int32),
                ("block", ctypes.c_int32), ("scale_bits", ctypes.c_int32)]


@dataclass(frozen=True)
class Format:
    """Element format ExMy, block size B and scale format EsM0 (Method, parameter list)."""
    ebits: int
    mbits: int
    block: int = 32
    scale_bits: int = 8

    @property
    def bits(self) -> int:
        return 1 + self.ebits + self.mbits

    def c(self) -> _CFormat:
        return _CFormat(self.ebits, self.mbits, self.block, self.scale_bits)


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.mxo_code_value.restype = ctypes.c_double
        L.mxo_code_value.argtypes = [ctypes.POINTER(_CFormat), ctypes.c_uint]
        L.mxo_scale_value.restype = ctypes.c_double
        L.mxo_scale_value.argtypes = [ctypes.POINTER(_CFormat), ctypes.c_uint]
        L.mxo_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().mxo_num_threads())


def packed_sizes(fmt: Format, tokens: int, hidden: int):
    """(code_bytes, scale_bytes, effective_bits) — Model Evaluation / Table 1 / Table 3."""
    cb, sb, eb = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_double()
    f = fmt.c()
    _check(lib().mxo_packed_sizes(ctypes.byref(f), ctypes.c_int64(tokens), ctypes.c_int64(hidden),
                                  ctypes.byref(cb), ctypes.byref(sb), ctypes.byref(eb)),
           "packed_sizes")
    return cb.value, sb.value, eb.value


def code_value(fmt: Format, code: int) -> float:
    f = fmt.c()
    return float(lib().mxo_code_value(ctypes.byref(f), ctypes.c_uint(code)))


def scale_value(fmt: Format, code: int) -> float:
    f = fmt.c()
    return float(lib().mxo_scale_value(ctypes.byref(f), ctypes.c_uint(code)))


def quantize_bf16(fmt: Format, x_bits: np.ndarray):
    """x_bits: uint16 [T, H] bfloat16 bit patterns -> (codes uint8 [T, H], scales uint8 [T, H/B])."""
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    T, H = x_bits.shape
    codes = np.empty((T, H), dtype=np.uint8)
    scales = np.empty((T, H // fmt.block if fmt.block else 0), dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_quantize_bf16(ctypes.byref(f), _ptr(x_bits), ctypes.c_int64(T),
                                   ctypes.c_int64(H), _ptr(codes), _ptr(scales)), "quantize_bf16")
    return codes, scales


def quantize_f32(fmt: Format, x: np.ndarray):
    """x: float32 [T, H] -> (codes uint8 [T, H], scales uint8 [T, H/B])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, H = x.shape
    codes = np.empty((T, H), dtype=np.uint8)
    scales = np.empty((T, H // fmt.block), dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_quantize_f32(ctypes.byref(f), _ptr(x), ctypes.c_int64(T), ctypes.c_int64(H),
                                  _ptr(codes), _ptr(scales)), "quantize_f32")
    return codes, scales


def pack(fmt: Format, codes: np.ndarray) -> np.ndarray:
    """uint8 [T, H] one code per byte -> uint8 [T, H*b/8] bit stream."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    T, H = codes.shape
    out = np.empty((T, H * fmt.bits // 8), dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_pack(ctypes.byref(f), _ptr(codes), ctypes.c_int64(T), ctypes.c_int64(H),
                          _ptr(out)), "pack")
    return out


def unpack(fmt: Format, packed: np.ndarray, hidden: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    T = packed.shape[0]
    out = np.empty((T, hidden), dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_unpack(ctypes.byref(f), _ptr(packed), ctypes.c_int64(T),
                            ctypes.c_int64(hidden), _ptr(out)), "unpack")
    return out


def pack_scales(fmt: Format, scales: np.ndarray) -> np.ndarray:
    """uint8 scale codes (any shape, one per block, row-major) -> the flat array that travels:
    the same bytes for s = 8, an s-bit stream for s < 8."""
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    n = scales.size
    out = np.zeros((n * fmt.scale_bits + 7) // 8, dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_pack_scales(ctypes.byref(f), _ptr(scales), ctypes.c_int64(n), _ptr(out)),
           "pack_scales")
    return out


def unpack_scales(fmt: Format, packed: np.ndarray, nblocks: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    out = np.empty(nblocks, dtype=np.uint8)
    f = fmt.c()
    _check(lib().mxo_unpack_scales(ctypes.byref(f), _ptr(packed), ctypes.c_int64(nblocks),
                                   _ptr(out)), "unpack_scales")
    return out


def dequantize(fmt: Format, codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    T, H = codes.shape
    out = np.empty((T, H), dtype=np.float32)
    f = fmt.c()
    _check(lib().mxo_dequantize(ctypes.byref(f), _ptr(codes), _ptr(scales), ctypes.c_int64(T),
                                ctypes.c_int64(H), _ptr(out)), "dequantize")
    return out


def dequant_reduce(fmt: Format, codes_list, scales_list) -> np.ndarray:
    """Left fold, in list order, of the decoded ranks with binary32 adds (Profiling)."""
    tp = len(codes_list)
    cs = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    ss = [np.ascontiguousarray(s, dtype=np.uint8) for s in scales_list]
    T, H = cs[0].shape
    out = np.empty((T, H), dtype=np.float32)
    cp = (ctypes.c_void_p * tp)(*[c.ctypes.data for c in cs])
    sp = (ctypes.c_void_p * tp)(*[s.ctypes.data for s in ss])
    f = fmt.c()
    _check(lib().mxo_dequant_reduce(ctypes.byref(f), ctypes.c_int(tp), cp, sp, ctypes.c_int64(T),
                                    ctypes.c_int64(H), _ptr(out)), "dequant_reduce")
    return out


def dequant_reduce_own(fmt: Format, own_rank: int, own_bits: np.ndarray, codes_list,
                       scales_list) -> np.ndarray:
    """The same fold with rank ``own_rank`` contributing its raw bf16 partial (Profiling)."""
    tp = len(codes_list)
    own_bits = np.ascontiguousarray(own_bits, dtype=np.uint16)
    T, H = own_bits.shape
    cs = [None if c is None else np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    ss = [None if s is None else np.ascontiguousarray(s, dtype=np.uint8) for s in scales_list]
    out = np.empty((T, H), dtype=np.float32)
    cp = (ctypes.c_void_p * tp)(*[None if c is None else c.ctypes.data for c in cs])
    sp = (ctypes.c_void_p * tp)(*[None if s is None else s.ctypes.data for s in ss])
    f = fmt.c()
    _check(lib().mxo_dequant_reduce_own(ctypes.byref(f), ctypes.c_int(tp), ctypes.c_int(own_rank),
                                        _ptr(own_bits), cp, sp, ctypes.c_int64(T),
                                        ctypes.c_int64(H), _ptr(out)), "dequant_reduce_own")
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _check(lib().mxo_round_to_bf16(_ptr(x), ctypes.c_int64(x.size), _ptr(out)), "round_to_bf16")
    return out


def sum_bf16(parts) -> np.ndarray:
    """The uncompressed reduction: binary32 left fold, in list order, of bf16 partials given as
    uint16 bit patterns (Profiling)."""
    ps = [np.ascontiguousarray(p, dtype=np.uint16) for p in parts]
    out = np.empty(ps[0].shape, dtype=np.float32)
    pp = (ctypes.c_void_p * len(ps))(*[p.ctypes.data for p in ps])
    _check(lib().mxo_sum_bf16(ctypes.c_int(len(ps)), pp, ctypes.c_int64(ps[0].size), _ptr(out)),
           "sum_bf16")
    return out


def sqnr_db(ref: np.ndarray, test: np.ndarray) -> float:
    """Quality proxy: SQNR in dB of ``test`` against ``ref`` (stands in for Model Evaluation's
    perplexity increase)."""
    ref = np.ascontiguousarray(ref, dtype=np.float32)
    test = np.ascontiguousarray(test, dtype=np.float32)
    assert ref.shape == test.shape
    out = ctypes.c_double()
    _check(lib().mxo_sqnr_db(_ptr(ref), _ptr(test), ctypes.c_int64(ref.size), ctypes.byref(out)),
           "sqnr_db")
    return out.value
