"""CPU-only checks of the C-ABI boundary: the library loads, exports every function the header
declares, and rejects bad arguments on the host before anything is enqueued."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2411_09510_amd as mxc
    return mxc.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mxc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxc_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported(L):
    names = declared_functions()
    assert {"mxc_quantize", "mxc_quantize_batched", "mxc_dequant_reduce", "mxc_requantize_chunk",
            "mxc_dequant_reduce_requantize", "mxc_dequant_reduce_own", "mxc_packed_sizes", "mxc_strerror", "mxc_copy_probe",
            "mxc_time_next_launch"} <= set(names)
    for n in names:
        assert getattr(L, n) is not None, n


def test_packed_sizes_and_effective_bits(L):
    import paper_2411_09510_amd as mxc
    assert mxc.packed_sizes(mxc.Format(2, 1, 32, 8), 4096, 8192) == (16 << 20, 1 << 20)
    assert mxc.packed_sizes(mxc.Format(2, 2, 32, 8), 4096, 8192) == (20 << 20, 1 << 20)
    assert mxc.packed_sizes(mxc.Format(3, 2, 16, 8), 4096, 8192) == (24 << 20, 2 << 20)
    assert mxc.packed_sizes(mxc.Format(2, 1, 32, 8), 0, 8192) == (0, 0)
    assert mxc.packed_sizes(mxc.Format(2, 1, 8, 5), 64, 4096) == (64 * 4096 // 2, 64 * 512 * 5 // 8)
    assert mxc.packed_sizes(mxc.Format(2, 1, 8, 5), 1, 24) == (12, 2)    # 3 blocks, 15 bits -> 2 bytes
    assert mxc.effective_bits(mxc.Format(2, 1, 32, 8)) == 4.25          # Table 3 caption
    assert mxc.effective_bits(mxc.Format(2, 1, 8, 5)) == 4.625          # Table 1 prints 4.6
    with pytest.raises(mxc.MxcError):
        mxc.packed_sizes(mxc.Format(2, 1, 32, 8), 4, 48)                # hidden % block
    with pytest.raises(mxc.MxcError):
        mxc.packed_sizes(mxc.Format(4, 1, 32, 8), 4, 64)
    with pytest.raises(mxc.MxcError):
        mxc.packed_sizes(mxc.Format(2, 1, 24, 8), 4, 48)
    with pytest.raises(mxc.MxcError):
        mxc.packed_sizes(mxc.Format(2, 1, 32, 3), 4, 64)
    with pytest.raises(mxc.MxcError):
        mxc.packed_sizes(mxc.Format(3, 4, 32, 8), 4, 64)                # 8 bits > 6


def test_host_side_argument_errors(L):
    """Errors are found before any HIP call, so fake (never dereferenced) pointers are enough."""
    import paper_2411_09510_amd as mxc
    from paper_2411_09510_amd.binding import _CFormat
    f = _CFormat(2, 1, 32, 8)
    fp = ctypes.byref(f)
    good, odd = 0x10000, 0x10004
    vp = ctypes.c_void_p
    assert L.mxc_quantize(fp, None, 4, 64, good, good, None) == -1
    assert L.mxc_quantize(None, good, 4, 64, good, good, None) == -1
    assert L.mxc_quantize(fp, good, 4, 48, good, good, None) == -3
    assert L.mxc_quantize(fp, good, -1, 64, good, good, None) == -3
    assert L.mxc_quantize(fp, good, 1 << 30, 1 << 20, good, good, None) == -3      # too large
    assert L.mxc_quantize(fp, odd, 4, 64, good, good, None) == -4
    assert L.mxc_quantize(fp, good, 4, 64, odd, good, None) == -4
    assert L.mxc_quantize(fp, good, 4, 64, good, 0x10001, None) == -4
    bad = _CFormat(2, 1, 12, 8)
    assert L.mxc_quantize(ctypes.byref(bad), good, 4, 64, good, good, None) == -2
    # empty tensors are fine and launch nothing
    assert L.mxc_quantize(fp, good, 0, 64, good, good, None) == 0
    arr = (vp * 2)(good, good)
    assert L.mxc_quantize_batched(fp, 0, arr, 4, 64, arr, arr, None) == -5
    assert L.mxc_quantize_batched(fp, 33, arr, 4, 64, arr, arr, None) == -5
    assert L.mxc_dequant_reduce(fp, 0, arr, arr, 4, 64, good, 0, None) == -5
    assert L.mxc_dequant_reduce(fp, 33, arr, arr, 4, 64, good, 0, None) == -5
    assert L.mxc_dequant_reduce(fp, 2, arr, arr, 4, 64, good, 7, None) == -7
    assert L.mxc_dequant_reduce(fp, 2, arr, arr, 4, 64, None, 0, None) == -1
    assert L.mxc_dequant_reduce(fp, 2, arr, arr, 4, 64, odd, 0, None) == -4
    assert L.mxc_dequant_reduce(fp, 2, arr, arr, 0, 64, good, 0, None) == 0
    nul = (vp * 2)(good, None)
    assert L.mxc_dequant_reduce(fp, 2, nul, arr, 4, 64, good, 0, None) == -1
    assert L.mxc_requantize_chunk(fp, good, 0, 6, 64, 4, 0, good, good, None) == -3   # 6 % 4
    assert L.mxc_requantize_chunk(fp, good, 0, 8, 64, 4, 4, good, good, None) == -5
    assert L.mxc_requantize_chunk(fp, good, 0, 8, 64, 4, -1, good, good, None) == -5
    assert L.mxc_requantize_chunk(fp, good, 5, 8, 64, 4, 0, good, good, None) == -7
    assert L.mxc_dequant_reduce_own(fp, 2, 2, good, arr, arr, 4, 64, good, 0, None) == -5
    assert L.mxc_dequant_reduce_own(fp, 2, -1, good, arr, arr, 4, 64, good, 0, None) == -5
    assert L.mxc_dequant_reduce_own(fp, 2, 0, None, arr, arr, 4, 64, good, 0, None) == -1
    assert L.mxc_dequant_reduce_own(fp, 2, 0, odd, arr, arr, 4, 64, good, 0, None) == -4
    assert L.mxc_dequant_reduce_own(fp, 2, 0, good, nul, arr, 4, 64, good, 0, None) == -1   # rank 1 NULL
    nul0 = (vp * 2)(None, good)
    assert L.mxc_dequant_reduce_own(fp, 2, 0, good, nul0, nul0, 0, 64, good, 0, None) == 0  # own may be NULL
    assert L.mxc_dequant_reduce_requantize(fp, 2, arr, arr, 4, 64, good, None, None) == -1
    assert L.mxc_dequant_reduce_requantize(fp, 2, arr, arr, 4, 64, good, 0x10002, None) == -4
    assert L.mxc_dequant_reduce_requantize(fp, 40, arr, arr, 4, 64, good, good, None) == -5
    small = _CFormat(2, 1, 8, 8)
    assert L.mxc_dequant_reduce_requantize(ctypes.byref(small), 2, arr, arr, 1, 8, good, good, None) == -3
    assert L.mxc_copy_probe(good, good, 24, None) == -3
    assert L.mxc_copy_probe(good, odd, 32, None) == -4
    assert L.mxc_copy_probe(good, good, 0, None) == 0
    assert L.mxc_time_next_launch(None, None) == 0          # disarming needs no device
    for code in range(-8, 1):
        assert L.mxc_strerror(code)
    assert b"gfx950" in L.mxc_version()
    assert mxc.version().startswith("mxc")


def test_binding_refuses_host_tensors():
    import torch
    import paper_2411_09510_amd as mxc
    with pytest.raises(ValueError):
        mxc.quantize(mxc.Format(2, 1), torch.zeros(4, 64, dtype=torch.bfloat16))


def test_binding_refuses_buffers_of_the_wrong_size():
    """The binding is the only layer that knows buffer sizes: a short, long or misshapen buffer
    raises before anything is launched (checked here with host tensors: the size check comes
    before the device check, so no GPU is needed)."""
    import torch
    import paper_2411_09510_amd as mxc
    f = mxc.Format(2, 1, 32, 8)
    T, H = 4, 64
    cb, sb = mxc.packed_sizes(f, T, H)
    u8 = lambda n: torch.zeros(n, dtype=torch.uint8)
    x = torch.zeros(T, H, dtype=torch.bfloat16)
    size = "holds .* bytes"
    with pytest.raises(ValueError, match=size):
        mxc.quantize(f, x, u8(cb - 1), u8(sb))
    with pytest.raises(ValueError, match=size):
        mxc.quantize(f, x, u8(cb), u8(sb + 1))
    with pytest.raises(ValueError, match="one 2-D shape"):
        mxc.quantize_batched(f, [x, torch.zeros(T, 2 * H, dtype=torch.bfloat16)])
    with pytest.raises(ValueError, match="same length"):
        mxc.quantize_batched(f, [x, x], [u8(cb)], [u8(sb), u8(sb)])
    with pytest.raises(ValueError, match=size):
        mxc.dequant_reduce(f, [u8(cb), u8(cb // 2)], [u8(sb), u8(sb)], T, H)
    with pytest.raises(ValueError, match=size):
        mxc.dequant_reduce(f, [u8(cb)], [u8(sb)], 2 * T, H)                  # caller's shape is wrong
    with pytest.raises(ValueError, match=size):
        mxc.dequant_reduce(f, [u8(cb)], [u8(sb)], T, H, out=torch.zeros(T, H // 2))
    with pytest.raises(ValueError, match="float32 or bfloat16"):
        mxc.dequant_reduce(f, [u8(cb)], [u8(sb)], T, H, out=torch.zeros(T, H, dtype=torch.float16))
    with pytest.raises(ValueError, match=size):
        mxc.dequant_reduce_own(f, 0, x, [None, u8(cb + 16)], [None, u8(sb)])
    with pytest.raises(ValueError, match=size):
        mxc.dequant_reduce_requantize(f, [u8(cb)], [u8(sb)], T, H, u8(cb), u8(sb - 1))
    with pytest.raises(ValueError, match=size):
        mxc.requantize_chunk(f, torch.zeros(T, H), 2, 0, u8(cb), u8(sb))     # a chunk is half of that
    with pytest.raises(ValueError, match="multiple of tp"):
        mxc.requantize_chunk(f, torch.zeros(T, H), 3, 0)
    with pytest.raises(ValueError, match=size):
        mxc.prepare_dequant_reduce(f, [u8(cb)], [u8(sb)], T, H, torch.zeros(T + 1, H))
    with pytest.raises(ValueError, match=size):
        mxc.prepare_quantize_batched(f, [x], [u8(cb)], [u8(2 * sb)])
    with pytest.raises(ValueError, match=size):
        mxc.prepare_dequant_reduce_requantize(f, [u8(cb)], [u8(sb)], T, H, u8(1), u8(sb))
    with pytest.raises(ValueError, match=size):
        mxc.prepare_requantize_chunk(f, torch.zeros(T, H), 1, 0, u8(cb), u8(1))
    with pytest.raises(ValueError, match=size):
        mxc.copy_probe(u8(16), u8(32))
    # right sizes get as far as the device check
    with pytest.raises(ValueError, match="device tensors only"):
        mxc.dequant_reduce(f, [u8(cb)], [u8(sb)], T, H, out=torch.zeros(T, H))


def test_integer_types_are_one_bit_exponent_floats(oracle_mod):
    """INT3/4/5 (Method, parameter list) = E1M1/E1M2/E1M3: a uniform symmetric grid."""
    import paper_2411_09510_amd as mxc
    for k in (3, 4, 5):
        f = mxc.int_format(k, 16, 5)
        assert (f.ebits, f.mbits, f.block, f.scale_bits) == (1, k - 2, 16, 5) and f.bits == k
        fo = oracle_mod.Format(f.ebits, f.mbits, f.block, f.scale_bits)
        vals = [oracle_mod.code_value(fo, c) for c in range(2 ** (k - 1))]
        assert vals == [c * vals[1] for c in range(2 ** (k - 1))]       # uniform grid
        assert mxc.effective_bits(f) == k + 5 / 16
    with pytest.raises(ValueError):
        mxc.int_format(8)


def test_bench_names_the_reduce_kernel_by_the_librarys_own_rule():
    """bench.py reports which reduce kernel a call launches; its rule must be the host
    dispatch's: same element type, same rank range, same tile size, same size limit."""
    import bench
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = open(os.path.join(root, "paper_2411_09510_amd", "csrc", "mxc_reduce.hpp")).read()
    disp = open(os.path.join(root, "paper_2411_09510_amd", "csrc", "mxc_dispatch.hpp")).read()
    m = re.search(r"kHalfFormMaxUnits = \(size_t\)(\d+) \* (\d+) / 8;", src)
    max_elems = int(m.group(1)) * int(m.group(2))
    min_ranks = int(re.search(r"kHalfFormMinRanks = (\d+);", src).group(1))
    max_ranks = int(re.search(r"kFastRanks = (\d+);", src).group(1))
    assert "kHalfFormOk = E::hw == HW_FP4" in src                       # E2M1 only
    assert "a.tp >= kHalfFormMinRanks && a.tp <= kFastRanks && a.units % 128 == 0 && a.units <= kHalfFormMaxUnits" in disp
    half, tile = "dequant_reduce_half_kernel", "dequant_reduce_tile_kernel"
    assert bench.reduce_kernel(2, 1, max_ranks, 4096, 8192) == half
    assert bench.reduce_kernel(2, 1, min_ranks, 1, 1024) == half
    assert bench.reduce_kernel(2, 1, min_ranks - 1, 4096, 8192) == tile
    assert bench.reduce_kernel(2, 1, max_ranks + 1, 4096, 8192) == tile
    assert bench.reduce_kernel(2, 1, max_ranks, max_elems // 8192, 8192) == half
    assert bench.reduce_kernel(2, 1, max_ranks, max_elems // 8192 + 1, 8192) == tile
    assert bench.reduce_kernel(2, 1, max_ranks, 3, 1056) == tile            # not whole 1024-element tiles
    assert bench.reduce_kernel(2, 2, max_ranks, 4096, 8192) == tile
    assert bench.reduce_kernel(3, 2, max_ranks, 4096, 8192) == tile
