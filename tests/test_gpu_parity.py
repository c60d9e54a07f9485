"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs.  Codes, scales and the float32 reduction are compared
bit for bit (NaN compared as NaN); the relative-error bar of 1e-6 for the reduction is also
asserted explicitly."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu

HOT = [(2, 1), (2, 2), (3, 2)]
ALL_ELEMENTS = [(1, 1), (1, 2), (1, 3), (1, 4), (2, 1), (2, 2), (2, 3), (3, 1), (3, 2)]


@pytest.fixture(scope="module")
def mxc():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2411_09510_amd as m
    m.lib()
    return m


def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def host(t):
    return t.cpu().numpy()


def dev_scales(oracle_mod, fo, codes):
    """Scale codes [T, H/B] -> the device array the library reads (bit stream for s < 8)."""
    if fo.scale_bits == 8:
        return torch.from_numpy(np.ascontiguousarray(codes)).cuda()
    return torch.from_numpy(oracle_mod.pack_scales(fo, codes)).cuda()


def host_scales(oracle_mod, fo, t, shape):
    """Device scale array as written by the library -> scale codes of the given shape; for
    s < 8 also checks that the stream is exactly the oracle's packing of those codes."""
    raw = host(t)
    if fo.scale_bits == 8:
        return raw.reshape(shape)
    n = int(np.prod(shape))
    codes = oracle_mod.unpack_scales(fo, raw, n)
    assert np.array_equal(raw.ravel(), oracle_mod.pack_scales(fo, codes)), "padding bits not zero"
    return codes.reshape(shape)


def same_f32(a, b):
    a, b = np.asarray(a, np.float32), np.asarray(b, np.float32)
    nan_a, nan_b = np.isnan(a), np.isnan(b)
    return np.array_equal(nan_a, nan_b) and np.array_equal(a.view(np.uint32)[~nan_a],
                                                            b.view(np.uint32)[~nan_b])


def check_quantize(mxc, oracle_mod, x, y, B, bits, s=8):
    fo = oracle_mod.Format(x, y, B, s)
    fg = mxc.Format(x, y, B, s)
    codes, scales = mxc.quantize(fg, dev_bf16(bits))
    torch.cuda.synchronize()
    ocodes, oscales = oracle_mod.quantize_bf16(fo, bits)
    assert np.array_equal(host_scales(oracle_mod, fo, scales, oscales.shape), oscales), "scales differ"
    got = oracle_mod.unpack(fo, host(codes), bits.shape[1])
    if not np.array_equal(got, ocodes):
        bad = np.argwhere(got != ocodes)[0]
        raise AssertionError(f"codes differ first at {tuple(bad)}: gpu {got[tuple(bad)]} oracle "
                             f"{ocodes[tuple(bad)]} input {bits[tuple(bad)]:#06x}")
    assert np.array_equal(host(codes), oracle_mod.pack(fo, ocodes)), "packing differs"
    return codes, scales, ocodes, oscales


# ------------------------------------------------------------------------ quantize ----------

@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
@pytest.mark.parametrize("B", [8, 16, 32])
def test_quantize_config1_all_formats(mxc, oracle_mod, x, y, B):
    w = workloads.CONFIGS[1]
    for r in range(w.tp):
        check_quantize(mxc, oracle_mod, x, y, B, workloads.partial_bf16(w, r))


@pytest.mark.parametrize("T,H", [(1, 32), (3, 64), (5, 1056), (7, 8192), (129, 96), (2, 40000 // 32 * 32),
                                 (1, 8192 + 32), (33, 2048 + 160)])
def test_quantize_ragged_shapes(mxc, oracle_mod, T, H):
    """Sizes that end inside a wave's tile, inside a workgroup's tile, and just past one."""
    w = workloads.Workload("ragged", 1, T, H, seed=17, n_outlier=1, outlier_mult=(30.0, 30.0))
    bits = workloads.partial_bf16(w, 0)
    for (x, y) in HOT + [(1, 1)]:
        for B in (8, 16, 32):
            check_quantize(mxc, oracle_mod, x, y, B, bits)


@pytest.mark.parametrize("x,y", [(2, 1), (2, 2), (3, 2), (1, 1), (3, 1), (1, 4)])
def test_quantize_sizes_that_are_not_multiples_of_32(mxc, oracle_mod, x, y):
    """Blocks of 8 or 16 allow tensors whose size is not a multiple of 32 elements: the last
    quad of lanes then holds 1 to 3 units and the packed stream ends inside a dword.  Outputs
    must be exact and nothing may be written past them (canaries), for every code width and
    for 8-bit and narrow scales."""
    for (B, T, H) in ((8, 1, 8), (8, 1, 40), (8, 3, 24), (8, 5, 1048), (8, 7, 2056), (16, 1, 16),
                      (16, 3, 48), (16, 5, 1040), (32, 3, 96)):
        for s in (8, 5):
            fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
            cb, sb = mxc.packed_sizes(fg, T, H)
            codes = torch.full((cb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            scales = torch.full((sb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            w = workloads.Workload("canary", 1, T, H, seed=3 + T + H)
            bits = workloads.partial_bf16(w, 0)
            mxc.quantize(fg, dev_bf16(bits), codes[:cb], scales[:sb])
            # the same through the binary32 front end (requantize of the exact values)
            codes32 = torch.full((cb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            scales32 = torch.full((sb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            xf = torch.from_numpy(workloads.bf16_bits_to_f32(bits)).cuda()
            mxc.requantize_chunk(fg, xf, 1, 0, codes32[:cb], scales32[:sb])
            torch.cuda.synchronize()
            ocodes, oscales = oracle_mod.quantize_bf16(fo, bits)
            for c_, s_ in ((codes, scales), (codes32, scales32)):
                assert (c_[cb:] == 0xA5).all() and (s_[sb:] == 0xA5).all(), (B, T, H, s)
                assert np.array_equal(host_scales(oracle_mod, fo, s_[:sb], oscales.shape), oscales)
                assert np.array_equal(host(c_[:cb]).reshape(T, -1), oracle_mod.pack(fo, ocodes)), (B, T, H, s)
            # and back: the reduce of this one partial is its exact decode
            out = torch.full((T * H + 64,), 7.0, dtype=torch.float32, device="cuda")
            mxc.dequant_reduce(fg, [codes[:cb]], [scales[:sb]], T, H, out=out[:T * H].view(T, H))
            torch.cuda.synchronize()
            assert (out[T * H:] == 7.0).all()
            assert same_f32(host(out[:T * H]).reshape(T, H), oracle_mod.dequantize(fo, ocodes, oscales))


@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
def test_quantize_every_bf16_value_every_alignment(mxc, oracle_mod, x, y):
    """All 65 536 bf16 bit patterns (non-finite ones made finite) beside anchors in many
    binades: every (value, shared exponent) pair the rounding can see."""
    B = 32
    allbits = np.arange(65536, dtype=np.uint32)
    finite = ((allbits >> 7) & 0xFF) != 0xFF
    allbits = np.where(finite, allbits, allbits & 0x807F).astype(np.uint16)
    anchors = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 40, 126, 127, 128, 129, 130, 133, 200, 247, 250,
               251, 252, 253, 254]
    rows = []
    for ae in anchors:
        blk = np.zeros((65536 // 16, B), dtype=np.uint16)
        blk[:, 0] = (ae << 7) | 0x35
        blk[:, 1:17] = allbits.reshape(-1, 16)
        blk[:, 17:32] = (allbits.reshape(-1, 16) ^ 0x8000)[:, :15]
        rows.append(blk)
    bits = np.concatenate(rows, axis=0)
    check_quantize(mxc, oracle_mod, x, y, B, bits)


@pytest.mark.parametrize("x,y", HOT)
def test_quantize_edge_tensors(mxc, oracle_mod, x, y):
    B = 32
    emax = 2 ** x - 1 - (2 ** (x - 1) - 1)
    maxval = 2.0 ** emax * (2 - 2.0 ** -y)
    blocks = []
    z = np.zeros(B, np.uint16)
    blocks.append(z.copy())                                   # all +0
    b = z.copy(); b[::2] = 0x8000; blocks.append(b)           # -0 mixed in
    b = z.copy(); b[:8] = [0x007F, 0x0040, 0x0020, 0x0010, 0x8030, 0x0001, 0x0050, 0x0060]
    blocks.append(b)                                          # bf16 subnormals only
    b = z.copy(); b[0] = 0x7F7F; b[1] = 0xFF7F; b[2] = 0x3F80; blocks.append(b)   # max finite
    for bad in (0x7F80, 0xFF80, 0x7FC0, 0xFFFF, 0x7F81):      # Inf / NaN anywhere in the block
        for pos in (0, 13, 31):
            b = z.copy(); b[:] = 0x3F80; b[pos] = bad; blocks.append(b)
    near = np.array([maxval, np.nextafter(np.float32(maxval), 0), maxval * 1.01, 2.0 ** (emax + 1) *
                     (1 - 2.0 ** -8), 2.0 ** emax, 1.0, 0.5, 0.25, 2.0 ** -10], np.float32)
    b = z.copy(); b[:len(near)] = workloads.f32_to_bf16_bits(near); blocks.append(b)
    b = z.copy(); b[0] = 0x0080; b[1] = 0x0040; blocks.append(b)          # smallest normal max
    bits = np.stack(blocks).astype(np.uint16)
    bits = np.concatenate([bits, bits[::-1]], axis=1)          # two blocks per row
    check_quantize(mxc, oracle_mod, x, y, B, bits)


@pytest.mark.parametrize("s", [4, 5, 6, 7])
def test_quantize_narrow_scale_formats(mxc, oracle_mod, s):
    w = workloads.small_like(workloads.CONFIGS[2], 32, 1024)
    bits = workloads.partial_bf16(w, 0)
    # stretch some rows far outside the narrow scale range
    f = workloads.bf16_bits_to_f32(bits)
    f[1] *= 2.0 ** 40
    f[2] *= 2.0 ** -40
    f[3, 5] = np.inf
    bits = workloads.f32_to_bf16_bits(np.nan_to_num(f, posinf=0, neginf=0))
    bits[3, 5] = 0x7F80
    for (x, y) in HOT:
        check_quantize(mxc, oracle_mod, x, y, 32, bits, s=s)


def test_quantize_batched_equals_single(mxc, oracle_mod):
    w = workloads.small_like(workloads.CONFIGS[3], 24, 2048)
    xs = [dev_bf16(workloads.partial_bf16(w, r)) for r in range(w.tp)]
    for (x, y) in HOT:
        fg = mxc.Format(x, y, 32, 8)
        cb, sb = mxc.quantize_batched(fg, xs)
        torch.cuda.synchronize()
        for r in range(w.tp):
            c1, s1 = mxc.quantize(fg, xs[r])
            assert torch.equal(c1, cb[r]) and torch.equal(s1, sb[r])
            oc, os_ = oracle_mod.quantize_bf16(oracle_mod.Format(x, y, 32, 8),
                                               workloads.partial_bf16(w, r))
            assert np.array_equal(host(sb[r]), os_)
            assert np.array_equal(host(cb[r]), oracle_mod.pack(oracle_mod.Format(x, y, 32, 8), oc))


# ------------------------------------------------------------------------ dequant-reduce ----

def oracle_partials(oracle_mod, fo, w):
    cs, ss = [], []
    for r in range(w.tp):
        c, s = oracle_mod.quantize_bf16(fo, workloads.partial_bf16(w, r))
        cs.append(c)
        ss.append(s)
    return cs, ss


def check_reduce(mxc, oracle_mod, fo, fg, cs, ss, T, H):
    packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in cs]
    scales = [dev_scales(oracle_mod, fo, s) for s in ss]
    out = mxc.dequant_reduce(fg, packed, scales, T, H)
    out16 = mxc.dequant_reduce(fg, packed, scales, T, H, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    want = oracle_mod.dequant_reduce(fo, cs, ss)
    got = host(out)
    assert same_f32(got, want), "float32 reduction differs"
    fin = np.isfinite(want)
    denom = np.abs(want[fin]).max() if fin.any() else 1.0
    assert np.abs(got[fin].astype(np.float64) - want[fin]).max() <= 1e-6 * max(denom, 1e-30)
    want16 = oracle_mod.round_to_bf16(want)
    assert np.array_equal(host(out16.view(torch.int16)).view(np.uint16), want16)
    return out


@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
@pytest.mark.parametrize("B", [8, 16, 32])
def test_reduce_config1_all_formats(mxc, oracle_mod, x, y, B):
    w = workloads.CONFIGS[1]
    fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
    cs, ss = oracle_partials(oracle_mod, fo, w)
    check_reduce(mxc, oracle_mod, fo, fg, cs, ss, w.tokens, w.hidden)


def test_reduce_and_fused_do_not_write_past_the_end(mxc, oracle_mod):
    """Canaries behind every output of the reduce kernels (f32, bf16, own-raw, fused), on ragged
    sizes, among them sizes that are not a multiple of 32 elements: their last chunk holds 8, 16
    or 24 elements, alone in a wave tile or behind whole tiles."""
    rng = np.random.default_rng(4)
    for (x, y, B, T, H) in ((2, 1, 32, 3, 96), (2, 2, 32, 5, 2080), (3, 2, 32, 1, 32), (2, 1, 8, 3, 40),
                            (3, 2, 16, 7, 48), (1, 1, 8, 1, 8), (2, 2, 8, 5, 1048), (2, 1, 16, 129, 80),
                            (3, 2, 8, 3, 2056)):
        fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
        tp = 3
        ocs = [rng.integers(0, 2 ** fo.bits, size=(T, H), dtype=np.uint8) for _ in range(tp)]
        oss = [rng.integers(100, 150, size=(T, H // B), dtype=np.uint8) for _ in range(tp)]
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in ocs]
        scales = [torch.from_numpy(v).cuda() for v in oss]
        n = T * H
        want = oracle_mod.dequant_reduce(fo, ocs, oss)
        for dt in (torch.float32, torch.bfloat16):
            buf = torch.full((n + 64,), 7.0, dtype=dt, device="cuda")
            mxc.dequant_reduce(fg, packed, scales, T, H, out=buf[:n].view(T, H))
            torch.cuda.synchronize()
            assert (buf[n:] == 7.0).all()
            if dt == torch.float32:
                assert same_f32(host(buf[:n]).reshape(T, H), want)
        own = dev_bf16(workloads.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32)))
        buf = torch.full((n + 64,), 7.0, dtype=torch.float32, device="cuda")
        mxc.dequant_reduce_own(fg, 1, own, packed, scales, out=buf[:n].view(T, H))
        torch.cuda.synchronize()
        assert (buf[n:] == 7.0).all()
        if n % 32 == 0:
            cb, sb = mxc.packed_sizes(fg, T, H)
            cbuf = torch.full((cb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            sbuf = torch.full((sb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
            mxc.dequant_reduce_requantize(fg, packed, scales, T, H, cbuf[:cb], sbuf[:sb])
            torch.cuda.synchronize()
            assert (cbuf[cb:] == 0xA5).all() and (sbuf[sb:] == 0xA5).all()
            oc, os_ = oracle_mod.quantize_f32(fo, want)
            assert np.array_equal(host(sbuf[:sb]).reshape(T, -1), os_)
            assert np.array_equal(host(cbuf[:cb]).reshape(T, -1), oracle_mod.pack(fo, oc))
        else:
            with pytest.raises(mxc.MxcError):
                mxc.dequant_reduce_requantize(fg, packed, scales, T, H)


@pytest.mark.parametrize("tp", [1, 2, 3, 4, 7, 8, 9, 16, 17, 32])
def test_reduce_any_tp(mxc, oracle_mod, tp):
    w = workloads.Workload("tp", tp, 9, 1056, seed=40 + tp, n_outlier=3, outlier_mult=(20.0, 100.0))
    for (x, y) in HOT:
        fo, fg = oracle_mod.Format(x, y, 32, 8), mxc.Format(x, y, 32, 8)
        cs, ss = oracle_partials(oracle_mod, fo, w)
        check_reduce(mxc, oracle_mod, fo, fg, cs, ss, w.tokens, w.hidden)


def test_reduce_arbitrary_codes_and_scales(mxc, oracle_mod):
    """Random code and scale bytes (not produced by the quantizer): every code, scale bytes 0
    (binary32-subnormal scale), 254 (products overflow to Inf) and 255 (NaN marker), far-apart
    binades so that the order of the adds shows."""
    rng = np.random.default_rng(9)
    T, H, tp = 6, 2048, 5
    for (x, y) in ALL_ELEMENTS:
        for B in (8, 32):
            fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
            cs = [rng.integers(0, 2 ** fo.bits, size=(T, H), dtype=np.uint8) for _ in range(tp)]
            ss = []
            for r in range(tp):
                s = rng.integers(100, 160, size=(T, H // B), dtype=np.uint8)
                s[0] = rng.integers(0, 256, size=H // B)
                s[1, ::3] = 0
                s[2, ::5] = 254
                s[3, ::7] = 255
                ss.append(s)
            check_reduce(mxc, oracle_mod, fo, fg, cs, ss, T, H)


@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
@pytest.mark.parametrize("B", [8, 32])
def test_reduce_every_code_every_position_every_scale(mxc, oracle_mod, x, y, B):
    """Decode check of the reduce kernels' conversions: every element code at every position of
    a 32-element chunk under every scale byte 0..255 (row t carries scale byte t), as the only
    partial (tp = 1: the output is the exact decode) and as the second of two partials.  Rows
    are 2^b chunks long, so every wave tile is full and takes the kernels' main path."""
    fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
    ncodes = 2 ** fo.bits
    T, H = 256, 32 * ncodes
    h = np.arange(H)
    codes = np.broadcast_to(((h % 32) + (h // 32)) % ncodes, (T, H)).astype(np.uint8).copy()
    scales = np.broadcast_to(np.arange(T, dtype=np.uint8)[:, None], (T, H // B)).copy()
    check_reduce(mxc, oracle_mod, fo, fg, [codes], [scales], T, H)
    other = np.full((T, H), 1, np.uint8)
    mid = np.full((T, H // B), 127, np.uint8)
    check_reduce(mxc, oracle_mod, fo, fg, [other, codes], [mid, scales], T, H)


def test_reduce_keeps_negative_zero_and_order(mxc, oracle_mod):
    fo, fg = oracle_mod.Format(2, 1, 32, 8), mxc.Format(2, 1, 32, 8)
    T, H = 1, 64
    negz = np.full((T, H), 8, np.uint8)
    s = np.full((T, H // 32), 127, np.uint8)
    out = check_reduce(mxc, oracle_mod, fo, fg, [negz] * 3, [s] * 3, T, H)
    assert np.all(np.signbit(host(out)))
    one = np.full((T, H), 2, np.uint8)
    big = np.full((T, H // 32), 127 + 24, np.uint8)
    a = check_reduce(mxc, oracle_mod, fo, fg, [one] * 3, [big, s, s], T, H)
    b = check_reduce(mxc, oracle_mod, fo, fg, [one] * 3, [s, s, big], T, H)
    assert float(a[0, 0]) == 2.0 ** 24 and float(b[0, 0]) == 2.0 ** 24 + 2


@pytest.mark.parametrize("x,y,B", [(2, 1, 32), (2, 2, 32), (3, 2, 32), (2, 1, 8), (1, 1, 16)])
def test_reduce_with_own_raw_partial(mxc, oracle_mod, x, y, B):
    """Profiling: N-1 decoded partials plus the worker's own uncompressed one, every own rank;
    a shape that takes the tile kernel and one (with small blocks) that does not."""
    for (T, H) in ((12, 1024), (3, 40)) if B == 8 else ((12, 1024),):
        w = workloads.Workload("own", 5, T, H, seed=77, n_outlier=2, outlier_mult=(20.0, 100.0))
        fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
        parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
        ocs, oss = oracle_partials(oracle_mod, fo, w)
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in ocs]
        scales = [torch.from_numpy(s).cuda() for s in oss]
        for own in range(w.tp):
            cs = [None if r == own else packed[r] for r in range(w.tp)]
            ss = [None if r == own else scales[r] for r in range(w.tp)]
            out = mxc.dequant_reduce_own(fg, own, dev_bf16(parts[own]), cs, ss)
            out16 = mxc.dequant_reduce_own(fg, own, dev_bf16(parts[own]), packed, scales,
                                           out_dtype=torch.bfloat16)
            torch.cuda.synchronize()
            want = oracle_mod.dequant_reduce_own(fo, own, parts[own],
                                                 [None if r == own else ocs[r] for r in range(w.tp)],
                                                 [None if r == own else oss[r] for r in range(w.tp)])
            assert same_f32(host(out), want)
            assert np.array_equal(host(out16.view(torch.int16)).view(np.uint16),
                                  oracle_mod.round_to_bf16(want))


@pytest.mark.parametrize("s", [4, 5, 6, 7])
def test_reduce_narrow_scale_formats(mxc, oracle_mod, s):
    """Scale streams of 4 to 7 bits per block, for blocks of 32, 16 and 8 (1, 2 and 4 fields per
    lane), on whole wave tiles plus a partial one, in every form of the reduction."""
    w = workloads.small_like(workloads.CONFIGS[2], 19, 544)
    for (x, y, B) in [(x, y, 32) for (x, y) in HOT] + [(2, 1, 16), (2, 2, 8), (1, 1, 8)]:
        fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
        cs, ss = oracle_partials(oracle_mod, fo, w)
        check_reduce(mxc, oracle_mod, fo, fg, cs, ss, w.tokens, w.hidden)
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in cs]
        scales = [dev_scales(oracle_mod, fo, v) for v in ss]
        own_bits = workloads.partial_bf16(w, 2)
        own = mxc.dequant_reduce_own(fg, 2, dev_bf16(own_bits), packed, scales)
        torch.cuda.synchronize()
        assert same_f32(host(own), oracle_mod.dequant_reduce_own(fo, 2, own_bits, cs, ss))


@pytest.mark.parametrize("B", [8, 16, 32])
@pytest.mark.parametrize("s", [8, 7, 5, 4])
def test_reduce_e2m1_tensors_of_whole_kilo_element_tiles(mxc, oracle_mod, B, s):
    """E2M1 tensors whose size is a multiple of 1024 elements, reduced over 6 to 8 ranks, take a
    form of the reduce kernel of their own (16 elements per lane, 1024 per wave, the rank count a
    compile-time constant): every rank count from 1 to 9 (those it covers and those on either
    side, which take the general form), 19 wave tiles (two workgroups and part of a third),
    arbitrary codes, the special scale codes, float32 and bf16 output, the fused form, and the
    own-raw form at every own rank."""
    rng = np.random.default_rng(1000 + 10 * B + s)
    T, H = 19, 1024
    fo, fg = oracle_mod.Format(2, 1, B, s), mxc.Format(2, 1, B, s)
    smax = 255 if s == 8 else 2 ** s - 1
    for tp in range(1, 10):
        cs = [rng.integers(0, 16, size=(T, H), dtype=np.uint8) for _ in range(tp)]
        ss = []
        for r in range(tp):
            lo = 100 if s == 8 else 0
            v = rng.integers(lo, min(lo + 60, smax + 1), size=(T, H // B), dtype=np.uint8)
            v[0] = rng.integers(0, smax + 1, size=H // B)
            v[1, r::3] = 0
            v[2, r::5] = smax - 1 if s == 8 else smax
            v[3, r::7] = smax
            ss.append(v)
        cs[0][4] = 8                                   # a row of -0 in every rank stays -0
        for r in range(1, tp):
            cs[r][4] = 8
        out = check_reduce(mxc, oracle_mod, fo, fg, cs, ss, T, H)
        assert np.all(np.signbit(host(out)[4]))
        if tp > 8:
            continue
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in cs]
        scales = [dev_scales(oracle_mod, fo, v) for v in ss]
        # the fused form, with canaries behind both outputs
        cb, sb = mxc.packed_sizes(fg, T, H)
        cbuf = torch.full((cb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        sbuf = torch.full((sb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        cf, sf_ = mxc.dequant_reduce_requantize(fg, packed, scales, T, H, cbuf[:cb].view(T, cb // T), sbuf[:sb])
        torch.cuda.synchronize()
        assert (cbuf[cb:] == 0xA5).all() and (sbuf[sb:] == 0xA5).all()
        oc, os_ = oracle_mod.quantize_f32(fo, oracle_mod.dequant_reduce(fo, cs, ss))
        assert np.array_equal(host_scales(oracle_mod, fo, sf_, os_.shape), os_), tp
        assert np.array_equal(host(cf), oracle_mod.pack(fo, oc)), tp
        own_bits = workloads.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32) * 3.0)
        for own in range(tp):
            got = mxc.dequant_reduce_own(fg, own, dev_bf16(own_bits), packed, scales)
            got16 = mxc.dequant_reduce_own(fg, own, dev_bf16(own_bits), packed, scales,
                                           out_dtype=torch.bfloat16)
            torch.cuda.synchronize()
            want = oracle_mod.dequant_reduce_own(fo, own, own_bits, cs, ss)
            assert same_f32(host(got), want), (tp, own)
            assert np.array_equal(host(got16.view(torch.int16)).view(np.uint16),
                                  oracle_mod.round_to_bf16(want)), (tp, own)


def test_bf16_output_rounding_at_every_bf16_value(mxc, oracle_mod):
    """Rounding of the binary32 sum to a bf16 output, at its hardest inputs: the own partial holds
    every bf16 bit pattern (65 536 elements: both signs, subnormals, Inf, NaN) and the one other
    rank adds a quarter, a half or three quarters of that element's bf16 unit in the last place
    (E2M1 codes 0.5, 1.0, 1.5 under a per-block scale of 2^(exponent - 8)), so that the sum lies
    below, exactly on and above the midpoint between two bf16 values for every one of them."""
    fo, fg = oracle_mod.Format(2, 1, 32, 8), mxc.Format(2, 1, 32, 8)
    T, H = 64, 1024                                   # 65 536 elements, whole 1024-element tiles
    own_bits = np.arange(65536, dtype=np.uint16).reshape(T, H)
    expfield = ((own_bits >> 7) & 0xFF).reshape(T, H // 32, 32)[:, :, 0].astype(np.int32)
    scale = np.clip(expfield - 8, 0, 254).astype(np.uint8)    # a block of 32 patterns shares its exponent
    for code in (1, 2, 3, 9, 10, 11):                 # +-0.5, +-1.0, +-1.5 times the scale
        other = np.full((T, H), code, np.uint8)
        for tp, own in ((2, 0), (2, 1), (7, 3)):      # the general and the 1024-element-tile forms
            cs = [np.zeros((T, H), np.uint8) for _ in range(tp)]
            ss = [np.full((T, H // 32), 127, np.uint8) for _ in range(tp)]
            k = (own + 1) % tp
            cs[k], ss[k] = other, scale
            packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in cs]
            scales = [torch.from_numpy(v).cuda() for v in ss]
            got16 = mxc.dequant_reduce_own(fg, own, dev_bf16(own_bits), packed, scales, out_dtype=torch.bfloat16)
            got32 = mxc.dequant_reduce_own(fg, own, dev_bf16(own_bits), packed, scales)
            torch.cuda.synchronize()
            want = oracle_mod.dequant_reduce_own(fo, own, own_bits, cs, ss)
            assert same_f32(host(got32), want), (code, tp, own)
            assert np.array_equal(host(got16.view(torch.int16)).view(np.uint16),
                                  oracle_mod.round_to_bf16(want)), (code, tp, own)
    # the midpoints really are among the sums: with +1.0 x scale the float32 sum of a positive
    # normal value has exactly the bit below bf16's last place set
    cs = [np.zeros((T, H), np.uint8), np.full((T, H), 2, np.uint8)]
    ss = [np.full((T, H // 32), 127, np.uint8), scale]
    s32 = oracle_mod.dequant_reduce_own(fo, 0, own_bits, cs, ss).view(np.uint32)
    pos_normal = (own_bits >= (9 << 7)) & (own_bits < (0xFF << 7))
    assert np.all((s32[pos_normal] & 0xFFFF) == 0x8000)


# ------------------------------------------------------------------------ requantize --------

@pytest.mark.parametrize("x,y,B", [(2, 1, 16), (2, 1, 32), (2, 2, 32), (3, 2, 32), (1, 3, 8)])
def test_requantize_chunks(mxc, oracle_mod, x, y, B):
    w = workloads.small_like(workloads.CONFIGS[4], 64, 1024)
    fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
    xs = [dev_bf16(workloads.partial_bf16(w, r)) for r in range(w.tp)]
    codes, scales = mxc.quantize_batched(fg, xs)
    red = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden)
    red16 = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    red_h = host(red)
    # end to end against the all-oracle pipeline (the reduction is bit-reproducible)
    ocs, oss = oracle_partials(oracle_mod, fo, w)
    assert same_f32(red_h, oracle_mod.dequant_reduce(fo, ocs, oss))
    rows = w.tokens // w.tp
    for c in range(w.tp):
        cc, sc = mxc.requantize_chunk(fg, red, w.tp, c)
        c16, s16 = mxc.requantize_chunk(fg, red16, w.tp, c)
        torch.cuda.synchronize()
        oc, os_ = oracle_mod.quantize_f32(fo, red_h[c * rows:(c + 1) * rows])
        assert np.array_equal(host(sc), os_)
        assert np.array_equal(host(cc), oracle_mod.pack(fo, oc))
        bits16 = host(red16.view(torch.int16)).view(np.uint16)[c * rows:(c + 1) * rows]
        oc, os_ = oracle_mod.quantize_bf16(fo, bits16)
        assert np.array_equal(host(s16), os_)
        assert np.array_equal(host(c16), oracle_mod.pack(fo, oc))


@pytest.mark.parametrize("x,y,B", [(2, 1, 32), (2, 1, 16), (2, 1, 8), (2, 2, 32), (3, 2, 32), (3, 2, 16),
                                   (1, 1, 32), (1, 3, 8), (2, 3, 32), (3, 1, 16), (1, 4, 32)])
def test_fused_reduce_requantize_equals_unfused_pair(mxc, oracle_mod, x, y, B):
    """The fused call must give, bit for bit, what dequant_reduce to binary32 followed by
    requantize gives, and both must match the oracle's pipeline."""
    rng = np.random.default_rng(x * 100 + y * 10 + B)
    for tp, T, H in ((8, 16, 1024), (3, 5, 2080), (1, 2, 64)):
        w = workloads.Workload("fused", tp, T, H, seed=60 + tp, n_outlier=2, outlier_mult=(20.0, 100.0))
        fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
        ocs, oss = oracle_partials(oracle_mod, fo, w)
        if tp == 3:                                   # arbitrary bytes too: NaN markers, far binades
            ocs = [rng.integers(0, 2 ** fo.bits, size=(T, H), dtype=np.uint8) for _ in range(tp)]
            oss = [rng.integers(90, 170, size=(T, H // B), dtype=np.uint8) for _ in range(tp)]
            oss[1][0, ::4] = 255
            oss[2][1, ::3] = 254
            oss[0][2, ::5] = 0
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in ocs]
        scales = [torch.from_numpy(s).cuda() for s in oss]
        red = mxc.dequant_reduce(fg, packed, scales, T, H)
        c2, s2 = mxc.requantize_chunk(fg, red, 1, 0)
        cf, sf_ = mxc.dequant_reduce_requantize(fg, packed, scales, T, H)
        torch.cuda.synchronize()
        assert torch.equal(sf_, s2) and torch.equal(cf, c2)
        want = oracle_mod.dequant_reduce(fo, ocs, oss)
        oc, os_ = oracle_mod.quantize_f32(fo, want)
        assert np.array_equal(host(sf_), os_)
        assert np.array_equal(host(cf), oracle_mod.pack(fo, oc))


@pytest.mark.parametrize("s", [4, 5, 6, 7])
def test_fused_and_requantize_with_narrow_scales(mxc, oracle_mod, s):
    """Narrow scale formats clamp at both ends (sums far above the range saturate, far below
    round to zero) and travel as an s-bit stream, in the fused form and in requantize alike;
    shapes with whole wave tiles, with a ragged tail, and one whose size is not a multiple of 32."""
    rng = np.random.default_rng(s)
    for (x, y, B, T, H, tp) in ((3, 2, 32, 8, 1024, 4), (2, 1, 32, 3, 2080, 3), (2, 2, 16, 5, 1040, 2),
                                (2, 1, 8, 9, 1032, 2), (1, 1, 8, 1, 40, 3)):
        fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
        top = 2 ** s - 1
        ocs = [rng.integers(0, 2 ** fo.bits, size=(T, H), dtype=np.uint8) for _ in range(tp)]
        oss = [rng.integers(0, top + 1, size=(T, H // B), dtype=np.uint8) for _ in range(tp)]
        packed = [torch.from_numpy(oracle_mod.pack(fo, c)).cuda() for c in ocs]
        scales = [dev_scales(oracle_mod, fo, v) for v in oss]
        cb, sb = mxc.packed_sizes(fg, T, H)
        assert scales[0].numel() == sb == (T * (H // B) * s + 7) // 8
        red = mxc.dequant_reduce(fg, packed, scales, T, H)
        # stretch the reduced tensor far outside the scale range for the requantize check
        wide = red.clone()
        wide[0] *= 2.0 ** 60
        if T > 2:
            wide[2] *= 2.0 ** -60
        sbuf = torch.full((sb + 16,), 0xA5, dtype=torch.uint8, device="cuda")
        c2, s2 = mxc.requantize_chunk(fg, wide, 1, 0, scales=sbuf[:sb],
                                      codes=torch.empty((T, cb // T), dtype=torch.uint8, device="cuda"))
        torch.cuda.synchronize()
        assert (sbuf[sb:] == 0xA5).all()
        want = oracle_mod.dequant_reduce(fo, ocs, oss)
        assert same_f32(host(red), want)
        oc, os_ = oracle_mod.quantize_f32(fo, host(wide))
        assert np.array_equal(host_scales(oracle_mod, fo, s2, os_.shape), os_)
        assert np.array_equal(host(c2), oracle_mod.pack(fo, oc))
        if (T * H) % 32 == 0:
            fbuf = torch.full((sb + 16,), 0xA5, dtype=torch.uint8, device="cuda")
            cf, sf_ = mxc.dequant_reduce_requantize(
                fg, packed, scales, T, H, torch.empty((T, cb // T), dtype=torch.uint8, device="cuda"),
                fbuf[:sb])
            torch.cuda.synchronize()
            assert (fbuf[sb:] == 0xA5).all()
            oc, os_ = oracle_mod.quantize_f32(fo, want)
            assert np.array_equal(host_scales(oracle_mod, fo, sf_, os_.shape), os_)
            assert np.array_equal(host(cf), oracle_mod.pack(fo, oc))


def test_requantize_f32_rounding_corners(mxc, oracle_mod):
    """binary32 inputs a hair around rounding midpoints, which need all 24 significand bits."""
    rng = np.random.default_rng(21)
    for (x, y) in ALL_ELEMENTS:
        fo, fg = oracle_mod.Format(x, y, 8, 8), mxc.Format(x, y, 8, 8)
        book = np.array([oracle_mod.code_value(fo, c) for c in range(2 ** (x + y))])
        mids = (book[:-1] + book[1:]) / 2
        rows = []
        for k in (-126, -100, -20, 0, 3, 60, 120):
            for mval in mids:
                base = np.float32(mval * 2.0 ** k)
                near = [np.nextafter(base, np.float32(0)), base, np.nextafter(base, np.float32(np.inf))]
                rows.append([np.float32(book[-1] * 2.0 ** k)] + near + [-near[0], -near[2], 0, 0])
        xin = np.array(rows, dtype=np.float32)
        rnd = (rng.standard_normal((4096, 8)) * np.exp(rng.standard_normal((4096, 1)) * 20)).astype(np.float32)
        sub = (rng.standard_normal((256, 8)) * 2.0 ** -140).astype(np.float32)       # subnormals
        spec = np.zeros((4, 8), np.float32)
        spec[0, 0] = np.inf; spec[1, 3] = np.nan; spec[2, :] = -0.0; spec[3, 0] = np.finfo(np.float32).max
        xin = np.concatenate([xin, rnd, sub, spec])
        pad = (-xin.shape[0]) % 4
        xin = np.concatenate([xin, np.zeros((pad, 8), np.float32)])
        t = torch.from_numpy(xin).cuda()
        cc, sc = mxc.requantize_chunk(fg, t, 1, 0)
        torch.cuda.synchronize()
        oc, os_ = oracle_mod.quantize_f32(fo, xin)
        assert np.array_equal(host(sc), os_)
        got = oracle_mod.unpack(fo, host(cc), 8)
        assert np.array_equal(got, oc), np.argwhere(got != oc)[:5]


# ------------------------------------------------------------------------ streams -----------

def test_calls_run_on_the_stream_they_are_given(mxc, oracle_mod):
    """Two independent pipelines issued on two non-default streams at once; each call passes its
    stream explicitly.  Results must be those of the oracle for both."""
    fo, fg = oracle_mod.Format(2, 1, 32, 8), mxc.Format(2, 1, 32, 8)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for k, st in enumerate(streams):
        w = workloads.Workload("streams", 4, 96, 4096, seed=500 + k, n_outlier=4,
                               outlier_mult=(20.0, 100.0))
        parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
        xs = [dev_bf16(p) for p in parts]
        jobs.append((w, parts, xs, st))
    torch.cuda.synchronize()
    outs = []
    for rep in range(3):
        for (w, parts, xs, st) in jobs:
            codes, scales = mxc.quantize_batched(fg, xs, stream=st)
            with torch.cuda.stream(st):
                out = torch.empty((w.tokens, w.hidden), dtype=torch.float32, device="cuda")
            mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out=out, stream=st)
            outs.append((w, parts, out, codes, scales))
    for st in streams:
        st.synchronize()
    for (w, parts, out, codes, scales) in outs:
        ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
        assert same_f32(host(out), oracle_mod.dequant_reduce(fo, list(ocs), list(oss)))
        for r in range(w.tp):
            assert np.array_equal(host(scales[r]), oss[r])


def test_timed_launch_gives_the_same_result_and_a_kernel_duration(mxc, oracle_mod):
    """Events armed for one launch are stamped by that launch only, leave its output unchanged,
    and measure a duration inside the host-side wall time of the synchronised call."""
    import time
    fo, fg = oracle_mod.Format(2, 2, 32, 8), mxc.Format(2, 2, 32, 8)
    w = workloads.Workload("timed", 4, 256, 4096, seed=77, n_outlier=4, outlier_mult=(20.0, 100.0))
    parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
    xs = [dev_bf16(p) for p in parts]
    codes, scales = mxc.quantize_batched(fg, xs)            # also warms the kernels up
    out = torch.empty((w.tokens, w.hidden), dtype=torch.float32, device="cuda")
    mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out=out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mxc.time_next_launch(ev[0], ev[1])
    codes, scales = mxc.quantize_batched(fg, xs)
    mxc.time_next_launch(ev[2], ev[3])
    mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out=out)
    mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out=out)   # not timed: pair was used
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    q_ms, r_ms = ev[0].elapsed_time(ev[1]), ev[2].elapsed_time(ev[3])
    assert 0.0 < q_ms < wall_ms and 0.0 < r_ms < wall_ms
    assert ev[1].elapsed_time(ev[2]) >= 0.0                # the reduce began after the quantize ended
    ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
    for r in range(w.tp):
        assert np.array_equal(host(codes[r]).reshape(w.tokens, -1), oracle_mod.pack(fo, ocs[r]))
        assert np.array_equal(host(scales[r]), oss[r])
    assert same_f32(host(out), oracle_mod.dequant_reduce(fo, list(ocs), list(oss)))


# ------------------------------------------------------------------------ HIP graphs --------

def test_calls_can_be_captured_in_a_hip_graph(mxc, oracle_mod):
    """The library allocates nothing and never synchronises, so a step (quantize all partials,
    reduce, requantize a chunk, fused form) can be recorded into a HIP graph.  The graph is
    replayed several times on fresh inputs, with eager work and synchronisations in between, and
    every replay is checked against the oracle."""
    w = workloads.small_like(workloads.CONFIGS[2], 64, 1024)
    fo, fg = oracle_mod.Format(2, 2, 32, 8), mxc.Format(2, 2, 32, 8)
    T, H, N = w.tokens, w.hidden, w.tp
    xs = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(N)]
    cb, sb = mxc.packed_sizes(fg, T, H)
    codes = [torch.zeros((T, cb // T), dtype=torch.uint8, device="cuda") for _ in range(N)]
    scales = [torch.zeros((T, sb // T), dtype=torch.uint8, device="cuda") for _ in range(N)]
    out = torch.zeros((T, H), dtype=torch.float32, device="cuda")
    cbc, sbc = mxc.packed_sizes(fg, T // N, H)
    cc = torch.zeros(cbc, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(sbc, dtype=torch.uint8, device="cuda")
    cf = torch.zeros(cb, dtype=torch.uint8, device="cuda")
    sf_ = torch.zeros(sb, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mxc.quantize_batched(fg, xs, codes, scales)
        mxc.dequant_reduce(fg, codes, scales, T, H, out=out)
        mxc.requantize_chunk(fg, out, N, 1, cc, sc)
        mxc.dequant_reduce_requantize(fg, codes, scales, T, H, cf, sf_)
    for replay in range(4):
        ww = workloads.Workload("graph", N, T, H, seed=300 + replay, n_outlier=3,
                                outlier_mult=(20.0, 100.0))
        parts = [workloads.partial_bf16(ww, r) for r in range(N)]
        for r in range(N):
            xs[r].copy_(dev_bf16(parts[r]))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
        want = oracle_mod.dequant_reduce(fo, list(ocs), list(oss))
        assert same_f32(host(out), want)
        for r in range(N):
            assert np.array_equal(host(scales[r]), oss[r])
            assert np.array_equal(host(codes[r]), oracle_mod.pack(fo, ocs[r]))
        rows = T // N
        oc, os_ = oracle_mod.quantize_f32(fo, want[rows:2 * rows])
        assert np.array_equal(host(sc).reshape(rows, -1), os_)
        assert np.array_equal(host(cc).reshape(rows, -1), oracle_mod.pack(fo, oc))
        oc, os_ = oracle_mod.quantize_f32(fo, want)
        assert np.array_equal(host(sf_).reshape(T, -1), os_)
        assert np.array_equal(host(cf).reshape(T, -1), oracle_mod.pack(fo, oc))
        # eager work between replays
        eager = mxc.dequant_reduce(fg, codes, scales, T, H)
        torch.cuda.synchronize()
        assert torch.equal(eager, out)


def test_narrow_scales_lose_non_finite_blocks_like_the_oracle(mxc, oracle_mod):
    """Rule 5 of the library's contract: with scales narrower than 8 bits a block that held a
    NaN decodes to zeros, so the all-decoded reduction is finite on every worker and the own-raw
    reduction is NaN only on the worker that owns the NaN.  GPU = oracle in every case."""
    T, H, B = 4, 2048, 32
    w = workloads.Workload("nf", 2, T, H, seed=77)
    parts = [workloads.partial_bf16(w, r) for r in range(2)]
    parts[0][1, 40] = 0x7FC0
    parts[0][2, 1000] = 0xFF80
    xs = [dev_bf16(p) for p in parts]
    for s in (5, 8):
        fo, fg = oracle_mod.Format(2, 2, B, s), mxc.Format(2, 2, B, s)
        codes, scales = mxc.quantize_batched(fg, xs)
        ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
        out = host(mxc.dequant_reduce(fg, codes, scales, T, H))
        own = [host(mxc.dequant_reduce_own(fg, r, xs[r], codes, scales)) for r in range(2)]
        torch.cuda.synchronize()
        assert same_f32(out, oracle_mod.dequant_reduce(fo, list(ocs), list(oss)))
        for r in range(2):
            assert same_f32(own[r], oracle_mod.dequant_reduce_own(fo, r, parts[r], list(ocs), list(oss)))
        if s == 8:
            assert np.isnan(out[1, 32:64]).all() and np.isnan(own[1][1, 32:64]).all()
        else:
            assert np.isfinite(out).all() and np.isfinite(own[1]).all()
            assert np.isnan(own[0][1, 40]) and np.isinf(own[0][2, 1000])


def test_an_empty_call_disarms_the_timing_events(mxc, oracle_mod):
    """Events armed for "the next launch" are dropped by a valid call on an empty tensor, so
    they do not stamp a later, unrelated kernel."""
    fg = mxc.Format(2, 1, 32, 8)
    w = workloads.small_like(workloads.CONFIGS[3], 2048, 8192)
    x = dev_bf16(workloads.partial_bf16(w, 0))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    e1.record()
    torch.cuda.synchronize()
    empty = torch.empty((0, 8192), dtype=torch.bfloat16, device="cuda")
    ce, se = torch.empty((0, 4096), dtype=torch.uint8, device="cuda"), torch.empty((0, 256), dtype=torch.uint8, device="cuda")
    before = e0.elapsed_time(e1)
    mxc.time_next_launch(e0, e1)
    # torch gives an empty tensor a null data pointer; the ABI wants non-null ones, so hand it
    # the addresses of a real buffer with zero rows
    import ctypes
    f = fg.c()
    rc = mxc.lib().mxc_quantize(ctypes.byref(f), x.data_ptr(), 0, 8192, x.data_ptr(), x.data_ptr(), None)
    assert rc == 0
    del empty, ce, se
    mxc.quantize(fg, x)                      # would have been stamped had the pair stayed armed
    torch.cuda.synchronize()
    assert e0.elapsed_time(e1) == before


# ------------------------------------------------------------------------ quality proxy -----

@pytest.mark.parametrize("x,y,B,s", [(2, 1, 32, 8), (2, 2, 32, 8), (3, 2, 32, 8), (2, 1, 32, 5), (2, 2, 8, 8)])
def test_quality_proxy_of_the_gpu_pipeline_equals_the_oracle_pipeline(mxc, oracle_mod, x, y, B, s):
    """SQNR of the reduced output against the uncompressed sum (the stand-in for the paper's
    perplexity tables): the GPU pipeline's figure is the oracle pipeline's figure, and the
    benchmark's own torch computation of it agrees."""
    import bench
    w = workloads.CONFIGS[1]
    fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
    parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
    xs = [dev_bf16(p) for p in parts]
    codes, scales = mxc.quantize_batched(fg, xs)
    out = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden)
    torch.cuda.synchronize()
    exact = oracle_mod.sum_bf16(parts)
    ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
    want = oracle_mod.sqnr_db(exact, oracle_mod.dequant_reduce(fo, list(ocs), list(oss)))
    got = oracle_mod.sqnr_db(exact, host(out))
    assert got == want and 5.0 < got < 40.0
    exact_dev = xs[0].float()
    for t in xs[1:]:
        exact_dev += t.float()
    assert np.array_equal(host(exact_dev).view(np.uint32), exact.view(np.uint32))
    assert abs(bench.sqnr_db(torch, out, exact_dev) - want) < 1e-6


# ------------------------------------------------------------------------ full size ---------

def test_full_size_config3_whole_tensor(mxc, oracle_mod):
    """The benchmark's launch configuration (all 8 partials of bf16 [4096 x 8192] in one batched
    launch, then one reduce), for the three element formats of the configuration: every code
    byte and scale byte of all 8 partials and every element of the reduced tensor against the
    oracle, in float32, in bf16, re-quantized by the fused call, and with rank 3's partial raw."""
    w = workloads.CONFIGS[3]
    parts = workloads.all_partials_bf16(w)
    xs = [dev_bf16(p) for p in parts]
    for (x, y, B, s) in w.formats:
        fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
        codes, scales = mxc.quantize_batched(fg, xs)
        out = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden)
        torch.cuda.synchronize()
        ocs, oss = [], []
        for r in range(w.tp):
            oc, os_ = oracle_mod.quantize_bf16(fo, parts[r])
            assert np.array_equal(host(scales[r]), os_), (x, y, r)
            assert np.array_equal(host(codes[r]), oracle_mod.pack(fo, oc)), (x, y, r)
            ocs.append(oc)
            oss.append(os_)
        want = oracle_mod.dequant_reduce(fo, ocs, oss)
        assert same_f32(host(out), want), (x, y)
        # the other forms of the reduction the benchmark times at this size: bf16 output, the
        # fused reduce + requantize, and the own-raw form (rank 3's view)
        out16 = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden, out_dtype=torch.bfloat16)
        cf, sf_ = mxc.dequant_reduce_requantize(fg, codes, scales, w.tokens, w.hidden)
        own = mxc.dequant_reduce_own(fg, 3, xs[3], codes, scales)
        torch.cuda.synchronize()
        assert np.array_equal(host(out16.view(torch.int16)).view(np.uint16), oracle_mod.round_to_bf16(want)), (x, y)
        oc, os_ = oracle_mod.quantize_f32(fo, want)
        assert np.array_equal(host(sf_), os_), (x, y)
        assert np.array_equal(host(cf), oracle_mod.pack(fo, oc)), (x, y)
        del oc, os_, out16, cf, sf_
        want_own = oracle_mod.dequant_reduce_own(fo, 3, parts[3], ocs, oss)
        assert same_f32(host(own), want_own), (x, y)
        del ocs, oss, want, want_own, own
        cb, sb = mxc.packed_sizes(fg, w.tokens, w.hidden)
        ratio = w.tokens * w.hidden * 2 / (cb + sb)
        assert abs(ratio - 16 / (fo.bits + s / B)) < 1e-9
        del codes, scales, out


@pytest.mark.parametrize("cfg", [2, 4, 5])
def test_full_size_other_configs_sampled_rows(mxc, oracle_mod, cfg):
    """Configurations 2, 4 and 5 at their full sizes, in the launch configuration the benchmark
    uses (batched quantize, one reduce, per-chunk requantize and the fused form where the
    configuration names requantization): some 280 rows, 36 drawn from every 1/tp row chunk,
    element by element against the oracle,
    every scale byte against the scale rule, sizes against the closed form."""
    w = workloads.CONFIGS[cfg]
    rng = np.random.default_rng(cfg)
    n_chunk = w.tokens // w.tp
    rows = np.unique(np.concatenate(
        [[0, n_chunk - 1, n_chunk, w.tokens - 1]] +
        [c * n_chunk + rng.integers(0, n_chunk, 36) for c in range(w.tp)]))
    parts = workloads.all_partials_bf16(w)
    xs = [dev_bf16(p) for p in parts]
    for (x, y, B, s) in w.formats:
        fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
        emax = 2 ** x - 1 - (2 ** (x - 1) - 1)
        codes, scales = mxc.quantize_batched(fg, xs)
        out = mxc.dequant_reduce(fg, codes, scales, w.tokens, w.hidden)
        torch.cuda.synchronize()
        ocs, oss = [], []
        for r in range(w.tp):
            oc, os_ = oracle_mod.quantize_bf16(fo, parts[r][rows])
            assert np.array_equal(host(scales[r][rows]), os_)
            assert np.array_equal(host(codes[r][rows]), oracle_mod.pack(fo, oc))
            ocs.append(oc)
            oss.append(os_)
            expf = torch.from_numpy(((parts[r] >> 7) & 0xFF).astype(np.int16)).cuda()
            blockmax = expf.view(w.tokens, -1, B).max(dim=2).values.to(torch.int32)
            assert torch.equal(scales[r].to(torch.int32), (blockmax - emax).clamp_(min=0))
        want = oracle_mod.dequant_reduce(fo, ocs, oss)
        got = host(out[rows])
        assert same_f32(got, want)
        if w.requantize:
            n_rows = w.tokens // w.tp
            for c in (0, w.tp - 1, 3):
                cc, sc = mxc.requantize_chunk(fg, out, w.tp, c)
                # the fused form on the compressed copies of that chunk
                cin = [codes[r][c * n_rows:(c + 1) * n_rows] for r in range(w.tp)]
                sin = [scales[r][c * n_rows:(c + 1) * n_rows] for r in range(w.tp)]
                cf, sf_ = mxc.dequant_reduce_requantize(fg, cin, sin, n_rows, w.hidden)
                torch.cuda.synchronize()
                assert torch.equal(cf, cc) and torch.equal(sf_, sc)
                sel = rows[(rows >= c * n_rows) & (rows < (c + 1) * n_rows)]
                if len(sel):
                    idx = np.searchsorted(rows, sel)
                    oc, os_ = oracle_mod.quantize_f32(fo, want[idx])
                    assert np.array_equal(host(sc[sel - c * n_rows]), os_)
                    assert np.array_equal(host(cc[sel - c * n_rows]), oracle_mod.pack(fo, oc))
        cb, sb = mxc.packed_sizes(fg, w.tokens, w.hidden)
        assert abs(w.tokens * w.hidden * 2 / (cb + sb) - 16 / (fo.bits + s / B)) < 1e-9
        del codes, scales, out


@pytest.mark.parametrize("x,y", [(2, 1), (2, 2)])
def test_tensor_beyond_two_to_the_32_elements(mxc, oracle_mod, x, y):
    """One tensor of 2^32 + 2^17 elements (32769 rows of 131072), so element indices, byte offsets
    of the bf16 input, of the packed codes and of the float32 output all cross 2^31 and 2^32
    inside the tensor.  Rows on both sides of every such boundary, the first and the last row
    are checked element by element against the oracle; the scale rule is checked everywhere."""
    T, H, B = 32769, 131072, 32
    fo, fg = oracle_mod.Format(x, y, B, 8), mxc.Format(x, y, B, 8)
    gen = torch.Generator(device="cuda").manual_seed(4100 + x * 10 + y)
    xd = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    for a in range(0, T, 4096):
        b = min(T, a + 4096)
        blk = torch.randn((b - a, H), generator=gen, device="cuda")
        blk *= torch.exp2(torch.randint(-12, 6, (b - a, 1), generator=gen, device="cuda").float())
        xd[a:b] = blk.bfloat16()
        del blk
    rows = np.array([0, 1, 8191, 8192, 16383, 16384, 16385, 24577, 32767, 32768])
    codes, scales = mxc.quantize(fg, xd)
    out = mxc.dequant_reduce(fg, [codes, codes], [scales, scales], T, H)
    out16 = mxc.dequant_reduce(fg, [codes, codes], [scales, scales], T, H, out_dtype=torch.bfloat16)
    cf, sf_ = mxc.dequant_reduce_requantize(fg, [codes, codes], [scales, scales], T, H)
    torch.cuda.synchronize()
    xr = host(xd[rows].view(torch.int16)).view(np.uint16)
    oc, os_ = oracle_mod.quantize_bf16(fo, xr)
    assert np.array_equal(host(scales[rows]), os_)
    assert np.array_equal(host(codes[rows]), oracle_mod.pack(fo, oc))
    want = oracle_mod.dequant_reduce(fo, [oc, oc], [os_, os_])
    assert same_f32(host(out[rows]), want)
    assert np.array_equal(host(out16[rows].view(torch.int16)).view(np.uint16),
                          oracle_mod.round_to_bf16(want))
    oc2, os2 = oracle_mod.quantize_f32(fo, want)
    assert np.array_equal(host(sf_[rows]), os2)
    assert np.array_equal(host(cf[rows]), oracle_mod.pack(fo, oc2))
    # scale rule on every block of the tensor
    emax = 2 ** x - 1 - (2 ** (x - 1) - 1)
    for a in range(0, T, 8192):
        b = min(T, a + 8192)
        expf = (xd[a:b].view(torch.int16) >> 7) & 0xFF
        blockmax = expf.view(b - a, -1, B).max(dim=2).values.to(torch.int32)
        assert torch.equal(scales[a:b].to(torch.int32), (blockmax - emax).clamp_(min=0))


# ------------------------------------------------------------------------ random cases ------

def random_cases(count, seed, tp_max=9, t_max=39, h_blocks=69):
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        x, y = ALL_ELEMENTS[rng.integers(len(ALL_ELEMENTS))]
        B = int(rng.choice([8, 16, 32]))
        s = int(rng.choice([8, 8, 8, 7, 6, 5, 4]))
        tp = int(rng.integers(1, tp_max + 1))
        T = int(rng.integers(1, t_max + 1))
        H = B * int(rng.integers(1, h_blocks + 1))
        cases.append((k, x, y, B, s, tp, T, H))
    return cases


def check_random_configuration(mxc, oracle_mod, k, x, y, B, s, tp, T, H):
    """Formats, scale widths, tp, shapes (ragged, not multiples of 32 elements included) and
    stress inputs drawn from a seeded generator; every entry point against the oracle."""
    fo, fg = oracle_mod.Format(x, y, B, s), mxc.Format(x, y, B, s)
    parts = [workloads.stress_bf16(9000 + 100 * k + r, T, H) for r in range(tp)]
    if k % 3 == 0:      # activations-like values instead, so that sums are not dominated by one rank
        w = workloads.Workload("rand", tp, T, H, seed=9000 + k, n_outlier=min(2, H),
                               outlier_mult=(20.0, 100.0))
        parts = [workloads.partial_bf16(w, r) for r in range(tp)]
    xs = [dev_bf16(p) for p in parts]
    codes, scales = mxc.quantize_batched(fg, xs)
    out = mxc.dequant_reduce(fg, codes, scales, T, H)
    out16 = mxc.dequant_reduce(fg, codes, scales, T, H, out_dtype=torch.bfloat16)
    own_rank = k % tp
    own = mxc.dequant_reduce_own(fg, own_rank, xs[own_rank], codes, scales)
    fused = mxc.dequant_reduce_requantize(fg, codes, scales, T, H) if (T * H) % 32 == 0 else None
    rq = mxc.requantize_chunk(fg, out, 1, 0)
    torch.cuda.synchronize()
    ocs, oss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
    for r in range(tp):
        assert np.array_equal(host_scales(oracle_mod, fo, scales[r], oss[r].shape), oss[r])
        assert np.array_equal(host(codes[r]).reshape(T, -1), oracle_mod.pack(fo, ocs[r]))
    want = oracle_mod.dequant_reduce(fo, list(ocs), list(oss))
    assert same_f32(host(out), want)
    assert np.array_equal(host(out16.view(torch.int16)).view(np.uint16), oracle_mod.round_to_bf16(want))
    want_own = oracle_mod.dequant_reduce_own(fo, own_rank, parts[own_rank], list(ocs), list(oss))
    assert same_f32(host(own), want_own)
    oc2, os2 = oracle_mod.quantize_f32(fo, want)
    for got in ([rq] if fused is None else [rq, fused]):
        assert np.array_equal(host_scales(oracle_mod, fo, got[1], os2.shape), os2)
        assert np.array_equal(host(got[0]).reshape(T, -1), oracle_mod.pack(fo, oc2))


@pytest.mark.parametrize("k,x,y,B,s,tp,T,H", random_cases(96, 20241109))
def test_random_configurations(mxc, oracle_mod, k, x, y, B, s, tp, T, H):
    check_random_configuration(mxc, oracle_mod, k, x, y, B, s, tp, T, H)


@pytest.mark.parametrize("k,x,y,B,s,tp,T,H", random_cases(32, 20241127, tp_max=32, t_max=150, h_blocks=160))
def test_random_configurations_many_ranks_many_tiles(mxc, oracle_mod, k, x, y, B, s, tp, T, H):
    """The same with up to 32 partials (more than 8 take the reduce kernel's general instance) and
    tensors of up to a few hundred wave tiles."""
    check_random_configuration(mxc, oracle_mod, 1000 + k, x, y, B, s, tp, T, H)
