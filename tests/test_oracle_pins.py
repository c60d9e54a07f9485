"""Pins of the CPU oracle against things other than itself (CPU only).

Each test checks the C oracle against a fact the paper prints, a closed form, an invariant, a
special case that reduces to a library routine, or a brute-force search written here with
different means (exact rationals / exhaustive enumeration of the code book).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

ALL_ELEMENTS = [(1, 1), (1, 2), (1, 3), (2, 1), (2, 2), (3, 1), (3, 2), (2, 3), (1, 4)]
HOT_ELEMENTS = [(2, 1), (2, 2), (3, 2)]


# ----------------------------------------------------------------------------- helpers ------

def read_codebooks():
    books = {}
    for line in open(os.path.join(GOLDEN, "codebooks.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, vals = line.split(":")
        x, y = (int(t) for t in key.split())
        books[(x, y)] = [float(v) for v in vals.split()]
    return books


def codebook_from_definition(x, y):
    """Magnitudes of ExMy written straight from the format definition with exact rationals."""
    beta = 2 ** (x - 1) - 1
    out = []
    for code in range(2 ** (x + y)):
        expf, mant = code >> y, code & (2 ** y - 1)
        if expf == 0:
            out.append(Fraction(mant, 2 ** y) * Fraction(2) ** (1 - beta))
        else:
            out.append((1 + Fraction(mant, 2 ** y)) * Fraction(2) ** (expf - beta))
    return out


def bf16_to_fraction(h):
    sign, ex, fr = h >> 15, (h >> 7) & 0xFF, h & 0x7F
    if ex == 0:
        mag = Fraction(fr) * Fraction(2) ** (-133)
    else:
        mag = Fraction(128 + fr) * Fraction(2) ** (ex - 134)
    return -mag if sign else mag


def floor_log2_fraction(m):
    """Largest k with 2^k <= m, by search (no logarithm)."""
    k = 0
    while Fraction(2) ** k > m:
        k -= 1
    while Fraction(2) ** (k + 1) <= m:
        k += 1
    return k


def brute_block(bits_list, x, y, s=8):
    """Quantize one block of bf16 bit patterns with exact rational arithmetic and a linear
    search over the code book: (scale byte, [codes])."""
    book = codebook_from_definition(x, y)
    beta = 2 ** (x - 1) - 1
    emax = 2 ** x - 1 - beta
    sbias = 2 ** (s - 1) - 1
    smax = 254 if s == 8 else 2 ** s - 1
    vals = [bf16_to_fraction(h) for h in bits_list]
    m = max(abs(v) for v in vals)
    if m == 0:
        sc = 0
    else:
        sc = min(max(floor_log2_fraction(m) - emax + sbias, 0), smax)
    scale = Fraction(2) ** (sc - sbias)
    codes = []
    for h, v in zip(bits_list, vals):
        p = abs(v) / scale
        best, best_d = None, None
        for c, q in enumerate(book):
            d = abs(p - q)
            if best is None or d < best_d or (d == best_d and c % 2 == 0 and best % 2 == 1):
                best, best_d = c, d
        codes.append(((h >> 15) << (x + y)) | best)
    return sc, codes


def np_brute(fmt, bits):
    """Vectorised nearest-code search in float64 (every quantity is an exact dyadic number):
    returns (codes [T,H], scales [T,H/B]).  floor(log2) is found by comparing with a table of
    powers of two, the nearest code by an argmin over the whole code book."""
    x, y, B, s = fmt.ebits, fmt.mbits, fmt.block, fmt.scale_bits
    beta = 2 ** (x - 1) - 1
    emax = 2 ** x - 1 - beta
    sbias = 2 ** (s - 1) - 1
    smax = 254 if s == 8 else 2 ** s - 1
    book = np.array([float(q) for q in codebook_from_definition(x, y)])
    v = workloads.bf16_bits_to_f32(bits).astype(np.float64)
    T, H = v.shape
    a = np.abs(v).reshape(T, H // B, B)
    m = a.max(axis=2)
    pow2 = np.array([2.0 ** k for k in range(-150, 130)])
    E = np.searchsorted(pow2, m, side="right") - 1 - 150          # 2^E <= m < 2^(E+1)
    sc = np.clip(E - emax + sbias, 0, smax)
    sc[m == 0] = 0
    scale = np.array([2.0 ** int(k) for k in range(-sbias, smax - sbias + 1)])[sc]
    p = a / scale[:, :, None]
    d = np.abs(p[..., None] - book)                               # [T, nb, B, ncodes]
    best = d.argmin(axis=-1)                                      # lowest code among equals
    nxt = np.minimum(best + 1, len(book) - 1)
    tie = (np.take_along_axis(d, nxt[..., None], -1)[..., 0] ==
           np.take_along_axis(d, best[..., None], -1)[..., 0]) & (nxt != best)
    best = np.where(tie & (best % 2 == 1), nxt, best)
    sign = (bits.reshape(T, H // B, B) >> 15).astype(np.int64)
    codes = (sign << (x + y)) | best
    return codes.reshape(T, H).astype(np.uint8), sc.astype(np.uint8)


# --------------------------------------------------------------- sizes / effective bits -----

def test_effective_bits_match_paper_tables(oracle_mod):
    """Table 1 column 3 and the Table 3 caption."""
    n = 0
    for line in open(os.path.join(GOLDEN, "effective_bits.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        b, block, s, printed, src = line.split()
        b, block, s, printed = int(b), int(block), int(s), float(printed)
        # any ExMy with that many bits has the same size
        for (x, y) in ALL_ELEMENTS:
            if 1 + x + y != b:
                continue
            fmt = oracle_mod.Format(x, y, block, s)
            _, _, eff = oracle_mod.packed_sizes(fmt, 64, 1024)
            if src == "table3_caption":
                assert eff == printed
            else:
                assert abs(eff - printed) <= 0.05 + 1e-12, (fmt, eff, printed)
            n += 1
    assert n >= 10


def test_compression_ratio_closed_form(oracle_mod):
    """Compression vs 16-bit activations = 16 / (b + s/B); the arrays' real byte counts give
    the same number when the scale is a whole byte (s = 8)."""
    expect = {(2, 1): 16 / 4.25, (2, 2): 16 / 5.25, (3, 2): 16 / 6.25}
    for (x, y), ratio in expect.items():
        fmt = oracle_mod.Format(x, y, 32, 8)
        cb, sb, eff = oracle_mod.packed_sizes(fmt, 4096, 8192)
        assert abs(16 / eff - ratio) < 1e-12
        assert abs((4096 * 8192 * 2) / (cb + sb) - ratio) < 1e-12
    assert round(16 / 4.25, 3) == 3.765 and round(16 / 5.25, 3) == 3.048 and round(16 / 6.25, 3) == 2.56
    # the paper's "3.5 - 4.5x" range (Abstract) is 16/4.6 ... 16/3.6 of Table 1
    lo = 16 / oracle_mod.packed_sizes(oracle_mod.Format(2, 1, 8, 5), 8, 64)[2]
    hi = 16 / oracle_mod.packed_sizes(oracle_mod.Format(1, 1, 8, 5), 8, 64)[2]
    assert round(lo, 1) == 3.5 and round(hi, 1) == 4.4


def test_scale_stream_and_wire_size_for_every_scale_format(oracle_mod):
    """Narrow scales travel as an s-bit stream, so the arrays' real sizes give the closed-form
    effective bits for every scale format (Table 1 was printed with 5-bit scales)."""
    rng = np.random.default_rng(8)
    for s in (4, 5, 6, 7, 8):
        fmt = oracle_mod.Format(2, 1, 8, s)
        T, H = 16, 1024
        cb, sb, eff = oracle_mod.packed_sizes(fmt, T, H)
        assert sb == T * (H // 8) * s // 8
        assert abs((cb + sb) * 8 / (T * H) - eff) < 1e-12 and eff == 4 + s / 8
        top = 255 if s == 8 else 2 ** s
        codes = rng.integers(0, top, size=(5, 13), dtype=np.uint8)          # 65 blocks: ragged tail
        packed = oracle_mod.pack_scales(fmt, codes)
        stream = sum(int(c) << (k * s) for k, c in enumerate(codes.ravel()))
        assert bytes(packed) == stream.to_bytes((65 * s + 7) // 8, "little")
        assert np.array_equal(oracle_mod.unpack_scales(fmt, packed, 65), codes.ravel())
    # FP4, block 8, 5-bit scale: 4.625 bits -> the paper's 3.5x
    cb, sb, eff = oracle_mod.packed_sizes(oracle_mod.Format(2, 1, 8, 5), 64, 4096)
    assert round(64 * 4096 * 2 / (cb + sb), 1) == 3.5


def test_packed_sizes_are_array_sizes(oracle_mod):
    for (x, y) in ALL_ELEMENTS:
        for B in (8, 16, 32):
            fmt = oracle_mod.Format(x, y, B, 8)
            T, H = 3, 64
            cb, sb, _ = oracle_mod.packed_sizes(fmt, T, H)
            codes = np.zeros((T, H), np.uint8)
            assert oracle_mod.pack(fmt, codes).size == cb == T * H * fmt.bits // 8
            assert sb == T * H // B


# ----------------------------------------------------------------------- code book ----------

def test_code_values_match_public_value_sets(oracle_mod):
    books = read_codebooks()
    assert set(books) >= {(2, 1), (3, 2), (2, 2), (1, 1), (1, 2), (1, 3), (3, 1)}
    for (x, y), mags in books.items():
        fmt = oracle_mod.Format(x, y, 32, 8)
        got = [oracle_mod.code_value(fmt, c) for c in range(2 ** (x + y))]
        assert got == mags, (x, y)
        neg = [oracle_mod.code_value(fmt, c | (1 << (x + y))) for c in range(2 ** (x + y))]
        assert neg == [-m for m in mags]
        assert np.signbit(neg[0])            # the -0 code decodes to -0.0


def test_code_values_match_definition_all_formats(oracle_mod):
    for (x, y) in ALL_ELEMENTS:
        fmt = oracle_mod.Format(x, y, 32, 8)
        book = codebook_from_definition(x, y)
        for c, q in enumerate(book):
            assert Fraction(oracle_mod.code_value(fmt, c)) == q
        assert all(b2 > b1 for b1, b2 in zip(book, book[1:]))     # code order = value order


def test_e1my_is_a_uniform_grid(oracle_mod):
    """Appendix ablation table: INT3/4/5 rows equal the E1M1/E1M2/E1M3 rows."""
    for y in (1, 2, 3, 4):
        fmt = oracle_mod.Format(1, y, 32, 8)
        vals = [oracle_mod.code_value(fmt, c) for c in range(2 ** (1 + y))]
        step = 2.0 ** (1 - y)
        assert vals == [c * step for c in range(2 ** (1 + y))]


def test_scales_are_powers_of_two(oracle_mod):
    for s in (4, 5, 6, 7, 8):
        fmt = oracle_mod.Format(2, 1, 32, s)
        top = 254 if s == 8 else 2 ** s - 1
        bias = 2 ** (s - 1) - 1
        for c in range(top + 1):
            v = oracle_mod.scale_value(fmt, c)
            assert Fraction(v) == Fraction(2) ** (c - bias)
    assert np.isnan(oracle_mod.scale_value(oracle_mod.Format(2, 1, 32, 8), 255))


# ----------------------------------------------------------------------- hand block ---------

def test_hand_worked_blocks(oracle_mod):
    fmt = oracle_mod.Format(2, 1, 32, 8)
    n = 0
    for line in open(os.path.join(GOLDEN, "hand_block_e2m1.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, vals, scale, codes = [t.strip() for t in line.split("|")]
        vals = np.array([float(v) for v in vals.split()], dtype=np.float32)
        x = np.zeros((1, 32), np.float32)
        x[0, :len(vals)] = vals
        want = [int(c) for c in codes.split()]
        for got_codes, got_scales in (oracle_mod.quantize_f32(fmt, x),
                                      oracle_mod.quantize_bf16(fmt, workloads.f32_to_bf16_bits(x))):
            assert got_scales[0, 0] == int(scale), name
            assert list(got_codes[0, :len(want)]) == want, name
            assert not got_codes[0, len(want):].any()
        n += 1
    assert n == 4


# ----------------------------------------------------------------------- brute force --------

@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
def test_exact_rational_brute_force_on_small_blocks(oracle_mod, x, y):
    """Nearest code by linear search with exact rationals; blocks of 8 drawn so that elements
    land on every part of the grid (top binade, subnormals, below half the smallest step)."""
    rng = np.random.default_rng(100 * x + y)
    fmt = oracle_mod.Format(x, y, 8, 8)
    blocks = []
    for _ in range(160):
        top = int(rng.choice([1, 2, 5, 60, 127, 128, 200, 254]))
        ex = np.clip(top - rng.integers(0, 9, size=8), 0, 254)
        fr = rng.integers(0, 128, size=8)
        sg = rng.integers(0, 2, size=8)
        blocks.append((sg << 15) | (ex << 7) | fr)
    bits = np.array(blocks, dtype=np.uint16)
    codes, scales = oracle_mod.quantize_bf16(fmt, bits)
    for i in range(bits.shape[0]):
        sc, cs = brute_block([int(h) for h in bits[i]], x, y)
        assert scales[i, 0] == sc, (i, bits[i])
        assert list(codes[i]) == cs, (i, bits[i])


@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
def test_exact_ties_go_to_even_code(oracle_mod, x, y):
    """Midpoints between neighbouring magnitudes, scaled into several binades: the code picked
    must be the even one (checked with exact rationals; midpoints need y+2 <= 8 bits)."""
    book = codebook_from_definition(x, y)
    fmt = oracle_mod.Format(x, y, 8, 8)
    emax = 2 ** x - 1 - (2 ** (x - 1) - 1)
    for k in (-100, -3, 0, 7, 90):
        top = float(book[-1]) * 2.0 ** k           # puts the block max in the top binade -> e = k
        for c in range(len(book) - 1):
            mid = float((book[c] + book[c + 1]) / 2) * 2.0 ** k
            xin = np.array([[top, mid, -mid, 0, 0, 0, 0, 0]], dtype=np.float32)
            bits = workloads.f32_to_bf16_bits(xin)
            assert workloads.bf16_bits_to_f32(bits)[0, 1] == np.float32(mid)   # representable
            codes, scales = oracle_mod.quantize_bf16(fmt, bits)
            assert scales[0, 0] == 127 + k
            even = c if c % 2 == 0 else c + 1
            assert codes[0, 1] == even and codes[0, 2] == even | (1 << (x + y)), (k, c)
            assert codes[0, 0] == len(book) - 1
    assert emax >= 1


@pytest.mark.parametrize("x,y,B", [(2, 1, 32), (2, 2, 32), (3, 2, 32), (2, 1, 16), (1, 2, 8),
                                   (3, 1, 8), (1, 1, 8), (1, 3, 16)])
def test_every_bf16_value_against_enumeration(oracle_mod, x, y, B):
    """Every one of the 65 536 bf16 bit patterns (non-finite ones replaced by finite values)
    next to anchors in many binades: nearest-code enumeration must agree everywhere."""
    fmt = oracle_mod.Format(x, y, B, 8)
    allbits = np.arange(65536, dtype=np.uint32)
    finite = ((allbits >> 7) & 0xFF) != 0xFF
    allbits = np.where(finite, allbits, allbits & 0x807F).astype(np.uint16)
    anchors_exp = [0, 1, 2, 3, 4, 5, 9, 64, 126, 127, 128, 131, 200, 250, 253, 254]
    rows = []
    for ae in anchors_exp:
        blk = np.zeros((65536, B), dtype=np.uint16)
        blk[:, 0] = (ae << 7) | 0x35                # anchor with a non-trivial fraction
        blk[:, 1] = allbits
        blk[:, 2] = allbits ^ 0x8000
        rows.append(blk)
    bits = np.concatenate(rows, axis=0)
    codes, scales = oracle_mod.quantize_bf16(fmt, bits)
    bcodes, bscales = np_brute(fmt, bits)
    assert np.array_equal(scales, bscales)
    assert np.array_equal(codes, bcodes)


def test_f32_inputs_against_enumeration(oracle_mod):
    """binary32 inputs (the requantize leg): 24-bit significands, including values a hair above
    and below rounding midpoints."""
    rng = np.random.default_rng(7)
    for (x, y) in HOT_ELEMENTS + [(1, 3)]:
        fmt = oracle_mod.Format(x, y, 8, 8)
        book = np.array([float(q) for q in codebook_from_definition(x, y)])
        mids = (book[:-1] + book[1:]) / 2
        rowsv = []
        for k in (-20, 0, 3):
            for mval in mids:
                base = np.float32(mval * 2.0 ** k)
                near = [np.nextafter(base, np.float32(0)), base, np.nextafter(base, np.float32(np.inf))]
                rowsv.append([book[-1] * 2.0 ** k] + near + [-near[0], -near[2], 0, 0])
        xin = np.array(rowsv, dtype=np.float32)
        xin = np.concatenate([xin, (rng.standard_normal((4096, 8)) *
                                    np.exp(rng.standard_normal((4096, 1)) * 3)).astype(np.float32)])
        codes, scales = oracle_mod.quantize_f32(fmt, xin)
        # enumeration in float64 on the float32 values
        a = np.abs(xin.astype(np.float64))
        m = a.max(axis=1)
        beta = 2 ** (x - 1) - 1
        emax = 2 ** x - 1 - beta
        pow2 = np.array([2.0 ** k for k in range(-160, 130)])
        E = np.searchsorted(pow2, m, side="right") - 1 - 160
        sc = np.clip(E - emax + 127, 0, 254)
        p = a / (2.0 ** (sc - 127.0))[:, None]
        d = np.abs(p[..., None] - book)
        best = d.argmin(-1)
        nxt = np.minimum(best + 1, len(book) - 1)
        tie = (np.take_along_axis(d, nxt[..., None], -1)[..., 0] ==
               np.take_along_axis(d, best[..., None], -1)[..., 0]) & (nxt != best)
        best = np.where(tie & (best % 2 == 1), nxt, best)
        want = (np.signbit(xin).astype(np.int64) << (x + y)) | best
        assert np.array_equal(scales[:, 0], sc.astype(np.uint8))
        assert np.array_equal(codes, want.astype(np.uint8))


# ----------------------------------------------------------------------- invariants ---------

@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
def test_representable_inputs_round_trip(oracle_mod, x, y):
    """Inputs of the form magnitude * 2^k whose block maximum sits in the top binade are
    reproduced exactly by quantize -> dequantize."""
    book = read_codebooks().get((x, y)) or [float(q) for q in codebook_from_definition(x, y)]
    rng = np.random.default_rng(5)
    B = 32
    fmt = oracle_mod.Format(x, y, B, 8)
    T, nb = 16, 8
    ks = rng.integers(-120, 100, size=(T, nb))
    idx = rng.integers(0, len(book), size=(T, nb, B))
    idx[:, :, 0] = len(book) - 1 - rng.integers(0, 2 ** y, size=(T, nb))   # top binade
    sign = rng.choice([-1.0, 1.0], size=(T, nb, B))
    vals = (np.array(book)[idx] * sign * (2.0 ** ks)[:, :, None]).reshape(T, nb * B).astype(np.float32)
    bits = workloads.f32_to_bf16_bits(vals)
    assert np.array_equal(workloads.bf16_bits_to_f32(bits), vals)
    codes, scales = oracle_mod.quantize_bf16(fmt, bits)
    back = oracle_mod.dequantize(fmt, codes, scales)
    assert np.array_equal(back.view(np.uint32), vals.view(np.uint32))
    assert np.array_equal(scales, (ks + 127).astype(np.uint8))


def test_scale_rule_and_error_bound(oracle_mod):
    """2^emax <= max|p| < 2^(emax+1) when the clamp is idle; |p - q| <= half a step of the
    format at p unless saturated; magnitudes are monotone in |v|."""
    w = workloads.small_like(workloads.CONFIGS[3], 64, 2048)
    bits = workloads.partial_bf16(w, 0)
    v = workloads.bf16_bits_to_f32(bits).astype(np.float64)
    for (x, y) in HOT_ELEMENTS:
        fmt = oracle_mod.Format(x, y, 32, 8)
        beta = 2 ** (x - 1) - 1
        emax = 2 ** x - 1 - beta
        maxval = 2.0 ** emax * (2 - 2.0 ** -y)
        codes, scales = oracle_mod.quantize_bf16(fmt, bits)
        sc = 2.0 ** (scales.astype(np.float64) - 127)
        p = np.abs(v).reshape(64, -1, 32) / sc[:, :, None]
        pmax = p.max(axis=2)
        assert np.all((pmax >= 2.0 ** emax) & (pmax < 2.0 ** (emax + 1)))
        q = np.abs(oracle_mod.dequantize(fmt, codes, np.full_like(scales, 127)).astype(np.float64)
                   ).reshape(p.shape)
        binade = np.maximum(np.floor(np.log2(np.maximum(p, 1e-300))), 1 - beta)
        half_step = 2.0 ** (binade - y) / 2
        ok = (np.abs(p - q) <= half_step) | ((p > maxval) & (q == maxval))
        assert ok.all()
        # monotone: sort by |p| within the tensor and check magnitudes never decrease
        order = np.argsort(p.ravel(), kind="stable")
        assert np.all(np.diff(q.ravel()[order]) >= 0)
        # signs are copied
        assert np.array_equal(codes >> (x + y), (bits >> 15).astype(np.uint8))


def test_values_between_maxval_and_next_binade_saturate(oracle_mod):
    for (x, y) in ALL_ELEMENTS:
        fmt = oracle_mod.Format(x, y, 8, 8)
        emax = 2 ** x - 1 - (2 ** (x - 1) - 1)
        maxval = 2.0 ** emax * (2 - 2.0 ** -y)
        hi = np.float32(2.0 ** (emax + 1) * (1 - 2.0 ** -8))       # largest bf16 below 2^(emax+1)
        xin = np.array([[hi, maxval, -hi, 0, 0, 0, 0, 0]], np.float32)
        codes, scales = oracle_mod.quantize_bf16(fmt, workloads.f32_to_bf16_bits(xin))
        top = 2 ** (x + y) - 1
        assert scales[0, 0] == 127
        assert list(codes[0, :3]) == [top, top, top | (1 << (x + y))]


def test_zero_subnormal_and_clamped_blocks(oracle_mod):
    fmt = oracle_mod.Format(2, 1, 8, 8)
    z = np.zeros((1, 8), np.uint16)
    z[0, 3] = 0x8000
    codes, scales = oracle_mod.quantize_bf16(fmt, z)
    assert scales[0, 0] == 0 and list(codes[0]) == [0, 0, 0, 8, 0, 0, 0, 0]
    # bf16 subnormals: value = fr * 2^-133; with scale 2^-127 p = fr / 64
    sub = np.array([[0x007F, 0x0040, 0x0020, 0x0010, 0x8030, 0x0001, 0x0050, 0x0060]], np.uint16)
    codes, scales = oracle_mod.quantize_bf16(fmt, sub)
    assert scales[0, 0] == 0
    # p = 1.984, 1.0, 0.5, 0.25 (tie 0|0.5 -> 0), -0.75 (tie 0.5|1 -> 1.0 = code 2), 1/64, 1.25
    # (tie 1|1.5 -> 1 = code 2), 1.5
    assert list(codes[0]) == [4, 2, 1, 0, 8 | 2, 0, 2, 3]
    # smallest normal max: biased exponent 1 -> E = -126 -> e = -128 clamps to -127
    one = np.array([[0x00C0, 0, 0, 0, 0, 0, 0, 0]], np.uint16)      # 1.5 * 2^-126
    codes, scales = oracle_mod.quantize_bf16(fmt, one)
    assert scales[0, 0] == 0 and codes[0, 0] == 5                   # p = 3.0 -> code 5
    # largest finite bf16: exponent 254 -> E = 127 -> scale byte 127 + 127 - 2 = 252
    big = np.array([[0x7F7F, 0xFF7F, 0x3F80, 0, 0, 0, 0, 0]], np.uint16)
    codes, scales = oracle_mod.quantize_bf16(fmt, big)
    assert scales[0, 0] == 252 and list(codes[0, :3]) == [7, 15, 0]


def test_non_finite_blocks(oracle_mod):
    fmt = oracle_mod.Format(2, 1, 8, 8)
    for bad in (0x7F80, 0xFF80, 0x7FC0, 0xFFFF):
        b = np.array([[0x3F80, bad, 0xC000, 0, 0, 0, 0, 0], [0x3F80] * 8], np.uint16)
        codes, scales = oracle_mod.quantize_bf16(fmt, b)
        assert scales[0, 0] == 255 and not codes[0].any()
        # 1.0 with e = -2: p = 4.0, the E2M1 code of 4 is 6
        assert scales[1, 0] == 125 and list(codes[1]) == [6] * 8
        out = oracle_mod.dequant_reduce(fmt, [codes], [scales])
        assert np.isnan(out[0]).all() and np.isfinite(out[1]).all()
    x = np.array([[1.0, np.inf, -2, 0, 0, 0, 0, 0]], np.float32)
    codes, scales = oracle_mod.quantize_f32(fmt, x)
    assert scales[0, 0] == 255 and not codes.any()


def test_narrow_scales_lose_non_finite_blocks_and_own_raw_replicas_diverge(oracle_mod):
    """Scales narrower than 8 bits have no marker: a block with a NaN stores zero codes and the
    largest scale code and decodes to zeros.  The all-decoded reduction is then finite on every
    worker; the own-raw reduction is NaN on the worker that owns the NaN and finite elsewhere."""
    fmt = oracle_mod.Format(2, 1, 8, 5)
    a = np.array([[0x3F80, 0x7FC0, 0xC000, 0, 0, 0, 0, 0] + [0x4000] * 8], np.uint16)   # NaN in block 0
    b = np.array([[0x3F80] * 16], np.uint16)
    ca, sa = oracle_mod.quantize_bf16(fmt, a)
    cb, sb = oracle_mod.quantize_bf16(fmt, b)
    assert sa[0, 0] == 31 and not ca[0, :8].any() and ca[0, 8:].all()
    out = oracle_mod.dequant_reduce(fmt, [ca, cb], [sa, sb])
    assert np.array_equal(out[0, :8], np.ones(8, np.float32)) and np.all(out[0, 8:] == 3.0)
    own0 = oracle_mod.dequant_reduce_own(fmt, 0, a, [ca, cb], [sa, sb])
    own1 = oracle_mod.dequant_reduce_own(fmt, 1, b, [ca, cb], [sa, sb])
    assert np.isnan(own0[0, 1]) and np.isfinite(np.delete(own0[0], 1)).all()
    assert np.isfinite(own1).all() and np.array_equal(own1, out)
    # with an 8-bit scale the marker keeps every replica NaN in that block
    fmt8 = oracle_mod.Format(2, 1, 8, 8)
    ca, sa = oracle_mod.quantize_bf16(fmt8, a)
    cb, sb = oracle_mod.quantize_bf16(fmt8, b)
    for res in (oracle_mod.dequant_reduce(fmt8, [ca, cb], [sa, sb]),
                oracle_mod.dequant_reduce_own(fmt8, 1, b, [ca, cb], [sa, sb])):
        assert np.isnan(res[0, :8]).all() and np.all(res[0, 8:] == 3.0)


def test_narrow_scale_formats_clamp_both_ends(oracle_mod):
    for s in (4, 5, 6, 7):
        fmt = oracle_mod.Format(2, 1, 8, s)
        bias, top = 2 ** (s - 1) - 1, 2 ** s - 1
        x = np.zeros((3, 8), np.float32)
        x[0, 0] = 2.0 ** 100       # far above the scale range: clamps high, element saturates
        x[1, 0] = 2.0 ** -100      # far below: clamps low, element rounds to 0
        x[2, 0] = 6.0              # e = 0
        codes, scales = oracle_mod.quantize_bf16(fmt, workloads.f32_to_bf16_bits(x))
        assert list(scales[:, 0]) == [top, 0, bias]
        assert list(codes[:, 0]) == [7, 0, 7]


# ----------------------------------------------------------------------- packing ------------

@pytest.mark.parametrize("x,y", ALL_ELEMENTS)
def test_pack_is_a_little_endian_bit_stream(oracle_mod, x, y):
    fmt = oracle_mod.Format(x, y, 8, 8)
    b = fmt.bits
    rng = np.random.default_rng(b)
    codes = rng.integers(0, 2 ** b, size=(5, 64), dtype=np.uint8)
    packed = oracle_mod.pack(fmt, codes)
    for t in range(5):
        stream = sum(int(c) << (j * b) for j, c in enumerate(codes[t]))     # big-int bit stream
        assert bytes(packed[t]) == stream.to_bytes(64 * b // 8, "little")
    assert np.array_equal(oracle_mod.unpack(fmt, packed, 64), codes)
    if b == 4:
        assert np.array_equal(packed, codes[:, 0::2] | (codes[:, 1::2] << 4))


# ----------------------------------------------------------------------- reduction ----------

def _quantized_ranks(oracle_mod, fmt, tp, T, H, seed):
    w = workloads.Workload("t", tp, T, H, seed, n_outlier=2, outlier_mult=(20.0, 100.0))
    cs, ss = [], []
    for r in range(tp):
        c, s = oracle_mod.quantize_bf16(fmt, workloads.partial_bf16(w, r))
        cs.append(c)
        ss.append(s)
    return cs, ss


def test_reduce_is_a_left_fold_of_float32_adds(oracle_mod):
    books = read_codebooks()
    for (x, y) in HOT_ELEMENTS:
        fmt = oracle_mod.Format(x, y, 32, 8)
        cs, ss = _quantized_ranks(oracle_mod, fmt, 8, 32, 512, 11)
        out = oracle_mod.dequant_reduce(fmt, cs, ss)
        # decode with the golden code book and numpy, then fold with float32 adds
        mags = np.array(books[(x, y)])
        ds = []
        for c, s in zip(cs, ss):
            val = mags[c & (2 ** (x + y) - 1)] * np.where(c >> (x + y), -1.0, 1.0)
            d = val * np.repeat(2.0 ** (s.astype(np.float64) - 127), 32, axis=1)
            assert np.array_equal(d.astype(np.float32).astype(np.float64), d)   # exact in fp32
            ds.append(d.astype(np.float32))
        acc = ds[0].copy()
        for d in ds[1:]:
            acc = (acc + d).astype(np.float32)
        assert np.array_equal(acc.view(np.uint32), out.view(np.uint32))
        # N = 1 is the exact decode
        one = oracle_mod.dequant_reduce(fmt, cs[:1], ss[:1])
        assert np.array_equal(one.view(np.uint32), ds[0].view(np.uint32))
        assert np.array_equal(oracle_mod.dequantize(fmt, cs[0], ss[0]).view(np.uint32),
                              ds[0].view(np.uint32))
        # against a float64 sum: error of a float32 left fold of N terms
        exact = np.sum([d.astype(np.float64) for d in ds], axis=0)
        bound = 8 * 2.0 ** -24 * np.sum([np.abs(d.astype(np.float64)) for d in ds], axis=0)
        assert np.all(np.abs(out - exact) <= bound)
        # a different rank order moves results by rounding only, and does move some
        perm = oracle_mod.dequant_reduce(fmt, cs[::-1], ss[::-1])
        assert np.all(np.abs(perm.astype(np.float64) - exact) <= bound)


def test_reduce_order_matters_when_binades_are_far_apart(oracle_mod):
    """(2^24 + 1) + 1 = 2^24 in binary32 (the tie goes to even twice) but (1 + 1) + 2^24 is
    exact: the fold must run in rank order."""
    fmt = oracle_mod.Format(2, 1, 8, 8)
    one = np.full((1, 8), 2, np.uint8)            # magnitude code 2 = 1.0
    big_s, unit_s = np.full((1, 1), 127 + 24, np.uint8), np.full((1, 1), 127, np.uint8)
    a = oracle_mod.dequant_reduce(fmt, [one, one, one], [big_s, unit_s, unit_s])
    b = oracle_mod.dequant_reduce(fmt, [one, one, one], [unit_s, unit_s, big_s])
    assert np.all(a == np.float32(2.0 ** 24)) and np.all(b == np.float32(2.0 ** 24 + 2))


def test_reduce_with_own_raw_partial_is_the_same_fold_with_one_exact_term(oracle_mod):
    """Profiling: N-1 decoded partials plus the worker's own raw one.  Checked against a numpy
    float32 fold, for every choice of the own rank, and against the all-decoded reduction when
    the own partial happens to be exactly representable."""
    fmt = oracle_mod.Format(2, 1, 32, 8)
    w = workloads.Workload("own", 4, 8, 256, 5, n_outlier=2, outlier_mult=(20.0, 100.0))
    parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
    qs = [oracle_mod.quantize_bf16(fmt, p) for p in parts]
    dec = [oracle_mod.dequantize(fmt, c, s) for c, s in qs]
    for own in range(w.tp):
        cs = [None if r == own else qs[r][0] for r in range(w.tp)]
        ss = [None if r == own else qs[r][1] for r in range(w.tp)]
        got = oracle_mod.dequant_reduce_own(fmt, own, parts[own], cs, ss)
        terms = [workloads.bf16_bits_to_f32(parts[r]) if r == own else dec[r] for r in range(w.tp)]
        acc = terms[0].copy()
        for d in terms[1:]:
            acc = (acc + d).astype(np.float32)
        assert np.array_equal(acc.view(np.uint32), got.view(np.uint32))
        assert not np.array_equal(got, oracle_mod.dequant_reduce(fmt, [q[0] for q in qs], [q[1] for q in qs]))
    # a representable own partial (its own decode) gives the all-decoded result
    rep = workloads.f32_to_bf16_bits(dec[1])
    assert np.array_equal(workloads.bf16_bits_to_f32(rep), dec[1])
    a = oracle_mod.dequant_reduce_own(fmt, 1, rep, [q[0] for q in qs], [q[1] for q in qs])
    b = oracle_mod.dequant_reduce(fmt, [q[0] for q in qs], [q[1] for q in qs])
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_reduce_starts_from_rank0_value_not_from_zero(oracle_mod):
    fmt = oracle_mod.Format(2, 1, 8, 8)
    negz = np.full((1, 8), 8, np.uint8)          # every code is -0
    s = np.full((1, 1), 127, np.uint8)
    out = oracle_mod.dequant_reduce(fmt, [negz, negz, negz], [s, s, s])
    assert np.all(out == 0) and np.all(np.signbit(out))
    # scale byte 0 is 2^-127, below the float32 normal range: 0.5 * 2^-127 = 2^-128 must survive
    c = np.full((1, 8), 1, np.uint8)
    s0 = np.zeros((1, 1), np.uint8)
    out = oracle_mod.dequant_reduce(fmt, [c, c], [s0, s0])
    assert np.all(out == np.float32(2.0 ** -127))


def test_round_to_bf16_matches_library_conversion(oracle_mod):
    import torch
    rng = np.random.default_rng(3)
    u = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    edge = np.array([0x00000000, 0x80000000, 0x3F808000, 0x3F818000, 0x3F808001, 0x7F7FFFFF,
                     0x7F7F8000, 0x00008000, 0x00018000, 0x007F8000, 0x7F800000, 0xFF800000,
                     0x00000001, 0x80000001, 0x3F80FFFF], dtype=np.uint32)
    x = np.concatenate([u, edge]).view(np.float32)
    got = oracle_mod.round_to_bf16(x)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all(got[nan] == 0x7FC0)


@pytest.mark.parametrize("x,y,f8", [(1, 2, "float8_e5m2"), (2, 2, "float8_e5m2"), (3, 2, "float8_e5m2"),
                                    (1, 3, "float8_e4m3fn"), (2, 3, "float8_e4m3fn")])
def test_element_rounding_against_library_float8_casts(oracle_mod, x, y, f8):
    """A format with 2 (3) mantissa bits is the low end of the code space of the 8-bit float
    E5M2 (E4M3): scaled so that the smallest normals coincide, rounding to the element format and
    the library's round-to-nearest-even cast to that 8-bit float pick the same code wherever the
    element format does not saturate.  This pins rounding, ties and subnormals of the oracle to
    a routine it shares nothing with."""
    import torch
    dt = getattr(torch, f8)
    hw_bias = 15 if f8 == "float8_e5m2" else 7
    B = 32
    fmt = oracle_mod.Format(x, y, B, 8)
    beta = 2 ** (x - 1) - 1
    magmask = 2 ** (x + y) - 1
    rng = np.random.default_rng(100 * x + y)
    # float32 inputs with full 24-bit significands, block maxima in assorted binades
    v = (rng.standard_normal((64, 16 * B)) * np.exp2(rng.integers(-20, 20, size=(64, 1)))).astype(np.float32)
    v[:, ::7] *= np.float32(0.03125)                       # plenty of values in the subnormal range
    codes, scales = oracle_mod.quantize_f32(fmt, v)
    e = scales.astype(np.int64) - 127
    p = v.astype(np.float64) * np.exp2(-np.repeat(e, B, axis=1).astype(np.float64))   # exact
    q = torch.from_numpy(p * 2.0 ** (beta - hw_bias)).to(torch.float32)               # exact: power of two
    byte = q.to(dt).view(torch.uint8).numpy()
    lib_mag, lib_sign = byte & 0x7F, byte >> 7
    mag, sign = codes & magmask, codes >> (x + y)
    assert np.array_equal(sign, lib_sign)
    inside = lib_mag <= magmask
    assert inside.mean() > 0.9
    assert np.array_equal(mag[inside], lib_mag[inside])
    assert np.all(mag[~inside] == magmask)                 # beyond the element format: saturated


# ----------------------------------------------------------------- quality proxy ------------

def test_uncompressed_sum_is_a_float32_left_fold(oracle_mod):
    rng = np.random.default_rng(11)
    parts = [workloads.f32_to_bf16_bits((rng.standard_normal((7, 96)) * 10.0 ** rng.integers(-3, 4))
                                        .astype(np.float32)) for _ in range(5)]
    got = oracle_mod.sum_bf16(parts)
    acc = workloads.bf16_bits_to_f32(parts[0]).copy()
    for p in parts[1:]:
        acc = (acc + workloads.bf16_bits_to_f32(p)).astype(np.float32)      # numpy float32 adds
    assert np.array_equal(got.view(np.uint32), acc.view(np.uint32))
    exact = sum(workloads.bf16_bits_to_f32(p).astype(np.float64) for p in parts)
    assert np.all(np.abs(got - exact) <= 5 * 2.0 ** -24 * sum(np.abs(workloads.bf16_bits_to_f32(p)) for p in parts))
    # the order of the adds shows: 2^24 + 1 + 1 against 1 + 1 + 2^24
    big, one = np.array([[0x4B80]], np.uint16), np.array([[0x3F80]], np.uint16)
    assert oracle_mod.sum_bf16([big, one, one])[0, 0] == 2.0 ** 24
    assert oracle_mod.sum_bf16([one, one, big])[0, 0] == 2.0 ** 24 + 2


def test_sqnr_closed_forms(oracle_mod):
    """SQNR pins: a relative error of 2^-k everywhere is 20 k log10(2) dB; an all-zero test
    tensor is 0 dB; equal tensors are +inf; an error that is orthogonal to the signal and a
    quarter of its power is 10 log10(4) dB."""
    rng = np.random.default_rng(12)
    ref = (rng.integers(1, 2 ** 12, size=(33, 64)) * rng.choice([-1.0, 1.0], size=(33, 64))).astype(np.float32)
    for k in (1, 4, 9):
        test = (ref.astype(np.float64) * (1.0 + 2.0 ** -k)).astype(np.float32)   # exact: 12 + k bits
        assert abs(oracle_mod.sqnr_db(ref, test) - 20.0 * k * np.log10(2.0)) < 1e-9
    assert abs(oracle_mod.sqnr_db(ref, np.zeros_like(ref))) < 1e-12
    assert oracle_mod.sqnr_db(ref, ref) == float("inf")
    a = np.zeros((2, 8), np.float32)
    a[0] = 4.0
    b = a.copy()
    b[1] = 2.0                                   # noise power 8 * 4, signal power 8 * 16
    assert abs(oracle_mod.sqnr_db(a, b) - 10.0 * np.log10(4.0)) < 1e-12
    # not symmetric: the reference is the first argument
    assert abs(oracle_mod.sqnr_db(b, a) - 10.0 * np.log10(5.0)) < 1e-12


def oracle_pipeline_sqnr(oracle_mod, w, x, y, B, s, parts=None):
    fo = oracle_mod.Format(x, y, B, s)
    parts = parts if parts is not None else [workloads.partial_bf16(w, r) for r in range(w.tp)]
    cs, ss = zip(*[oracle_mod.quantize_bf16(fo, p) for p in parts])
    return oracle_mod.sqnr_db(oracle_mod.sum_bf16(parts), oracle_mod.dequant_reduce(fo, list(cs), list(ss)))


def test_quality_trends_of_the_parameter_list(oracle_mod):
    """The three trends the paper's perplexity tables show (Model Evaluation, Table 1; appendix
    ablation table), on the quality proxy of the synthetic partials: a mantissa bit buys 5 to 7 dB
    with a 2- or 3-bit exponent (3 to 4 dB on the uniform grids of a 1-bit exponent, where the
    block's range rather than the step limits the error); smaller blocks are never worse; the
    scale width does not matter down to E5M0."""
    w = workloads.CONFIGS[1]
    parts = [workloads.partial_bf16(w, r) for r in range(w.tp)]
    q = lambda x, y, B=32, s=8: oracle_pipeline_sqnr(oracle_mod, w, x, y, B, s, parts)
    # (1) one more mantissa bit at the same exponent width
    for x, ys, lo, hi in ((1, (1, 2, 3, 4), 2.5, 6.0), (2, (1, 2, 3), 4.5, 7.5), (3, (1, 2), 4.5, 7.5)):
        vals = [q(x, y) for y in ys]
        for a, b in zip(vals, vals[1:]):
            assert lo < b - a < hi, (x, ys, vals)
    # (2) block 8 >= block 16 >= block 32 (the paper's Table 1: perplexity falls with block size)
    for (x, y) in HOT_ELEMENTS + [(1, 2)]:
        b8, b16, b32 = q(x, y, 8), q(x, y, 16), q(x, y, 32)
        assert b8 >= b16 - 0.05 and b16 >= b32 - 0.05, (x, y, b8, b16, b32)
    assert q(2, 1, 8) > q(2, 1, 32) + 0.5
    # (3) scale formats E8M0 ... E5M0 give the same result (appendix ablation: identical rows)
    for (x, y) in HOT_ELEMENTS:
        ref = q(x, y, 32, 8)
        for s in (7, 6, 5):
            assert abs(q(x, y, 32, s) - ref) < 1e-9, (x, y, s)
    # E2M1 / E2M2 / E3M2 at block 32 keep their order
    assert q(2, 1) < q(2, 2) < q(3, 2)


# ----------------------------------------------------------------------- generators ---------

def test_workload_generators_are_seeded_and_shaped():
    w = workloads.CONFIGS[1]
    a = workloads.partial_bf16(w, 0)
    b = workloads.partial_bf16(w, 0)
    c = workloads.partial_bf16(w, 1)
    assert a.shape == (128, 1024) and a.dtype == np.uint16
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    _, idx, mult = workloads.channel_profile(w)
    assert len(idx) == 4 and np.all(mult[idx] == 50.0) and mult.sum() == 1024 - 4 + 200
    v = np.abs(workloads.bf16_bits_to_f32(a))
    rest = np.delete(np.arange(1024), idx)
    assert v[:, idx].mean() > 10 * v[:, rest].mean()                # outlier channels stand out
    assert np.array_equal(workloads.partial_bf16(w, 1, slice(5, 9)), c[5:9])
    import torch
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(workloads.f32_to_bf16_bits(x),
                          torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
