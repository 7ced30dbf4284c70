"""Pins of the CPU oracle against things other than itself: the paper's printed worked example,
brute force, closed forms, exact rational arithmetic and numpy's own fp16 / fp64 routines."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16(bits):
    return np.array(bits, dtype=np.uint16).view(np.float16)


def f16_exact(bits: int) -> Fraction:
    """Value of an fp16 bit pattern as an exact rational, from the IEEE definition."""
    s, e, m = bits >> 15, (bits >> 10) & 31, bits & 1023
    assert e != 31
    v = Fraction(m, 1 << 24) if e == 0 else Fraction(1024 + m, 1024) * Fraction(2) ** (e - 15)
    return -v if s else v


def read_table2():
    rows, avg = [], None
    with open(os.path.join(GOLDEN, "table2_example.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            if parts[0] == "avg":
                avg = [float(v) for v in parts[1:]]
            else:
                rows.append([float(v) for v in parts])
    return np.array(rows), avg


# ---------------------------------------------------------------- Table 2 (worked example)
@pytest.mark.parametrize("L,qcol,wcol,avg_i", [(15, 1, 2, 0), (7, 3, 4, 1), (10, 5, 6, 2)])
def test_table2_levels_and_reconstruction(orc, L, qcol, wcol, avg_i):
    tab, avg = read_table2()
    w = tab[:, 0].astype(np.float32)
    q, s_bits, o_bits = orc.quantize_block(w, L)
    assert q.tolist() == tab[:, qcol].astype(int).tolist()
    wq = np.array([orc.dequant_value(int(v), s_bits, o_bits) for v in q], np.uint16).view(np.float16).astype(np.float64)
    # printed to three decimals; the fp16 header moves a value by at most ~1e-3 at this magnitude
    assert np.max(np.abs(wq - tab[:, wcol])) <= 1.6e-3
    err = np.mean(np.abs(wq - tab[:, 0]))
    assert abs(err - avg[avg_i]) < 1e-3


def test_table2_35bit_is_exact(orc):
    tab, _ = read_table2()
    q, s_bits, o_bits = orc.quantize_block(tab[:, 0].astype(np.float32), 10)
    assert f16([s_bits])[0] == np.float16(0.25) and f16([o_bits])[0] == np.float16(-1.0)
    wq = f16([orc.dequant_value(int(v), s_bits, o_bits) for v in q]).astype(np.float64)
    assert wq.tolist() == tab[:, 6].tolist()
    # Eq.4 on the example's levels
    codes = [orc.pair_encode(int(q[2 * i]), int(q[2 * i + 1])) for i in range(6)]
    assert codes == [0, 24, 37, 50, 85, 109]


def test_table2_ideal_parameters_match_three_decimals():
    """Eq.1/Eq.2 in exact arithmetic (no fp16 header) reproduce the printed w' to the printed digits:
    shows that reading Eq.2 as q*scale+offset with scale=(max-min)/L is the table's arithmetic."""
    tab, avg = read_table2()
    w = [Fraction(str(v)) for v in tab[:, 0]]
    for L, qcol, wcol, a in [(15, 1, 2, avg[0]), (7, 3, 4, avg[1]), (10, 5, 6, avg[2])]:
        mn, mx = min(w), max(w)
        errs = []
        for i, v in enumerate(w):
            t = (v - mn) / (mx - mn) * L
            q = int(t + Fraction(1, 2))
            assert q == int(tab[i, qcol])
            wp = Fraction(q, L) * (mx - mn) + mn
            assert abs(float(wp) - tab[i, wcol]) < 5.1e-4
            errs.append(abs(wp - v))
        assert abs(float(sum(errs) / len(errs)) - a) < 5.1e-4


# ---------------------------------------------------------------- Eq.1/3: brute force and bounds
def _cases(rng):
    for L in (1, 3, 7, 10, 15, 255):
        for n in (1, 2, 5, 12, 32, 64):
            for sigma in (1e-3, 0.02, 3.0):
                yield L, (rng.standard_normal(n) * sigma).astype(np.float32)


def test_levels_minimise_reconstruction_error_brute_force(orc):
    rng = np.random.default_rng(7)
    for L, w in _cases(rng):
        q, s_bits, o_bits = orc.quantize_block(w, L)
        s, o = f16_exact(s_bits), f16_exact(o_bits)
        assert q.min() >= 0 and q.max() <= L
        if s == 0:
            assert not q.any()
            continue
        for wi, qi in zip(w, q):
            wv = Fraction(float(wi))
            errs = [abs(wv - (o + j * s)) for j in range(L + 1)]
            # the encoder works in fp32: allow a few ulp of (w-o)/s around an exact tie
            assert errs[int(qi)] <= min(errs) + s * Fraction(L, 1 << 21)


def test_half_step_error_bound(orc):
    rng = np.random.default_rng(8)
    for L, w in _cases(rng):
        q, s_bits, o_bits = orc.quantize_block(w, L)
        s, o = f16_exact(s_bits), f16_exact(o_bits)
        mn, mx = Fraction(float(w.min())), Fraction(float(w.max()))
        # delta: how far the fp16 header moved the two ends of the level grid
        delta = max(Fraction(0), o - mn, mx - (o + L * s))
        for wi, qi in zip(w, q):
            rec = o + int(qi) * s
            assert abs(Fraction(float(wi)) - rec) <= s / 2 + delta + s * Fraction(L, 1 << 21)


def test_end_levels_present_and_level_count(orc):
    rng = np.random.default_rng(9)
    for fmt, L in ((orc.Q3H_B64, 10), (orc.Q4_B64, 15), (orc.Q4_B32, 15), (orc.Q8_B64, 255), (orc.Q8_B32, 255),
                   (orc.Q6_B64, 63), (orc.Q5_B64, 31), (orc.Q3_B32, 7), (orc.Q2_B32, 3)):
        assert orc.levels(fmt) == L + 1
        w = (rng.standard_normal((16, 256)) * 0.02).astype(np.float32)
        q, s, o = orc.quantize(fmt, w)
        Bs = orc.block_size(fmt)
        qb = q.reshape(-1, Bs)
        wb = w.reshape(-1, Bs)
        assert qb.max() <= L
        # zero-centred blocks: the minimum maps to level 0 and the maximum to level L
        assert (qb[np.arange(len(qb)), wb.argmin(1)] == 0).all()
        assert (qb[np.arange(len(qb)), wb.argmax(1)] == L).all()
    # 3.5-bit: exactly 11 distinct levels occur (Eq.3), all of them on a ramp
    ramp = np.linspace(-1, 1, 64, dtype=np.float32)
    q, _, _ = orc.quantize_block(ramp, 10)
    assert sorted(set(q.tolist())) == list(range(11))


def test_round_is_half_away_from_zero(orc):
    # scale 1, offset 0 exactly: t = w, so 0.5 -> 1, 1.5 -> 2, 2.5 -> 3 (ties-to-even would give 0, 2, 2)
    w = np.array([0, 0.5, 1.5, 2.5, 3.49, 3.51, 10], np.float32)
    q, s_bits, o_bits = orc.quantize_block(w, 10)
    assert f16([s_bits])[0] == 1 and f16([o_bits])[0] == 0
    assert q.tolist() == [0, 1, 2, 3, 3, 4, 10]


def test_constant_block_and_signed_zero(orc):
    q, s_bits, o_bits = orc.quantize_block(np.full(64, 0.37, np.float32), 10)
    assert not q.any() and s_bits == 0
    assert f16([o_bits])[0] == np.float16(0.37)
    assert orc.dequant_value(0, s_bits, o_bits) == o_bits            # w' = offset
    q, s_bits, o_bits = orc.quantize_block(np.array([-0.0] * 8, np.float32), 15)
    assert o_bits == 0 and s_bits == 0                               # -0 stored as +0
    # range below the smallest fp16 subnormal: scale underflows to zero -> all levels 0
    q, s_bits, _ = orc.quantize_block(np.array([1.0, 1.0 + 1.2e-7], np.float32), 10)
    assert s_bits == 0 and not q.any()


def test_power_of_two_rescaling_leaves_levels_unchanged(orc):
    rng = np.random.default_rng(10)
    w = (rng.standard_normal(64) * 0.02).astype(np.float32)
    for L in (10, 15, 255):
        q0, s0, o0 = orc.quantize_block(w, L)
        for e in (-1, 2, 7):      # stays inside fp16's normal range, where scaling by 2^e is exact
            q1, s1, o1 = orc.quantize_block(w * np.float32(2.0 ** e), L)
            assert q1.tolist() == q0.tolist()
            assert f16_exact(s1) == f16_exact(s0) * Fraction(2) ** e
            assert f16_exact(o1) == f16_exact(o0) * Fraction(2) ** e


def test_blocks_run_along_rows(orc):
    """A block is Bs consecutive elements of a row: changing one element only changes its own block."""
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((3, 192)) * 0.02).astype(np.float32)
    q0, s0, o0 = orc.quantize(orc.Q3H_B64, w)
    w2 = w.copy()
    w2[1, 70] = 5.0                     # row 1, second block of that row
    q1, s1, o1 = orc.quantize(orc.Q3H_B64, w2)
    changed = (q0 != q1).reshape(3, 3, 64).any(-1)
    assert changed.tolist() == [[False] * 3, [False, True, False], [False] * 3]
    assert (s0 != s1).tolist() == changed.tolist()
    # per-block result equals the single-block routine
    qb, sb, ob = orc.quantize_block(w2[1, 64:128], 10)
    assert qb.tolist() == q1[1, 64:128].tolist() and sb == s1[1, 1] and ob == o1[1, 1]


# ---------------------------------------------------------------- Eq.4 / Eq.5
def test_pair_code_round_trip_all_121(orc):
    seen = set()
    for a in range(11):
        for b in range(11):
            c = orc.pair_encode(a, b)
            assert 0 <= c <= 120 < 128           # seven bits suffice
            assert c == a * 11 + b
            assert orc.pair_decode(c) == (a, b)
            seen.add(c)
    assert seen == set(range(121))


# ---------------------------------------------------------------- Table 3: bit budget
def test_bits_per_weight_match_table3(orc):
    with open(os.path.join(GOLDEN, "table3_bits_per_weight.txt")) as fh:
        rows = [l.split() for l in fh if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for name, bs, bpw in rows:
        fmt = orc.FORMATS[name]
        assert orc.block_size(fmt) == int(bs)
        for r, c in ((1, 64), (7, 4096), (4096, 11008)):
            assert Fraction(orc.packed_bytes(fmt, r, c) * 8, r * c) == Fraction(bpw)
    assert orc.packed_bytes(orc.Q3H_B64, 4, 100) == -1          # cols not a multiple of the block
    # the 2-bit format is named in Section 1's feature list only; with the 3-bit format's block size it stores 3 bits/weight
    assert orc.block_size(orc.Q2_B32) == 32 and orc.packed_bytes(orc.Q2_B32, 7, 4096) * 8 == 3 * 7 * 4096


# ---------------------------------------------------------------- fp16 conversions vs numpy
def test_f16_to_f32_all_patterns(orc):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = orc.f16_bits_to_f32(bits)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(ref)], ref.view(np.uint32)[~np.isnan(ref)])
    assert np.isnan(got[np.isnan(ref)]).all()


def test_f64_to_f16_round_to_nearest_even(orc):
    rng = np.random.default_rng(12)
    vals = [0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001,
            3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5]
    vals += list(rng.standard_normal(4000) * 0.02) + list(rng.standard_normal(2000) * 300)
    vals += list(rng.standard_normal(2000) * 1e-6)
    # exact midpoints between neighbouring fp16 values (ties)
    b = rng.integers(0, 0x7BFF, 3000).astype(np.uint16)
    lo = b.view(np.float16).astype(np.float64)
    hi = (b + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list((lo + hi) / 2) + list(-(lo + hi) / 2)
    vals = np.array(vals, np.float64)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.f64_to_f16_bits(vals), ref)
    v32 = vals.astype(np.float32)
    with np.errstate(over="ignore"):
        ref32 = v32.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.f32_to_f16_bits(v32), ref32)


# ---------------------------------------------------------------- Eq.2: exact, single rounding
def test_dequant_value_is_exact_then_rounded_once(orc):
    rng = np.random.default_rng(13)
    scales = [0x0000, 0x0001, 0x0203, 0x03FF, 0x0400, 0x1C01, 0x211F, 0x2E66, 0x3C00, 0x5555, 0x7000]
    offsets = [0x0000, 0x8001, 0x83FF, 0xA3D7, 0x23D7, 0xB001, 0x3C00, 0xBC01, 0xF000, 0x7000]
    scales += rng.integers(0, 0x7000, 40).tolist()
    offsets += rng.integers(0, 0x7000, 20).tolist() + (rng.integers(0, 0x7000, 20) | 0x8000).tolist()
    for s in scales:
        for o in offsets:
            for q in (0, 1, 2, 5, 9, 10, 15, 128, 254, 255):
                exact = q * f16_exact(s) + f16_exact(o)
                as_f64 = float(exact)
                assert Fraction(as_f64) == exact             # fits a double, so numpy rounds it once
                with np.errstate(over="ignore"):
                    ref = int(np.float64(as_f64).astype(np.float16).view(np.uint16))
                got = orc.dequant_value(q, int(s), int(o))
                if exact == 0:
                    assert got & 0x7FFF == 0
                else:
                    assert got == ref, (hex(s), hex(o), q)


def test_dequant_matrix_and_double_rounding_case(orc):
    # a header for which fp32-then-fp16 rounding differs from rounding the exact value once
    found = None
    for s in range(0x1400, 0x3000, 7):
        for o in (0x3C01, 0xBC01, 0x4401):
            for q in (3, 5, 7, 9, 10):
                exact = q * f16_exact(s) + f16_exact(o)
                once = int(np.float64(float(exact)).astype(np.float16).view(np.uint16))
                twice = int(np.float32(float(exact)).astype(np.float16).view(np.uint16))
                if once != twice:
                    found = (q, s, o, once)
                    break
    if found is not None:
        q, s, o, once = found
        assert orc.dequant_value(q, s, o) == once
    rng = np.random.default_rng(14)
    w = (rng.standard_normal((4, 128)) * 0.02).astype(np.float32)
    for fmt in range(9):
        q, s, o = orc.quantize(fmt, w)
        d = orc.dequant(fmt, q, s, o)
        Bs = orc.block_size(fmt)
        for r in range(4):
            for k in (0, 1, 63, 64, 127):
                assert d[r, k] == orc.dequant_value(int(q[r, k]), int(s[r, k // Bs]), int(o[r, k // Bs]))
        # reconstruction error of the fp16 output stays within half a step plus fp16 rounding
        sv = s.view(np.float16).astype(np.float64).repeat(Bs, axis=1)
        assert np.all(np.abs(d.view(np.float16).astype(np.float64) - w) <= 0.5 * sv + 2e-4)


# ---------------------------------------------------------------- packing
def test_canonical_record_bytes(orc):
    rng = np.random.default_rng(15)
    for fmt, L in ((orc.Q3H_B64, 10), (orc.Q4_B32, 15), (orc.Q4_B64, 15), (orc.Q8_B32, 255), (orc.Q8_B64, 255),
                   (orc.Q6_B64, 63), (orc.Q5_B64, 31), (orc.Q3_B32, 7), (orc.Q2_B32, 3)):
        Bs = orc.block_size(fmt)
        rows, cols = 3, 2 * Bs
        q = rng.integers(0, L + 1, (rows, cols)).astype(np.uint8)
        s = rng.integers(0, 0x7000, (rows, 2)).astype(np.uint16)
        o = rng.integers(0, 0x7000, (rows, 2)).astype(np.uint16)
        rec = orc.pack_canonical(fmt, q, s, o)
        assert rec.size == orc.packed_bytes(fmt, rows, cols)
        per = rec.size // (rows * 2)
        for b in range(rows * 2):
            r, kb = divmod(b, 2)
            blk = bytes(rec[b * per:(b + 1) * per])
            assert int.from_bytes(blk[0:2], "little") == s[r, kb] and int.from_bytes(blk[2:4], "little") == o[r, kb]
            qb = q[r, kb * Bs:(kb + 1) * Bs].tolist()
            if L == 255:
                assert list(blk[4:]) == qb
            elif L == 15:
                assert list(blk[4:]) == [qb[2 * j] | qb[2 * j + 1] << 4 for j in range(Bs // 2)]
            elif L == 10:
                big = sum((qb[2 * j] * 11 + qb[2 * j + 1]) << (7 * j) for j in range(32))
                assert blk[4:] == big.to_bytes(28, "little")
            else:                                   # k-bit levels as one little-endian number, level j at bit k j
                k = (L + 1).bit_length() - 1
                big = sum(v << (k * j) for j, v in enumerate(qb))
                assert blk[4:] == big.to_bytes(Bs * k // 8, "little")
        q2, s2, o2 = orc.unpack_canonical(fmt, rec, rows, cols)
        assert np.array_equal(q2, q) and np.array_equal(s2, s) and np.array_equal(o2, o)


def unpack_device_reference(fmt_name, packed, rows, cols):
    """The device layout read back with numpy, written from the layout's specification
    (include/iflow.h), independently of the oracle's packer."""
    packed = np.asarray(packed, np.uint8)
    if fmt_name == "Q3H_B64":
        nbk = cols // 64
        q = np.zeros((rows, cols), np.uint8)
        s = np.zeros((rows, nbk), np.uint16)
        o = np.zeros((rows, nbk), np.uint16)
        words = packed.view("<u4").reshape(rows, nbk * 8)
        for r in range(rows):
            for kb in range(nbk):
                t, j = divmod(kb, 64)
                n_t = min(64, nbk - 64 * t)
                base = t * 64 * 8
                W = [int(words[r, base + (i // 4) * n_t * 4 + j * 4 + (i % 4)]) for i in range(8)]
                S = O = 0
                for i in range(8):
                    c = [W[i] & 127, (W[i] >> 16) & 127, (W[i] >> 7) & 127, (W[i] >> 23) & 127]
                    for m in range(4):
                        q[r, kb * 64 + 8 * i + 2 * m] = c[m] // 11
                        q[r, kb * 64 + 8 * i + 2 * m + 1] = c[m] % 11
                    S |= ((W[i] >> 14) & 3) << (2 * i)
                    O |= ((W[i] >> 30) & 3) << (2 * i)
                s[r, kb], o[r, kb] = S, O
        return q, s, o
    bits, Bs = int(fmt_name[1]), int(fmt_name[-2:])
    nbk = cols // Bs
    ncode = rows * cols * bits // 8
    hdr = packed[ncode:].view("<u2").reshape(rows, nbk, 2)
    if bits == 8:
        q = packed[:ncode].reshape(rows, cols).copy()
    elif bits != 4:
        # bit planes, least significant first: 6 = 4 + 2, 5 = 4 + 1, 3 = 2 + 1, 2 = 2; in a plane of width w a 32-bit word
        # holds 32/w consecutive weights, even ones in the low half, odd ones in the high half, each in order
        q = np.zeros((rows, cols), np.uint8)
        at, shift = 0, 0
        for w in {6: (4, 2), 5: (4, 1), 3: (2, 1), 2: (2,)}[bits]:
            n = 32 // w
            words = packed[at:at + rows * cols * w // 8].view("<u4").reshape(rows, cols // n)
            for e in range(n):
                field = (words >> ((e // 2) * w + 16 * (e % 2))) & ((1 << w) - 1)
                q[:, e::n] |= (field << shift).astype(np.uint8)
            at += rows * cols * w // 8
            shift += w
        assert at == ncode
    else:
        words = packed[:ncode].view("<u4").reshape(rows, cols // 8)
        q = np.zeros((rows, cols), np.uint8)
        for p, v in enumerate([0, 2, 4, 6, 1, 3, 5, 7]):
            q[:, v::8] = (words >> (4 * p)) & 15
    return q, hdr[:, :, 0].copy(), hdr[:, :, 1].copy()


@pytest.mark.parametrize("name", ["Q3H_B64", "Q4_B32", "Q4_B64", "Q8_B32", "Q8_B64", "Q6_B64", "Q5_B64", "Q3_B32", "Q2_B32"])
@pytest.mark.parametrize("rows,nblocks", [(1, 1), (3, 5), (2, 64), (2, 65), (2, 172)])
def test_device_layout_round_trip(orc, name, rows, nblocks):
    fmt = orc.FORMATS[name]
    L = orc.levels(fmt) - 1
    cols = nblocks * orc.block_size(fmt)
    rng = np.random.default_rng(16 + nblocks)
    q = rng.integers(0, L + 1, (rows, cols)).astype(np.uint8)
    s = rng.integers(0, 0x10000, (rows, nblocks)).astype(np.uint16)
    o = rng.integers(0, 0x10000, (rows, nblocks)).astype(np.uint16)
    dev = orc.pack_device(fmt, q, s, o)
    assert dev.size == orc.packed_bytes(fmt, rows, cols)
    q2, s2, o2 = unpack_device_reference(name, dev, rows, cols)
    assert np.array_equal(q2, q) and np.array_equal(s2, s) and np.array_equal(o2, o)
    # same multiset of information as the canonical record: equal size, and rows stay separable for Q3H
    assert dev.size == orc.pack_canonical(fmt, q, s, o).size
    if name == "Q3H_B64" and rows > 1:
        one = orc.pack_device(fmt, q[1:2], s[1:2], o[1:2])
        assert np.array_equal(dev[one.size:2 * one.size], one)


# ---------------------------------------------------------------- matmul: the definition
def test_gemm_equals_numpy_fp64(orc):
    rng = np.random.default_rng(17)
    w16 = (rng.standard_normal((37, 192)) * 0.02).astype(np.float16)
    x16 = rng.standard_normal((5, 192)).astype(np.float16)
    y = orc.gemm(w16.view(np.uint16), x16.view(np.uint16))
    ref = x16.astype(np.float64) @ w16.astype(np.float64).T          # non-square: a transposed operand fails
    assert y.shape == (5, 37)
    assert np.allclose(y, ref, rtol=1e-13, atol=1e-15)
    y4 = orc.gemm(w16.view(np.uint16), x16.view(np.uint16), threads=4)
    assert np.array_equal(y4, y)                                     # row-parallel: same per-row order
    y32 = orc.gemm_f32(w16.view(np.uint16), x16.view(np.uint16)).view(np.float16).astype(np.float64)
    assert np.max(np.abs(y32 - ref)) <= 2e-3 * np.sqrt(np.mean(ref ** 2))


def test_gemm_special_vectors(orc):
    rng = np.random.default_rng(18)
    w = (rng.standard_normal((6, 128)) * 0.02).astype(np.float32)
    w[2, 64:128] = 0.125                                              # a constant block
    q, s, o = orc.quantize(orc.Q3H_B64, w)
    d = orc.dequant(orc.Q3H_B64, q, s, o)
    dv = d.view(np.float16).astype(np.float64)
    e = np.zeros((1, 128), np.float16)
    e[0, 77] = 1
    assert np.array_equal(orc.gemm(d, e.view(np.uint16))[0], dv[:, 77])          # unit vector picks a column
    ones = np.ones((1, 128), np.float16)
    assert np.allclose(orc.gemm(d, ones.view(np.uint16))[0], dv.sum(1), rtol=1e-14)
    x = rng.standard_normal((1, 128)).astype(np.float16)
    xm = x.copy()
    xm[0, :64] = 0
    # constant block: its contribution is offset * sum(x)
    assert np.isclose(orc.gemm(d, xm.view(np.uint16))[0, 2], 0.125 * xm.astype(np.float64).sum(), rtol=1e-13)
    # linearity in x (exact for a power-of-two multiple)
    assert np.array_equal(orc.gemm(d, (x * np.float16(4)).view(np.uint16)), 4 * orc.gemm(d, x.view(np.uint16)))


def test_qgemm_from_canonical_record(orc):
    rng = np.random.default_rng(19)
    w = (rng.standard_normal((9, 256)) * 0.02).astype(np.float32)
    x = rng.standard_normal((3, 256)).astype(np.float16)
    for fmt in range(9):
        q, s, o = orc.quantize(fmt, w)
        rec = orc.pack_canonical(fmt, q, s, o)
        y, used = orc.qgemm_canonical(fmt, rec, 9, 256, x.view(np.uint16), threads=2)
        ref = x.astype(np.float64) @ orc.dequant(fmt, q, s, o).view(np.float16).astype(np.float64).T
        assert used >= 1 and np.allclose(y, ref, rtol=1e-13, atol=1e-15)
        # quantization error of the product is small against the unquantized product's spread
        full = x.astype(np.float64) @ w.astype(np.float64).T
        bound = {0: 0.01, 1: 0.01, 2: 0.12, 3: 0.15, 4: 0.25, 5: 0.04, 6: 0.08, 7: 0.3, 8: 0.7}[fmt]
        assert np.sqrt(np.mean((y - full) ** 2)) <= bound * np.sqrt(np.mean(full ** 2))


def test_reconstruction_error_follows_table3_order(orc):
    """Table 3's perplexities rise from left to right: Q8, Q6, Q5, Q4_B32, Q4_B64, Q3H, Q3_B32 - and the text states that
    the 3.5-bit format is clearly better than the 3-bit one at the same 4 bits per weight.  On Gaussian weights the
    root-mean-square reconstruction error of Eq.1/Eq.2 (Eq.3 for Q3H) must follow the same order, each step by a clear
    margin; the 2-bit format (not in the table) comes last.  Every format halves the error of a 1-bit-coarser one, about."""
    rng = np.random.default_rng(21)
    w = (rng.standard_normal((64, 1024)) * 0.02).astype(np.float32)
    order = ["Q8_B32", "Q8_B64", "Q6_B64", "Q5_B64", "Q4_B32", "Q4_B64", "Q3H_B64", "Q3_B32", "Q2_B32"]
    err = []
    for name in order:
        fmt = orc.FORMATS[name]
        q, s, o = orc.quantize(fmt, w)
        d = orc.dequant(fmt, q, s, o).view(np.float16).astype(np.float64)
        err.append(np.sqrt(np.mean((d - w) ** 2)))
    for a, b, na, nb in zip(err, err[1:], order, order[1:]):
        assert a < b, (na, nb, a, b)
    e = dict(zip(order, err))
    assert e["Q3_B32"] > 1.15 * e["Q3H_B64"]                       # "significantly" better at equal storage
    assert 1.8 < e["Q5_B64"] / e["Q6_B64"] < 2.3 and 1.8 < e["Q4_B64"] / e["Q5_B64"] < 2.3
    assert 2.0 < e["Q2_B32"] / e["Q3_B32"] < 2.8                   # 7 steps against 3


# ---- the modules around a linear layer (oracle/decode_ops.py): pinned to library routines, closed forms and identities ----
def _bits(x):
    return np.asarray(x, dtype=np.float16).view(np.uint16)


def test_rms_normalization_matches_the_library_routine_and_closed_forms():
    import torch
    from oracle import decode_ops as ops
    rng = np.random.default_rng(77)
    x = rng.standard_normal(1000).astype(np.float16)
    g = (1.0 + 0.1 * rng.standard_normal(1000)).astype(np.float16)
    eps = 1e-5
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (1000,),
                                       weight=torch.from_numpy(g.astype(np.float64)), eps=eps).numpy()
    mine = x.astype(np.float64) * g.astype(np.float64) * ops.rms_scale(_bits(x), eps)
    assert np.max(np.abs(mine - ref)) <= 1e-12 * np.max(np.abs(ref))
    # a constant vector: mean of squares is c^2
    c = np.full(64, 3.0, np.float16)
    assert abs(ops.rms_scale(_bits(c), 0.25) - 1.0 / np.sqrt(9.25)) < 1e-15
    # scaling x by 2 halves the scale when eps is 0 (no dropped mean, no misplaced square)
    assert abs(ops.rms_scale(_bits(2 * x), 0.0) * 2 - ops.rms_scale(_bits(x), 0.0)) < 1e-12
    # the stored product x*g: exact in fp32, so fp32 multiply + one rounding is the same single rounding
    want = (x.astype(np.float32) * g.astype(np.float32)).astype(np.float16).view(np.uint16)
    assert np.array_equal(ops.gain(_bits(x), _bits(g)), want)
    assert np.array_equal(ops.gain(_bits(x), _bits(np.ones(1000, np.float16))), _bits(x))


def test_silu_matches_the_library_routine_and_identities():
    import torch
    from oracle import decode_ops as ops
    rng = np.random.default_rng(78)
    a = (3.0 * rng.standard_normal(2000)).astype(np.float16)
    b = rng.standard_normal(2000).astype(np.float16)
    ref = torch.nn.functional.silu(torch.from_numpy(a.astype(np.float64))).numpy()
    assert np.max(np.abs(ops.silu(a.astype(np.float64)) - ref)) <= 1e-14
    assert ops.silu(0.0) == 0.0
    t = np.linspace(-12, 12, 97)
    assert np.max(np.abs(ops.silu(t) - ops.silu(-t) - t)) < 1e-13          # silu(a) - silu(-a) = a
    assert abs(float(ops.silu(30.0)) - 30.0) < 1e-10 and abs(float(ops.silu(-30.0))) < 1e-10
    want = (ref * b.astype(np.float64)).astype(np.float16).view(np.uint16)
    assert np.array_equal(ops.silu_mul(_bits(a), _bits(b)), want)
    # gate and up are not interchangeable: silu acts on the first argument only
    assert not np.array_equal(ops.silu_mul(_bits(a), _bits(b)), ops.silu_mul(_bits(b), _bits(a)))


def test_fused_gemv_reduces_to_the_plain_product(orc):
    from oracle import decode_ops as ops
    rng = np.random.default_rng(79)
    w = (0.05 * rng.standard_normal((37, 128))).astype(np.float16)
    v = rng.standard_normal(128).astype(np.float16)
    r = rng.standard_normal(37).astype(np.float16)
    plain = orc.gemm(_bits(w), _bits(v))[0]
    assert np.max(np.abs(ops.fused_gemv(_bits(w), _bits(v)) - plain)) < 1e-12
    y = ops.fused_gemv(_bits(w), _bits(v), 0.37, _bits(r))
    assert np.max(np.abs(y - (0.37 * plain + r.astype(np.float64)))) < 1e-12
    # unit vector: column k of W', scaled, plus the residual
    e = np.zeros(128, np.float16); e[5] = 1.0
    assert np.max(np.abs(ops.fused_gemv(_bits(w), _bits(e), 2.0, _bits(r)) - (2.0 * w[:, 5].astype(np.float64) + r.astype(np.float64)))) < 1e-15


def test_gated_gemv_is_the_library_feed_forward_gate(orc):
    import torch
    from oracle import decode_ops as ops
    rng = np.random.default_rng(80)
    wg = (0.3 * rng.standard_normal((29, 192))).astype(np.float16)
    wu = (0.3 * rng.standard_normal((29, 192))).astype(np.float16)
    v = rng.standard_normal(192).astype(np.float16)
    t = lambda a: torch.from_numpy(a.astype(np.float64))
    ref = (torch.nn.functional.silu(torch.nn.functional.linear(t(v), t(wg)) * 0.7) * (torch.nn.functional.linear(t(v), t(wu)) * 0.7)).numpy()
    got = ops.gated_gemv(_bits(wg), _bits(wu), _bits(v), 0.7)
    assert np.max(np.abs(got - ref)) <= 1e-13
    # the two matrices are not interchangeable, and the two plain products composed by hand give the same
    assert np.max(np.abs(got - ops.gated_gemv(_bits(wu), _bits(wg), _bits(v), 0.7))) > 1e-3
    g, u = orc.gemm(_bits(wg), _bits(v))[0], orc.gemm(_bits(wu), _bits(v))[0]
    assert np.max(np.abs(ops.gated_gemv(_bits(wg), _bits(wu), _bits(v)) - ops.silu(g) * u)) <= 1e-13
    # an up projection of all ones times e_k with a gate row of large weights: silu(a) -> a
    e = np.zeros(192, np.float16); e[3] = 1.0
    big = np.zeros((1, 192), np.float16); big[0, 3] = 40.0
    one = np.zeros((1, 192), np.float16); one[0, 3] = 1.0
    assert abs(float(ops.gated_gemv(_bits(big), _bits(one), _bits(e))[0]) - 40.0) < 1e-10


def test_unsplit_layer_definitions_are_the_library_compositions(orc):
    """rms_linear / silu_linear / gated_rms - the definitions GPU parity is judged by - against torch's own rms_norm, linear
    and silu composed in fp64, and against special cases a dropped term, a swapped operand or a misplaced eps would break."""
    import torch
    import torch.nn.functional as F
    from oracle import decode_ops as ops
    rng = np.random.default_rng(81)
    rows, cols = 23, 320
    w = (0.2 * rng.standard_normal((rows, cols))).astype(np.float16)
    w2 = (0.2 * rng.standard_normal((rows, cols))).astype(np.float16)
    x = (2.0 * rng.standard_normal(cols)).astype(np.float16)
    g = (1.0 + 0.3 * rng.standard_normal(cols)).astype(np.float16)
    r = rng.standard_normal(rows).astype(np.float16)
    a = (2.0 * rng.standard_normal(cols)).astype(np.float16)
    t = lambda v: torch.from_numpy(v.astype(np.float64))
    eps = 1e-3
    n_ref = F.rms_norm(t(x), (cols,), weight=t(g), eps=eps)
    assert np.max(np.abs(ops.rms_norm(_bits(x), _bits(g), eps) - n_ref.numpy())) <= 1e-13
    ref = (F.linear(n_ref, t(w)) + t(r)).numpy()
    assert np.max(np.abs(ops.rms_linear(_bits(w), _bits(x), _bits(g), eps, _bits(r)) - ref)) <= 1e-12
    assert np.max(np.abs(ops.rms_linear(_bits(w), _bits(x), _bits(g), eps) - F.linear(n_ref, t(w)).numpy())) <= 1e-12
    ref = (F.linear(F.silu(t(a)) * t(x), t(w)) + t(r)).numpy()
    assert np.max(np.abs(ops.silu_linear(_bits(w), _bits(a), _bits(x), _bits(r)) - ref)) <= 1e-12
    assert np.max(np.abs(ops.silu_linear(_bits(w), _bits(a), _bits(x)) - ops.silu_linear(_bits(w), _bits(x), _bits(a)))) > 1e-3
    ref = (F.silu(F.linear(n_ref, t(w))) * F.linear(n_ref, t(w2))).numpy()
    assert np.max(np.abs(ops.gated_rms(_bits(w), _bits(w2), _bits(x), _bits(g), eps) - ref)) <= 1e-12
    ref = (F.silu(F.linear(t(x), t(w))) * F.linear(t(x), t(w2))).numpy()
    assert np.max(np.abs(ops.gated_rms(_bits(w), _bits(w2), _bits(x)) - ref)) <= 1e-11
    # special cases: unit gains and eps = 0 on a vector of +-c: the normalized vector is sign(x), so W n = W sign(x) exactly
    c = np.where(rng.random(cols) < 0.5, -3.0, 3.0).astype(np.float16)
    ones = np.ones(cols, np.float16)
    want = orc.gemm(_bits(w), _bits(np.sign(c).astype(np.float16)))[0]
    assert np.max(np.abs(ops.rms_linear(_bits(w), _bits(c), _bits(ones), 0.0) - want)) <= 1e-12
    # eps sits under the root, next to the mean: mean x^2 = 9, eps = 7 -> divide by 4
    assert np.max(np.abs(ops.rms_linear(_bits(w), _bits(c), _bits(ones), 7.0) - 0.75 * want)) <= 1e-12
    # scaling x leaves the normalized product unchanged when eps = 0; the gains act per column (not per row)
    assert np.max(np.abs(ops.rms_linear(_bits(w), _bits(2 * x), _bits(g), 0.0) - ops.rms_linear(_bits(w), _bits(x), _bits(g), 0.0))) <= 1e-12
    e5 = np.zeros(cols, np.float16); e5[5] = 1.0
    only5 = ops.rms_linear(_bits(w), _bits(x), _bits(e5), 0.0)
    assert np.max(np.abs(only5 - w[:, 5].astype(np.float64) * float(x[5]) * ops.rms_scale(_bits(x), 0.0))) <= 1e-13
    # the split evaluation order (fp16(x g) in front, scalar behind) agrees with the definition up to that one rounding
    split = ops.fused_gemv(_bits(w), ops.gain(_bits(x), _bits(g)), ops.rms_scale(_bits(x), eps), _bits(r))
    full = ops.rms_linear(_bits(w), _bits(x), _bits(g), eps, _bits(r))
    assert 0 < np.max(np.abs(split - full)) <= 2.0 ** -11 * np.sum(np.abs(w.astype(np.float64)), axis=1).max() * 8.0


# ---- grouped-query attention for one decode step (oracle/attention.py) ----
def test_gqa_decode_matches_the_library_routine_and_special_cases():
    import torch
    from oracle import attention as att
    rng = np.random.default_rng(80)
    n_heads, n_kv, d, max_seq, T = 8, 2, 16, 40, 33
    q = rng.standard_normal((n_heads, d)).astype(np.float16)
    k = rng.standard_normal((n_kv, max_seq, d)).astype(np.float16)
    v = rng.standard_normal((n_kv, max_seq, d)).astype(np.float16)
    scale = 0.3
    got = att.gqa_decode(_bits(q), _bits(k), _bits(v), T, scale)
    # the library's scaled dot-product attention in fp64, keys/values repeated per group (group j serves heads 4j .. 4j+3)
    tq = torch.from_numpy(q.astype(np.float64))[None, :, None, :]
    tk = torch.from_numpy(k[:, :T].astype(np.float64)).repeat_interleave(n_heads // n_kv, dim=0)[None]
    tv = torch.from_numpy(v[:, :T].astype(np.float64)).repeat_interleave(n_heads // n_kv, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)[0, :, 0, :].numpy()
    assert np.max(np.abs(got - ref)) < 1e-12
    # positions past seq_len are never read
    k2, v2 = k.copy(), v.copy()
    k2[:, T:] = 100.0; v2[:, T:] = -100.0
    assert np.array_equal(att.gqa_decode(_bits(q), _bits(k2), _bits(v2), T, scale), got)
    # one cached position: the output is that position's value, whatever the query
    one = att.gqa_decode(_bits(q), _bits(k), _bits(v), 1, scale)
    assert np.array_equal(one, np.repeat(v[:, 0].astype(np.float64), n_heads // n_kv, axis=0))
    # identical keys: uniform weights, the mean of the values
    kc = np.broadcast_to(k[:, :1], k.shape).copy()
    uni = att.gqa_decode(_bits(q), _bits(kc), _bits(v), T, scale)
    assert np.max(np.abs(uni - np.repeat(v[:, :T].astype(np.float64).mean(axis=1), n_heads // n_kv, axis=0))) < 1e-13
    # the order of the cached positions does not matter
    perm = rng.permutation(T)
    kp, vp = k.copy(), v.copy()
    kp[:, :T] = k[:, perm]; vp[:, :T] = v[:, perm]
    assert np.max(np.abs(att.gqa_decode(_bits(q), _bits(kp), _bits(vp), T, scale) - got)) < 1e-13
    # as many groups as heads is multi-head attention: head i with key/value head i
    k8 = rng.standard_normal((n_heads, max_seq, d)).astype(np.float16)
    v8 = rng.standard_normal((n_heads, max_seq, d)).astype(np.float16)
    mha = att.gqa_decode(_bits(q), _bits(k8), _bits(v8), T, scale)
    for i in (0, 5):
        alone = att.gqa_decode(_bits(q[i:i + 1]), _bits(k8[i:i + 1]), _bits(v8[i:i + 1]), T, scale)
        assert np.array_equal(mha[i:i + 1], alone)
    # a dominant score: softmax saturates to the value at that position (no overflow in exp)
    qb = np.zeros((1, d), np.float16); qb[0, 0] = 200.0
    kb = np.zeros((1, 5, d), np.float16); kb[0, 3, 0] = 50.0
    vb = rng.standard_normal((1, 5, d)).astype(np.float16)
    sat = att.gqa_decode(_bits(qb), _bits(kb), _bits(vb), 5, 1.0)
    assert np.all(np.isfinite(sat)) and np.max(np.abs(sat[0] - vb[0, 3].astype(np.float64))) < 1e-12


# ---- rotary position embedding (oracle/rope.py): pinned to complex multiplication and to the properties that define it ----
def test_rope_is_a_complex_rotation_with_the_published_properties():
    from oracle import rope as R
    rng = np.random.default_rng(90)
    d, base = 128, 10000.0
    x = rng.standard_normal((5, d))
    # (1) position 0 is the identity, in both pairings
    for mode in (R.ADJACENT, R.HALVES):
        assert np.array_equal(R.rotate_fp64(x, 0, base, mode), x)
    # (2) the pair (a, b) as the complex number a + ib is multiplied by exp(i p base^(-2i/d)) - numpy's complex exponential
    for p in (1, 7, 1000, 123457):
        z = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * p * base ** (-2.0 * np.arange(d // 2) / d))
        got = R.rotate_fp64(x, p, base, R.ADJACENT)
        assert np.max(np.abs(got[:, 0::2] - z.real)) < 1e-9 and np.max(np.abs(got[:, 1::2] - z.imag)) < 1e-9
    # (3) the first pair turns by p radians (frequency 1), the last one by p * base^(-(d-2)/d)
    e = np.zeros(d); e[0] = 1.0
    r = R.rotate_fp64(e, 3, base, R.ADJACENT)
    assert abs(r[0] - np.cos(3.0)) < 1e-15 and abs(r[1] - np.sin(3.0)) < 1e-15 and not r[2:].any()
    e = np.zeros(d); e[d - 2] = 1.0
    r = R.rotate_fp64(e, 5, base, R.ADJACENT)
    assert abs(r[d - 2] - np.cos(5.0 * base ** (-(d - 2) / d))) < 1e-15
    # (4) rotations compose: position p1 then p2 is position p1 + p2; every pair keeps its length
    a = R.rotate_fp64(R.rotate_fp64(x, 11, base, R.ADJACENT), 30, base, R.ADJACENT)
    assert np.max(np.abs(a - R.rotate_fp64(x, 41, base, R.ADJACENT))) < 1e-12
    r = R.rotate_fp64(x, 999, base, R.ADJACENT)
    assert np.max(np.abs(r[:, 0::2] ** 2 + r[:, 1::2] ** 2 - x[:, 0::2] ** 2 - x[:, 1::2] ** 2)) < 1e-12
    # (5) what it is for: the score of a rotated query and a rotated key depends on the distance of their positions only
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    s1 = R.rotate_fp64(q, 100, base, R.ADJACENT) @ R.rotate_fp64(k, 90, base, R.ADJACENT)
    s2 = R.rotate_fp64(q, 4010, base, R.ADJACENT) @ R.rotate_fp64(k, 4000, base, R.ADJACENT)
    assert abs(s1 - s2) < 1e-9
    # (6) the two pairings are the same rotation on permuted components: (2i, 2i+1) <-> (i, i + d/2)
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])        # adjacent order -> halves order
    h = R.rotate_fp64(x[:, perm], 77, base, R.HALVES)
    assert np.max(np.abs(h - R.rotate_fp64(x, 77, base, R.ADJACENT)[:, perm])) < 1e-15
    # (7) the step: queries come back rotated, row `position` of the caches receives the rotated keys and the plain values,
    #     every other row is left alone
    n_heads, n_kv, max_seq, pos = 4, 2, 6, 3
    q16 = _bits(rng.standard_normal((n_heads, d))); k16 = _bits(rng.standard_normal((n_kv, d))); v16 = _bits(rng.standard_normal((n_kv, d)))
    kc = _bits(rng.standard_normal((n_kv, max_seq, d))).copy(); vc = _bits(rng.standard_normal((n_kv, max_seq, d))).copy()
    kc0, vc0 = kc.copy(), vc.copy()
    qr = R.rope_append(q16, k16, v16, pos, base, R.HALVES, kc, vc)
    assert np.array_equal(qr, R.rope(q16, pos, base, R.HALVES)) and np.array_equal(kc[:, pos], R.rope(k16, pos, base, R.HALVES))
    assert np.array_equal(vc[:, pos], v16)
    keep = np.arange(max_seq) != pos
    assert np.array_equal(kc[:, keep], kc0[:, keep]) and np.array_equal(vc[:, keep], vc0[:, keep])
    # stored values are the exact rotation rounded once: within half an fp16 step of it
    exact = R.rotate_fp64(q16.view(np.float16).astype(np.float64), pos, base, R.HALVES)
    got = qr.view(np.float16).astype(np.float64)
    assert np.all(np.abs(got - exact) <= np.maximum(np.abs(exact), 2.0 ** -14) * 2.0 ** -11)
