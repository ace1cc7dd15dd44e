"""Pins for the oracle's BFP cast / decode (Sec. II-B, Eq. (1)).  CPU only.

The checks here do not reuse the oracle's code: exact rational arithmetic (fractions), the
mathematical invariants of the format, brute-force enumeration over every exponent, and
hand-worked fixtures.
"""
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import kvbfp_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def quant_rows(x, n, p, perm=None):
    """x: float32 [rows][D] -> (mant [rows][D*p/8], exp [rows][D/n]) through the oracle."""
    x = np.asarray(x, dtype=np.float32)
    rows, D = x.shape
    m, e = O.quantize_append(x.reshape(1, rows, 1, D), n, p, rows, 0,
                             perm=None if perm is None else np.asarray(perm, np.int32).reshape(1, D))
    return m[0, 0], e[0, 0]


def codes_of(mant_row, p):
    if p == 8:
        return [int(b) for b in mant_row]
    out = []
    for b in mant_row:
        out += [int(b) & 0xF, int(b) >> 4]
    return out


def frac_rne(v: Fraction) -> int:
    fl = v.numerator // v.denominator
    rem = v - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def pow2(e: int) -> Fraction:
    return Fraction(2) ** e


def brute_block(vals, p):
    """Definition by enumeration: smallest E in 1..255 whose unclamped RNE of the maximum fits."""
    qmax = 2 ** (p - 1) - 1
    fr = [Fraction(float(v)) for v in vals]
    amax = max(abs(f) for f in fr)
    if amax == 0:
        return 0, [0] * len(vals)
    for E in range(1, 256):
        e = E - 127 - (p - 2)
        if frac_rne(amax / pow2(e)) <= qmax:
            break
    else:
        raise AssertionError("no exponent fits")
    codes = []
    for f in fr:
        m = frac_rne(abs(f) / pow2(e))
        # RNE is symmetric, so rounding |x| and restoring the sign equals rounding x
        s = 1 if (f < 0 and m != 0) else 0
        codes.append((s << (p - 1)) | m)
    return E, codes


def f32(v):
    return np.float32(v)


def nextafter32(v, up=True):
    return np.nextafter(np.float32(v), np.float32(np.inf if up else -np.inf))


# --------------------------------------------------------------------------- golden
def read_golden():
    cases = []
    with open(os.path.join(GOLDEN, "bfp_blocks_hand_worked.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p, vals, E, codes = [s.strip() for s in line.split(";")]
            cases.append((int(p), [float(v) for v in vals.split()], int(E),
                          [int(c, 16) for c in codes.split()]))
    return cases


@pytest.mark.parametrize("case", read_golden())
@pytest.mark.parametrize("n", [16, 32])
def test_hand_worked_blocks(case, n):
    p, vals, E, codes = case
    x = np.zeros((1, 128), dtype=np.float32)
    # put the block second in the row so block indexing is exercised too
    x[0, n:n + len(vals)] = vals
    mant, exp = quant_rows(x, n, p)
    got = codes_of(mant[0], p)
    assert int(exp[0, 1]) == E
    assert got[n:n + len(vals)] == codes
    assert all(c == 0 for c in got[:n]) and int(exp[0, 0]) == 0


def test_storage_bits_per_element():
    # Sec. I / Sec. III: BFP12 = 4-bit mantissas + 8-bit exponent per block; footprint
    # p + 8/n bits per element, half of 8-bit storage up to the exponent overhead.
    for n, p, bits in [(32, 4, 4.25), (16, 4, 4.5), (64, 4, 4.125), (128, 4, 4.0625), (16, 8, 8.5)]:
        ms, es = O.plane_shapes(1, 1, 128, n, p, 1)
        assert (ms[-1] + es[-1]) * 8 / 128 == bits
    ms, es = O.plane_shapes(1, 1, 128, 32, 4, 1)
    assert ms[-1] == 64 and es[-1] == 4


# --------------------------------------------------------------------------- brute force (P4)
def tiny_grid(p):
    qmax = 2 ** (p - 1) - 1
    vals = [0.0, -0.0]
    for k in (-3, 0, 5):
        for m in range(0, 2 * qmax + 3):
            vals.append(m * 0.5 * 2.0 ** k)           # integers and exact ties
        b = (qmax + 0.5) * 2.0 ** k                      # the bump boundary and its neighbours
        vals += [b, float(nextafter32(b, True)), float(nextafter32(b, False))]
    vals += [-v for v in vals]
    return [float(f32(v)) for v in vals]


@pytest.mark.parametrize("p", [4, 8])
def test_brute_force_tiny_blocks(p):
    rng = np.random.default_rng(7 + p)
    grid = tiny_grid(p)
    blocks = []
    for _ in range(400):
        k = int(rng.integers(1, 5))
        blocks.append([grid[i] for i in rng.integers(0, len(grid), size=k)])
    # every grid value alone, so each boundary is hit as the block maximum
    blocks += [[v] for v in grid]
    x = np.zeros((len(blocks), 128), dtype=np.float32)
    for r, b in enumerate(blocks):
        x[r, 16:16 + len(b)] = b
    mant, exp = quant_rows(x, 16, p)
    for r, b in enumerate(blocks):
        E, codes = brute_block(b, p)
        got = codes_of(mant[r], p)
        assert int(exp[r, 1]) == E, (b, E, int(exp[r, 1]))
        assert got[16:16 + len(b)] == codes, (b, codes, got[16:16 + len(b)])


@pytest.mark.parametrize("p", [4, 8])
def test_brute_force_extreme_exponents(p):
    # subnormal, smallest normal, largest finite: the b = 8 bit exponent must cover all of fp32
    sub = struct.unpack("<f", struct.pack("<I", 0x00000001))[0]
    big = float(np.finfo(np.float32).max)
    tiny = float(np.finfo(np.float32).tiny)
    blocks = [[sub], [sub * 5, -sub * 3], [tiny, tiny * 0.75], [big], [big, -big / 3],
              [struct.unpack("<f", struct.pack("<I", 0x007FFFFF))[0]], [1e-30, 3e-31], [3e38, 1e38]]
    x = np.zeros((len(blocks), 128), dtype=np.float32)
    for r, b in enumerate(blocks):
        x[r, :len(b)] = b
    mant, exp = quant_rows(x, 16, p)
    for r, b in enumerate(blocks):
        bb = [float(v) for v in x[r, :len(b)]]
        E, codes = brute_block(bb, p)
        assert 1 <= E <= 255
        assert int(exp[r, 0]) == E
        assert codes_of(mant[r], p)[:len(b)] == codes


# --------------------------------------------------------------------------- invariants
def random_blocks(rng, rows, D=128):
    """Mixed magnitudes: Gaussians over many binades, outliers, exact ties, zeros, subnormals."""
    x = rng.standard_normal((rows, D)).astype(np.float32)
    x *= (2.0 ** rng.integers(-140, 120, size=(rows, 1))).astype(np.float32)
    out = rng.integers(0, D, size=rows)
    x[np.arange(rows), out] *= np.float32(37.0)
    x[rng.random((rows, D)) < 0.05] = 0.0
    return x.astype(np.float32)


def exact_decode(codes, E, p):
    qm = 2 ** (p - 1) - 1
    out = []
    for c in codes:
        m = c & qm
        s = c >> (p - 1)
        v = Fraction(m) * pow2(E - 127 - (p - 2))
        out.append(-v if s else v)
    return out


@pytest.mark.parametrize("p", [4, 8])
@pytest.mark.parametrize("n", [16, 32, 64, 128])
def test_half_ulp_bound_and_code_range(n, p):
    # P1: |x - 2^e M| <= 2^(e-1) for every element; codes stay in the symmetric range, -0 never
    # stored; every non-zero block is normalised (max |M| >= 2^(p-2)).
    rng = np.random.default_rng(1000 + n + p)
    x = random_blocks(rng, 48)
    mant, exp = quant_rows(x, n, p)
    qmax = 2 ** (p - 1) - 1
    for r in range(x.shape[0]):
        codes = codes_of(mant[r], p)
        for b in range(128 // n):
            E = int(exp[r, b])
            blk = [Fraction(float(v)) for v in x[r, b * n:(b + 1) * n]]
            cs = codes[b * n:(b + 1) * n]
            if all(v == 0 for v in blk):
                assert E == 0 and all(c == 0 for c in cs)
                continue
            assert 1 <= E <= 255
            mags = [c & qmax for c in cs]
            assert all(c != (1 << (p - 1)) for c in cs), "negative zero stored"
            assert 2 ** (p - 2) <= max(mags) <= qmax or E == 1
            half = pow2(E - 127 - (p - 2) - 1)
            for v, d in zip(blk, exact_decode(cs, E, p)):
                assert abs(v - d) <= half
                assert d == 0 or (d > 0) == (v > 0)


@pytest.mark.parametrize("p", [4, 8])
def test_representable_blocks_round_trip_exactly(p):
    # P2: x_j = 2^f m_j with |m_j| <= q_max comes back exactly (the pair (E, M) may be renormalised)
    rng = np.random.default_rng(5 + p)
    qmax = 2 ** (p - 1) - 1
    rows = 64
    m = rng.integers(-qmax, qmax + 1, size=(rows, 128))
    f = rng.integers(-120, 100, size=(rows, 128 // 16)).repeat(16, axis=1)
    x = (m * 2.0 ** f).astype(np.float32)
    assert np.array_equal(x.astype(np.float64), m * 2.0 ** f)
    mant, exp = O.quantize_append(x.reshape(1, rows, 1, 128), 16, p, rows, 0)
    back = O.dequantize(mant, exp, 128, 16, p, 0, rows)[0, :, 0, :]
    assert np.array_equal(back, x.astype(np.float64))


@pytest.mark.parametrize("p", [4, 8])
@pytest.mark.parametrize("n", [16, 32])
def test_idempotent(n, p):
    # P3: casting the decoded values again reproduces the same bytes
    rng = np.random.default_rng(11 + n + p)
    x = np.clip(random_blocks(rng, 64), -1e30, 1e30).astype(np.float32)
    x[np.abs(x) < 1e-30] = 0                             # keep decoded values inside fp32 normals
    mant, exp = O.quantize_append(x.reshape(1, 64, 1, 128), n, p, 64, 0)
    back = O.dequantize(mant, exp, 128, n, p, 0, 64)
    b32 = back.astype(np.float32)
    assert np.array_equal(b32.astype(np.float64), back)
    mant2, exp2 = O.quantize_append(b32, n, p, 64, 0)
    assert np.array_equal(mant, mant2) and np.array_equal(exp, exp2)


@pytest.mark.parametrize("p", [4, 8])
def test_power_of_two_covariance_and_sign_flip(p):
    # P5: scaling by 2^k moves only the exponent bytes; negating flips only sign bits of non-zero codes
    rng = np.random.default_rng(3 + p)
    x = rng.standard_normal((32, 128)).astype(np.float32)
    x[:, 5] *= 30
    x[rng.random(x.shape) < 0.1] = 0
    m0, e0 = quant_rows(x, 32, p)
    for k in (-40, -3, 9, 60):
        mk, ek = quant_rows(x * np.float32(2.0 ** k), 32, p)
        assert np.array_equal(mk, m0)
        assert np.array_equal(ek.astype(int), np.where(e0 > 0, e0.astype(int) + k, 0))
    mn, en = quant_rows(-x, 32, p)
    assert np.array_equal(en, e0)
    for r in range(x.shape[0]):
        c0, cn = codes_of(m0[r], p), codes_of(mn[r], p)
        sb = 1 << (p - 1)
        for a, b in zip(c0, cn):
            assert b == (a ^ sb if a != 0 else 0)


def test_decode_matches_eq1_on_every_code():
    # every (code, E) pair decodes to (-1)^s * |M| * 2^(E-127-(p-2)); checked in exact rationals
    for p in (4, 8):
        qmax = 2 ** (p - 1) - 1
        ncodes = 2 ** p
        D = 128
        for E in (0, 1, 60, 127, 129, 200, 255):
            row_codes = [(i % ncodes) for i in range(D)]
            if p == 4:
                mant = np.array([row_codes[2 * i] | (row_codes[2 * i + 1] << 4) for i in range(D // 2)],
                                dtype=np.uint8)
            else:
                mant = np.array(row_codes, dtype=np.uint8)
            exp = np.full((D // 16,), E, dtype=np.uint8)
            out = O.dequantize(mant.reshape(1, 1, 1, -1), exp.reshape(1, 1, 1, -1), D, 16, p, 0, 1)[0, 0, 0]
            for j, c in enumerate(row_codes):
                want = Fraction(c & qmax) * pow2(E - 127 - (p - 2)) * (-1 if c >> (p - 1) else 1)
                assert Fraction(float(out[j])) == want


def test_perm_gather_equals_prepermuted_rows():
    # quantizing with a permutation == quantizing rows that were permuted beforehand (Sec. II-C:
    # the reorder can live in the weights, so rows may arrive already permuted)
    rng = np.random.default_rng(99)
    x = rng.standard_normal((20, 128)).astype(np.float32)
    x[:, [3, 77, 100]] *= 25
    perm = rng.permutation(128).astype(np.int32)
    m1, e1 = quant_rows(x, 16, 4, perm=perm)
    m2, e2 = quant_rows(x[:, perm], 16, 4)
    assert np.array_equal(m1, m2) and np.array_equal(e1, e2)
    # and decoding with the permutation restores the original channel order
    mant, exp = O.quantize_append(x.reshape(1, 20, 1, 128), 16, 4, 20, 0, perm=perm.reshape(1, 128))
    d_perm = O.dequantize(mant, exp, 128, 16, 4, 0, 20, perm=perm.reshape(1, 128))[0, :, 0]
    d_raw = O.dequantize(mant, exp, 128, 16, 4, 0, 20)[0, :, 0]
    assert np.array_equal(d_perm[:, perm], d_raw)


def test_append_positions_and_untouched_bytes():
    rng = np.random.default_rng(5)
    B, H, D, S = 2, 3, 128, 10
    mant = np.full((B, H, S, 64), 0xAB, dtype=np.uint8)
    exp = np.full((B, H, S, 8), 0xCD, dtype=np.uint8)
    x = rng.standard_normal((B, 2, H, D)).astype(np.float32)
    O.quantize_append(x, 16, 4, S, [3, 7], mant=mant, exp=exp)
    for b, p0 in enumerate([3, 7]):
        for t in range(S):
            if not (p0 <= t < p0 + 2):
                assert np.all(mant[b, :, t] == 0xAB) and np.all(exp[b, :, t] == 0xCD)
        ref_m, ref_e = O.quantize_append(x[b:b + 1], 16, 4, 2, 0)
        assert np.array_equal(mant[b, :, p0:p0 + 2], ref_m[0])
        assert np.array_equal(exp[b, :, p0:p0 + 2], ref_e[0])
    with pytest.raises(ValueError):
        O.quantize_append(x, 16, 4, S, [3, 9], mant=mant, exp=exp)
