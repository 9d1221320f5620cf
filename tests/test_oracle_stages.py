"""Pins for the reference codec's arithmetic stages (exponent, block floating
point, lifting, negabinary).  Each check compares the oracle with something
other than itself: a closed form on IEEE bit fields, exact integer/rational
arithmetic in Python, an exhaustive inverse, or a matrix identity."""
import itertools
from fractions import Fraction

import numpy as np

from paper_2409_02423_amd import workloads

M = (1 << 28) - 1


def _blocks(seed=1):
    e = workloads.edge_values(seed)
    return e.reshape(-1, 4)


# ---- stage 1: shared exponent ------------------------------------------------

def _closed_form_E(block):
    """On IEEE fields: E = max exponent field + 1 when some field is non-zero;
    1 when only subnormals are non-zero; 0 for an all-zero block."""
    bits = block.view(np.uint32)
    F = (bits >> 23) & 0xFF
    mant = bits & 0x7FFFFF
    if F.max() > 0:
        return int(F.max()) + 1
    return 1 if mant.any() else 0


def test_exponent_closed_form_on_ieee_fields(oracle):
    for blk in _blocks():
        assert oracle.block_exponent(blk) == _closed_form_E(blk), blk


def test_exponent_examples(oracle):
    f = np.float32
    assert oracle.block_exponent([0, 0, 0, 0]) == 0
    assert oracle.block_exponent([-0.0, 0.0, -0.0, 0.0]) == 0
    assert oracle.block_exponent([1, 2, 3, 4]) == 130          # 4 = 0.5 * 2^3
    assert oracle.block_exponent([0.75, 0, 0, 0]) == 127        # 0.75 * 2^0
    assert oracle.block_exponent([1, 0, 0, 0]) == 128           # 0.5 * 2^1
    assert oracle.block_exponent([0, -1, 0, 0]) == 128
    assert oracle.block_exponent([f(1.4e-45), 0, 0, 0]) == 1    # clamp at e = -126
    assert oracle.block_exponent([f(1.1754944e-38), 0, 0, 0]) == 2  # 2^-126 = 0.5 * 2^-125
    assert oracle.block_exponent([f(3.4028235e38), 0, 0, 0]) == 255


# ---- stage 2: block floating point ------------------------------------------

def _closed_form_q(block, E):
    bits = block.view(np.uint32).astype(np.int64)
    F = (bits >> 23) & 0xFF
    s = (bits & 0x7FFFFF) + np.where(F > 0, 1 << 23, 0)
    sign = np.where(bits >> 31, -1, 1)
    Fp = np.maximum(F, 1)
    Fmax = E - 1
    if F.max() == 0:           # all-subnormal block: x = s*2^-149, e = -126, so q = s*2^(28+126-149) = s*32
        return sign * s * 32 * (E != 0)
    sh = Fmax - Fp
    q = np.where(sh >= 28, 0, (s * 16) >> np.minimum(sh, 63))
    return sign * q


def test_quantise_closed_form_and_range(oracle):
    for blk in _blocks():
        E = oracle.block_exponent(blk)
        if E == 0:
            continue
        q = oracle.quantise(blk, E)
        assert np.array_equal(q.astype(np.int64), _closed_form_q(blk, E)), (blk, q)
        assert np.abs(q.astype(np.int64)).max() <= M
        # the largest value uses the top fraction bit unless the block is subnormal-only
        if E > 1:
            assert np.abs(q.astype(np.int64)).max() >= 1 << 27


def test_quantise_is_exact_truncation(oracle):
    """q = trunc(x * 2^(28-e)) in exact rational arithmetic."""
    rng = np.random.default_rng(5)
    blocks = _blocks()
    for blk in blocks[rng.choice(len(blocks), 400, replace=False)]:
        E = oracle.block_exponent(blk)
        if E == 0:
            continue
        q = oracle.quantise(blk, E)
        for xi, qi in zip(blk, q):
            exact = Fraction(float(xi)) * Fraction(2) ** (28 - (E - 127))
            t = int(abs(exact))  # floor of the magnitude
            assert int(qi) == (t if exact >= 0 else -t)


def test_dequantise_two_roundings(oracle):
    """float(q) with round-to-nearest-even, then scaling by 2^(e-28) rounded
    again only when the result is subnormal; overflow gives infinity."""
    rng = np.random.default_rng(6)
    qs = np.concatenate([rng.integers(-(1 << 31), 1 << 31, size=2000),
                         [0, 1, -1, M, -M, (1 << 24) + 1, (1 << 25) + 3, -(1 << 25) - 1,
                          (1 << 31) - 1, -(1 << 31), 3, 5, 7, 0x1FFFFFF, 0x3000001]])
    Es = np.concatenate([rng.integers(1, 256, size=len(qs) - 8), [1, 1, 2, 3, 24, 25, 255, 254]])
    with np.errstate(over="ignore"):
        for q, E in zip(qs, Es):
            got = oracle.dequantise([q, q, -q if q > -(1 << 31) else 0, 0], int(E))
            first = np.float64(np.float32(np.int64(q)))           # RNE int -> fp32
            want = np.float32(first * 2.0 ** (int(E) - 127 - 28))  # exact product, RNE to fp32
            assert got[0].view(np.uint32) == want.view(np.uint32), (q, E, got[0], want)
            assert got[3].view(np.uint32) == 0


def test_dequantise_double_rounding_literals(oracle):
    """Cases where rounding the exact value q * 2^(E-155) once differs from what the format
    says (int -> fp32 first, then the scaling).  With E = 1 the scale is 2^-154, i.e. q/32
    in units of the smallest subnormal 2^-149.  q = 2^25+17: fp32 spacing in [2^25, 2^26) is
    4, so float(q) = 2^25+16, and (2^25+16)/32 = 2^20 + 1/2 is a tie that goes to the even
    2^20 (bits 0x00100000); the exact (2^25+17)/32 = 2^20 + 17/32 would round to 2^20+1.
    q = 2^26+17: spacing 8, float(q) = 2^26+16, /32 = 2^21 + 1/2 -> 2^21 (exact: 2^21+1).
    E = 2 halves the divisor: q = 2^25+9 -> float 2^25+8 -> /16 = 2^21 + 1/2 -> 2^21."""
    for q, E, bits in ((33554449, 1, 0x00100000), (-33554449, 1, 0x80100000),
                       (67108881, 1, 0x00200000), (-67108881, 1, 0x80200000),
                       (33554441, 2, 0x00200000), (-33554441, 2, 0x80200000)):
        got = oracle.dequantise([q, 0, 0, 0], E)
        assert int(got[0].view(np.uint32)) == bits, (q, E, hex(int(got[0].view(np.uint32))))


# ---- stage 3: lifting ----------------------------------------------------------

def test_lift_inverse_exhaustive_small(oracle):
    rng = range(-8, 9)
    for v in itertools.product(rng, repeat=4):
        w = oracle.fwd_lift(v)
        assert tuple(oracle.inv_lift(w)) == v


def test_lift_inverse_extremes_and_random(oracle):
    vals = [M, -M, M - 1, -(M - 1), 0, 1, -1]
    for v in itertools.product(vals, repeat=4):
        w = oracle.fwd_lift(v)
        assert tuple(int(t) for t in oracle.inv_lift(w)) == v
        w64 = np.abs(w.astype(np.int64))
        # magnitudes of the basis rows' gains (1, 3, 2, 2) times M, plus the floors' slack;
        # far inside the range 32 negabinary digits can express
        assert w64[0] <= M + 2 and w64[1] <= 3 * M + 2 and w64[2] <= 2 * M + 2 and w64[3] <= 2 * M + 2
    rng = np.random.default_rng(11)
    for v in rng.integers(-M, M + 1, size=(20000, 4)):
        w = oracle.fwd_lift(v)
        assert np.array_equal(oracle.inv_lift(w), v)
    # the inverse is also exact on arbitrary 32-bit words (wrap-around arithmetic),
    # which is what decoding arbitrary bytes relies on
    for v in rng.integers(-(1 << 31), 1 << 31, size=(5000, 4)):
        w = oracle.inv_lift(v)
        assert np.array_equal(oracle.fwd_lift(w), v.astype(np.int32))


def test_lift_equals_basis_matrix_when_no_floor_discards(oracle):
    """On multiples of 16 no shift drops a bit and the transform is the matrix
    [[1,1,1,1]/4, [5,1,-1,-5]/4, [-1,1,1,-1]/2, [-1,3,-3,1]/4]."""
    A = [[Fraction(1, 4)] * 4,
         [Fraction(5, 4), Fraction(1, 4), Fraction(-1, 4), Fraction(-5, 4)],
         [Fraction(-1, 2), Fraction(1, 2), Fraction(1, 2), Fraction(-1, 2)],
         [Fraction(-1, 4), Fraction(3, 4), Fraction(-3, 4), Fraction(1, 4)]]
    assert tuple(oracle.fwd_lift([16, 0, 0, 0])) == (4, 20, -8, -4)
    assert tuple(oracle.fwd_lift([0, 16, 0, 0])) == (4, 4, 8, 12)
    assert tuple(oracle.fwd_lift([0, 0, 16, 0])) == (4, -4, 8, -12)
    assert tuple(oracle.fwd_lift([0, 0, 0, 16])) == (4, -20, -8, 4)
    rng = np.random.default_rng(12)
    for v in rng.integers(-(1 << 23), 1 << 23, size=(3000, 4)) * 16:
        w = oracle.fwd_lift(v)
        want = [sum(a * int(x) for a, x in zip(row, v)) for row in A]
        assert [Fraction(int(t)) for t in w] == want


def test_lift_constant_block_has_only_a_mean(oracle):
    rng = np.random.default_rng(13)
    for c in rng.integers(-M, M + 1, size=2000):
        assert tuple(oracle.fwd_lift([c] * 4)) == (c, 0, 0, 0)


# ---- stage 4: negabinary -------------------------------------------------------

def _value_of_digits(u):
    return sum(((u >> k) & 1) * (-2) ** k for k in range(32))


def test_negabinary_digits_sum_to_value(oracle):
    for c in range(-(1 << 12), 1 << 12):
        assert _value_of_digits(oracle.negabinary(c)) == c
    rng = np.random.default_rng(14)
    for c in rng.integers(-3 * M, 3 * M + 1, size=20000):
        u = oracle.negabinary(int(c))
        assert _value_of_digits(u) == c
        assert oracle.inv_negabinary(u) == c


def test_negabinary_is_a_bijection_on_words(oracle):
    rng = np.random.default_rng(15)
    for u in rng.integers(0, 1 << 32, size=20000):
        c = oracle.inv_negabinary(int(u))
        assert oracle.negabinary(c) == u
        # inside the range 32 digits can express, the digits give the value itself
        v = _value_of_digits(int(u))
        assert -(1 << 31) > v or v >= (1 << 31) or v == c
    assert oracle.negabinary(0) == 0
    assert oracle.negabinary(1) == 1
    assert oracle.negabinary(-1) == 0b11
    assert oracle.negabinary(2) == 0b110
    assert oracle.negabinary(-2) == 0b10
    assert oracle.negabinary(3) == 0b111
