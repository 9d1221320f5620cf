"""Pins for the lossless reference codec (oracle/zl_ref.c, format ZL-1): each stage
against numpy library routines or its defining property, whole streams against closed
forms for inputs whose planes are known, a worked example derived by hand, and
losslessness on every kind of bit pattern."""
import os

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
C, G, H = 8192, 256, 32


@pytest.fixture(scope="module")
def zl():
    from oracle import zl_ref
    zl_ref.lib()
    return zl_ref


def _rng(seed):
    return np.random.default_rng(7000 + seed)


def _header(s):
    w = s[:32].view(np.uint32)
    return dict(magic=int(w[0]), chunks=int(w[1]), n=int(w[2]) | int(w[3]) << 32, total=int(w[4]) | int(w[5]) << 32,
                zero=int(w[6]) | int(w[7]) << 32)


def _table(s, chunks):
    return s[H: H + 8 * chunks].view(np.uint64)


# ---- stages ----------------------------------------------------------------------------

def test_word_order_is_a_bijection_of_16_byte_reads(zl):
    idx = np.array([[zl.word_index(g, j) for j in range(32)] for g in range(G)])
    assert sorted(idx.reshape(-1).tolist()) == list(range(C))
    # every aligned run of four consecutive words belongs to one group, in order
    assert (idx[:, 1::4] == idx[:, 0::4] + 1).all() and (idx[:, 3::4] == idx[:, 0::4] + 3).all()
    assert (idx[:, 0::4] % 4 == 0).all()
    # read number t of 256 lanes (16 bytes each) covers words 1024t .. 1024t + 1023, lane g at 4g
    for t in range(8):
        assert (idx[:, 4 * t] == 1024 * t + 4 * np.arange(G)).all()


def test_residuals_against_numpy(zl):
    r = _rng(1)
    mag, sign = np.uint32(0x7FFFFFFF), np.uint32(0x80000000)
    for t in range(60):
        w = r.integers(0, 1 << 32, size=32, dtype=np.uint64).astype(np.uint32)
        if t % 3 == 1:
            w >>= np.uint32(r.integers(1, 31))      # small magnitudes, no sign
        if t % 3 == 2:
            w = (w & np.uint32(0x807FFFFF)) | np.uint32(0x3A000000)      # floats of one binade
        m, res = zl.residuals(w)
        assert m == int((w & mag).max())
        assert np.array_equal(res & sign, w & sign)                      # signs kept
        assert np.array_equal((res & mag).astype(np.int64), m - (w & mag).astype(np.int64))
        assert (res & mag).min() == 0                                    # the largest magnitude is at distance 0
        assert np.array_equal(zl.words(m, res), w)
    c = np.full(32, 0xBEADBEEF, dtype=np.uint32)
    m, res = zl.residuals(c)
    assert m == 0x3EADBEEF and (res == 0x80000000).all()
    # values of one binade: distances below 2^23, so bits 23..30 of every residual are zero
    f = (np.float32(1.0) + r.random(32).astype(np.float32)).view(np.uint32)
    assert not (zl.residuals(f)[1] & np.uint32(0x7F800000)).any()
    # residuals no encoder produces still decode: the distance wraps within 31 bits
    odd = np.zeros(32, dtype=np.uint32); odd[3] = 5; odd[4] = 0x80000007
    assert zl.words(2, odd)[3] == 0x7FFFFFFD and zl.words(2, odd)[4] == 0xFFFFFFFB and zl.words(2, odd)[0] == 2


def test_planes_against_numpy_transpose(zl):
    r = _rng(2)
    for _ in range(50):
        w = r.integers(0, 1 << 32, size=32, dtype=np.uint64).astype(np.uint32)
        bits = (w[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1        # [j, k]
        want = (bits.T.astype(np.uint64) << np.arange(32, dtype=np.uint64)[None, :]).sum(axis=1).astype(np.uint32)
        assert np.array_equal(zl.planes(w), want)
        assert np.array_equal(zl.unplanes(zl.planes(w)), w)
        assert np.array_equal(zl.planes(zl.planes(w)), w)          # a transpose is its own inverse
    for j, k in ((0, 0), (5, 31), (31, 0), (17, 9)):
        one = np.zeros(32, dtype=np.uint32)
        one[j] = np.uint32(1) << np.uint32(k)
        p = zl.planes(one)
        assert p[k] == np.uint32(1) << np.uint32(j) and np.count_nonzero(p) == 1


# ---- whole streams with known planes -----------------------------------------------------

def test_hand_derived_example(zl):
    lines = [l.split() for l in open(os.path.join(HERE, "golden", "zl1_vectors.txt")) if l.strip() and l[0] != "#"]
    n = int(lines[0][1])
    total = int(lines[1][1])
    want = np.zeros(total, dtype=np.uint8)
    for l in lines[2:]:
        off = int(l[0])
        words = np.array([int(h, 16) for h in l[1:]], dtype=np.uint32)
        want[off: off + 4 * words.size] = words.view(np.uint8)
    x = np.array([1, 3, 0x80000000, 0, 7], dtype=np.uint32)
    assert n == x.size and total == 2112
    got = zl.compress(x, guard=64)
    assert got.size == total and np.array_equal(got, want)
    assert np.array_equal(zl.decompress(got, n), x)


@pytest.mark.parametrize("n", [0, 1, 5, C - 1, C, C + 1, 3 * C, 3 * C + 4097])
def test_zero_message(zl, n):
    s = zl.compress(np.zeros(n, dtype=np.uint32), guard=16)
    chunks = -(-n // C)
    h = _header(s)
    assert h == dict(magic=0x31304C5A, chunks=chunks, n=n, total=H + 8 * chunks + 2048 * chunks, zero=0)
    assert s.size == h["total"] and zl.stream_bytes(s) == s.size
    assert np.array_equal(_table(s, chunks), (np.uint64(2) << np.uint64(62)) | (np.uint64(2048) * np.arange(1, chunks + 1, dtype=np.uint64)))
    assert not s[H + 8 * chunks:].any()
    assert np.array_equal(zl.decompress(s, n), np.zeros(n, dtype=np.uint32))


@pytest.mark.parametrize("v", [1, 0x80000000, 0x3F800000, 0xFFFFFFFF, 0x80010001])
def test_constant_message(zl, v):
    """All words equal: every distance is zero, so only the sign plane can be non-zero
    (all ones, for a negative constant); the references hold the magnitude."""
    chunks = 3
    s = zl.compress(np.full(chunks * C, v, dtype=np.uint32))
    neg = v >> 31
    assert s.size == H + chunks * (8 + 8 * G + 4 * G * neg)
    body = s[H + 8 * chunks:].view(np.uint32).reshape(chunks, 2 * G + G * neg)
    assert (body[:, :G] == v & 0x7FFFFFFF).all() and (body[:, G:2 * G] == neg << 31).all() and (body[:, 2 * G:] == 0xFFFFFFFF).all()
    assert (zl.decompress(s, chunks * C) == v).all()


def test_sizes_for_random_and_for_16_bit_content(zl):
    r = _rng(3)
    n = 2 * C
    x = r.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    s = zl.compress(x)
    assert s.size == zl.max_compressed_size(n) == H + 2 * (8 + 8 * G + 4 * C)       # no plane of 32 random residuals is zero
    assert np.array_equal(zl.decompress(s, n), x)
    top = x & np.uint32(0xFFFF0000)                                                 # bf16 content widened to 32 bits
    s = zl.compress(top)
    assert s.size == H + 2 * (8 + 8 * G + 4 * G * 16)                               # distances keep the empty lower half
    assert (s[H + 16 + 4 * G: H + 16 + 8 * G].view(np.uint32) == 0xFFFF0000).all()
    assert np.array_equal(zl.decompress(s, n), top)
    # the last chunk of a ragged message is filled with zeros: one real word w leaves group 0 with
    # reference |w|, its own residual the bare sign and 31 residuals |w|: the planes of |w|'s one bits
    w = int(x[C])
    planes = bin(w & 0x7FFFFFFF).count("1") + (w >> 31)
    assert zl.compress(x[: C + 1]).size == H + 16 + (8 * G + 4 * C) + (8 * G + 4 * planes)
    assert zl.max_compressed_size(0) == H and zl.max_compressed_size(1) == H + 8 + 8 * G + 4 * C


def test_chunks_are_independent(zl):
    r = _rng(4)
    a = workloads.gradient_iid(2 * C, config=1, index=3).view(np.uint32)
    b = r.integers(0, 1 << 20, size=C + 77, dtype=np.uint64).astype(np.uint32)
    sa, sb, sab = zl.compress(a), zl.compress(b), zl.compress(np.concatenate([a, b]))
    pa, pb = sa[H + 16:], sb[H + 16:]
    assert np.array_equal(sab[H + 32:], np.concatenate([pa, pb]))
    ta, tb, tab = _table(sa, 2), _table(sb, 2), _table(sab, 4)
    mask = np.uint64((1 << 62) - 1)
    assert np.array_equal(tab[:2], ta) and np.array_equal(tab[2:] & mask, (tb & mask) + (ta[1] & mask))
    assert (tab >> np.uint64(62) == 2).all()


def _messages():
    e = workloads.edge_values(5)
    nan_inf = np.array([np.nan, -np.nan, np.inf, -np.inf, 0.0, -0.0] * 50, dtype=np.float32)
    smooth = np.cumsum(workloads.gradient_iid(3 * C + 5, std=1e-4)).astype(np.float32)
    return [("edge", e), ("nan_inf", nan_inf), ("smooth", smooth),
            ("gradient", workloads.gradient_iid(2 * C + 9)), ("activation", workloads.activation_gelu(C + 4000)),
            ("moments", workloads.adam_second_moments(2 * C)), ("lowrank", workloads.gradient_lowrank(64, 300)),
            ("bits", _rng(5).integers(0, 1 << 32, size=C + 3, dtype=np.uint64).astype(np.uint32))]


@pytest.mark.parametrize("name,x", _messages(), ids=[m[0] for m in _messages()])
def test_lossless_on_every_kind_of_bit_pattern(zl, name, x):
    w = np.ascontiguousarray(x).view(np.uint32)
    s = zl.compress(w, guard=32)
    assert s.size <= zl.max_compressed_size(w.size) and zl.stream_bytes(s) == s.size
    assert np.array_equal(zl.decompress(s, w.size), w)
    # a receive buffer longer than the stream is fine
    assert np.array_equal(zl.decompress(np.concatenate([s, np.zeros(100, np.uint8)]), w.size), w)


def test_similar_values_shrink_the_stream(zl):
    """What the codec is for (Sec. II-A: similarity between consecutive values): values of
    one magnitude share their upper exponent bits, whose planes vanish; a smooth series
    shares more; half-precision content shares the empty lower half."""
    n = 8 * C
    raw = 4 * n
    grad = workloads.gradient_iid(n)
    assert 0.85 < zl.compress(grad).size / raw < 0.93     # about 4 of 32 planes go, 2 words per group are added
    smooth = np.cumsum(workloads.gradient_iid(n, std=1e-6)).astype(np.float32) + np.float32(1.0)
    assert zl.compress(smooth).size / raw < 0.45
    half = (workloads.activation_gelu(n).view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    assert zl.compress(half).size / raw < 0.45


def test_malformed_streams_are_rejected(zl):
    x = workloads.gradient_iid(C + 10).view(np.uint32)
    s = zl.compress(x)
    n = x.size

    def bad(t, nn=n):
        with pytest.raises(zl.StreamError):
            zl.decompress(t, nn)

    bad(s[:16])
    bad(s[:-1])                                  # truncated
    bad(s, n + 1)                                # not this message's length
    t = s.copy(); t[0] ^= 1; bad(t)              # magic
    t = s.copy(); t[H + 7] = 0x40; bad(t)        # table entry not marked complete
    t = s.copy(); t[H:H + 8].view(np.uint64)[0] += np.uint64(4); bad(t)     # chunk 0 ends where its words do not
    t = s.copy(); assert t[H + 16 + 4 * G + 3] & 0x7F != 0x7F                     # values of one magnitude: upper planes absent
    t[H + 16 + 4 * G + 3] |= 0x7F; bad(t)                                         # bitmap promises more planes than stored
    t = s.copy(); t[16:24].view(np.uint64)[0] += np.uint64(8); bad(t)       # total beyond the buffer


def test_16_bit_messages(zl):
    """A 16-bit message is coded as its words shifted into the upper halves: the stream is that
    of the 32-bit message (for bf16: of the values widened to fp32, which numpy confirms through
    its own float32 -> bf16 truncation), every 16-bit pattern comes back, and the empty lower
    halves cost nothing."""
    every = np.arange(65536, dtype=np.uint16)
    s = zl.compress16(every, guard=16)
    assert np.array_equal(s, zl.compress(every.astype(np.uint32) << np.uint32(16)))
    assert np.array_equal(zl.decompress16(s, every.size), every)
    r = _rng(9)
    f = (workloads.activation_gelu(3 * C + 77) * np.float32(3.0)).astype(np.float32)
    bf = (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)                 # bf16 by truncation
    widened = (bf.astype(np.uint32) << np.uint32(16)).view(np.float32)
    assert np.array_equal(zl.compress16(bf), zl.compress(widened))
    assert np.array_equal(zl.decompress(zl.compress16(bf), bf.size, dtype=np.float32).view(np.uint32), widened.view(np.uint32))
    h = f.astype(np.float16)
    sh = zl.compress16(h)
    assert np.array_equal(zl.decompress16(sh, h.size, dtype=np.float16).view(np.uint16), h.view(np.uint16))
    # per value: 16 bits in, at most 16 planes + reference + bitmap out; similar magnitudes drop some more
    assert sh.size < 2 * h.size * (16 + 2) / 16 + 64 and zl.compress16(bf).size < 2 * bf.size
    assert zl.compress16(np.zeros(0, dtype=np.uint16)).size == 32
    odd = r.integers(0, 65536, size=C + 5, dtype=np.uint16)
    assert np.array_equal(zl.decompress16(zl.compress16(odd), odd.size), odd)
