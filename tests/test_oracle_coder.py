"""Pins for the reference embedded bit-plane coder.

The encoder is checked against a re-derivation of its output in closed form
per plane (runs of newly significant coefficients), against the lossless
round trip and against the prefix property; the decoder is checked by brute
force: for every prefix of every stream over a small domain, it must return
the lightest coefficient tuple whose stream starts with that prefix."""
import itertools

import numpy as np

FULL = 7 * 32  # no plane costs more than 7 bits


def _planewise_closed_form(u):
    """Stream derived from the rules rather than by following them: in plane k
    the coefficients below n are copied; then every set bit j >= n costs a
    group bit 1, the zeros skipped since the previous hit, and its own 1
    unless j is the last index; a final group bit 0 follows unless index 3
    has been reached."""
    out = []
    n = 0
    for k in range(31, -1, -1):
        p = [(int(x) >> k) & 1 for x in u]
        out += p[:n]
        hits = [j for j in range(n, 4) if p[j]]
        start = n
        for j in hits:
            out.append(1)
            out += [0] * (j - start)
            if j < 3:
                out.append(1)
            start = j + 1
        if start < 4:
            out.append(0)
        n = start
    return out


def _random_words(rng, count):
    """Words with a random number of leading zero planes, as coefficients have."""
    w = rng.integers(0, 1 << 32, size=(count, 4), dtype=np.uint64)
    sh = rng.integers(0, 33, size=(count, 4)).astype(np.uint64)
    return (w >> sh).astype(np.uint32)


def test_encoder_matches_planewise_closed_form(oracle):
    rng = np.random.default_rng(21)
    words = list(_random_words(rng, 3000))
    words += [np.array(t, dtype=np.uint32) << np.uint32(29) for t in itertools.product(range(8), repeat=4)][::7]
    words += [np.zeros(4, dtype=np.uint32), np.full(4, 0xFFFFFFFF, dtype=np.uint32)]
    for u in words:
        bits, w = oracle.encode_planes(u, FULL)
        want = _planewise_closed_form(u)
        assert w == len(want) <= FULL
        assert list(bits[:w]) == want
        assert not bits[w:].any()


def test_lossless_with_unlimited_budget(oracle):
    rng = np.random.default_rng(22)
    for u in _random_words(rng, 5000):
        bits, _ = oracle.encode_planes(u, FULL)
        assert np.array_equal(oracle.decode_planes(bits, FULL), u)


def test_stream_is_embedded(oracle):
    """A smaller budget yields a prefix of the larger budget's stream."""
    rng = np.random.default_rng(23)
    for u in _random_words(rng, 500):
        full, w = oracle.encode_planes(u, FULL)
        for b in (1, 2, 7, 8, 9, 24, 40, 56, 88, 120):
            part, wb = oracle.encode_planes(u, b)
            assert wb == min(b, w)
            assert np.array_equal(part, full[:b])


def test_stream_length_limits(oracle):
    """All-zero words cost one bit per plane; all-ones cost 7 then 4 per plane."""
    bits, w = oracle.encode_planes(np.zeros(4, dtype=np.uint32), FULL)
    assert w == 32 and not bits.any()
    bits, w = oracle.encode_planes(np.full(4, 0xFFFFFFFF, dtype=np.uint32), FULL)
    assert w == 7 + 31 * 4 and bits[:w].all()


def _weight(v):
    # fewer set bits first; among equal counts, ones at lower indices first
    return sum(bin(int(x)).count("1") * (10 + i) for i, x in enumerate(v))


def test_decoder_by_brute_force_search(oracle):
    """Domain: every tuple with digits only in planes 31..29 (8^4 tuples).
    For each budget b and each distinct b-bit prefix, the decoder must return
    the minimum-weight tuple among all tuples whose stream has that prefix:
    unseen bits are zero, and a group known to hold a one that was not yet
    located gets it at the lowest index still possible."""
    tuples = [tuple(t) for t in itertools.product(range(8), repeat=4)]
    maxb = 24
    streams = {}
    for t in tuples:
        u = np.array(t, dtype=np.uint32) << np.uint32(29)
        bits, _ = oracle.encode_planes(u, maxb)
        streams[t] = tuple(int(x) for x in bits)
    for b in range(0, maxb + 1):
        groups = {}
        for t, s in streams.items():
            groups.setdefault(s[:b], []).append(t)
        for prefix, members in groups.items():
            best = min(members, key=_weight)
            # the minimum is unique
            assert sum(1 for m in members if _weight(m) == _weight(best)) == 1
            got = oracle.decode_planes(np.array(prefix + (1,) * 4, dtype=np.uint8), b)
            assert tuple(int(x) >> 29 for x in got) == best, (b, prefix)
            assert all(int(x) & ((1 << 29) - 1) == 0 for x in got)


def test_decoder_never_reads_past_budget(oracle):
    """Bits after the budget must not influence the result."""
    rng = np.random.default_rng(24)
    for u in _random_words(rng, 300):
        for b in (8, 24, 56, 88):
            bits, _ = oracle.encode_planes(u, b)
            a = oracle.decode_planes(np.concatenate([bits, np.zeros(8, np.uint8)]), b)
            c = oracle.decode_planes(np.concatenate([bits, np.ones(8, np.uint8)]), b)
            assert np.array_equal(a, c)
