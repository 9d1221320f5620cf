"""Pins for the reference codec as a whole: stored vectors, sizes, zero and
constant blocks, the error bound, monotonicity in the rate, ragged tails, and
the reduce step as a composition checked with numpy's fp32 adds."""
import os

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RATES = (4, 8, 12, 16, 20, 24, 28, 32)


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [c.strip() for c in line.split(";")]


def _f32_from_hex(words):
    return np.array([int(w, 16) for w in words.split()], dtype=np.uint32).view(np.float32)


def _block_bytes(hexint, rate):
    return np.frombuffer(int(hexint, 16).to_bytes(rate // 2, "little"), dtype=np.uint8)


def test_stored_block_vectors(oracle):
    count = 0
    for rate, xin, comp, dec in _rows("zc1_vectors.txt"):
        rate = int(rate)
        x = _f32_from_hex(xin)
        want = _block_bytes(comp, rate)
        got = oracle.encode_block(x, rate)
        assert np.array_equal(got, want), (rate, xin)
        assert np.array_equal(oracle.compress(x, rate), want)
        d = oracle.decode_block(want, rate)
        assert np.array_equal(d.view(np.uint32), _f32_from_hex(dec).view(np.uint32)), (rate, xin)
        count += 1
    assert count == 9


def test_stored_reduce_vectors(oracle):
    blocks = {"A": np.array([1, 2, 3, 4], dtype=np.float32),
              "B": np.array([0.001, -0.002, 0.0005, 0], dtype=np.float32)}
    for rate, names, comp in _rows("zc1_reduce_vectors.txt"):
        rate = int(rate)
        ins = [oracle.compress(blocks[n], rate) for n in names.split()]
        got = oracle.reduce_compressed(ins, 4, rate)
        assert np.array_equal(got, _block_bytes(comp, rate)), (rate, names)
    c = oracle.compress(blocks["A"], 8)
    assert np.array_equal(oracle.decompress(oracle.reduce_compressed([c, c], 4, 8), 4, 8),
                          np.array([2, 4, 6, 8], dtype=np.float32))


def test_compressed_size_is_exact(oracle):
    for rate in RATES:
        for n in (0, 4, 8, 1 << 10, 1 << 20, 4 * 12345):
            assert oracle.compressed_size(n, rate) == n * rate // 8
        for n in (1, 2, 3, 5, 7, 1001):
            assert oracle.compressed_size(n, rate) == ((n + 3) // 4) * (rate // 2)
    for bad in (0, 1, 3, 5, 6, 36, -4):
        assert oracle.compressed_size(64, bad) == 0


def test_writes_exactly_the_stated_bytes(oracle):
    """Bytes after the compressed size and floats after n stay untouched."""
    import ctypes
    x = workloads.gradient_iid(1000 + 3)
    L = oracle.lib()
    for rate in RATES:
        for n in (1003, 1000, 1):
            size = oracle.compressed_size(n, rate)
            buf = np.full(size + 16, 0xA5, dtype=np.uint8)
            assert L.zc_ref_compress(x.ctypes.data, n, rate, buf.ctypes.data, size) == 0
            assert (buf[size:] == 0xA5).all()
            out = np.full(n + 8, np.float32(-77.0), dtype=np.float32)
            assert L.zc_ref_decompress(buf.ctypes.data, n, rate, out.ctypes.data) == 0
            assert (out[n:] == np.float32(-77.0)).all()
            assert L.zc_ref_compress(x.ctypes.data, n, rate, buf.ctypes.data, size - 1) == -4
    assert L.zc_ref_compress(x.ctypes.data, 8, 7, buf.ctypes.data, 100) == -2


def test_zero_blocks_are_zero_bytes(oracle):
    x = np.zeros(64, dtype=np.float32)
    x[5] = -0.0
    for rate in RATES:
        c = oracle.compress(x, rate)
        assert not c.any()
        d = oracle.decompress(c, 64, rate)
        assert not d.view(np.uint32).any()       # +0.0 everywhere


def test_header_byte_is_the_block_exponent(oracle):
    x = workloads.edge_values(3)
    for rate in (4, 16, 32):
        c = oracle.compress(x, rate).reshape(-1, rate // 2)
        for j in range(0, len(c), 37):
            assert c[j, 0] == oracle.block_exponent(x[4 * j:4 * j + 4])


def test_streams_are_embedded_across_rates(oracle):
    """The block at a lower rate is a bit prefix of the block at a higher rate."""
    x = np.concatenate([workloads.edge_values(4)[:2000], workloads.gradient_iid(2000)])
    full = oracle.compress(x, 32).reshape(-1, 16)
    for rate in RATES[:-1]:
        c = oracle.compress(x, rate).reshape(-1, rate // 2)
        assert np.array_equal(c, full[:, :rate // 2])


def test_constant_blocks(oracle):
    rng = np.random.default_rng(31)
    consts = np.concatenate([
        rng.standard_normal(300).astype(np.float32) * np.float32(1e-3),
        rng.integers(1, 1 << 31, size=300, dtype=np.int64).astype(np.uint32).view(np.float32),
        -rng.integers(1 << 23, 0x7F000000, size=100, dtype=np.int64).astype(np.uint32).view(np.float32)])
    consts = consts[np.isfinite(consts) & (np.abs(consts) < 2.0 ** 127)]
    for rate in RATES:
        x = np.repeat(consts, 4)
        d = oracle.decompress(oracle.compress(x, rate), x.size, rate).reshape(-1, 4)
        # a constant block always decodes to a constant block
        assert (d == d[:, :1]).all()
        if rate >= 16:  # and to the same constant once the mean's digits fit
            assert np.array_equal(d[:, 0].view(np.uint32), consts.view(np.uint32))
    # normal powers of two: the mean is +-2^27, whose one or two negabinary digits
    # fit the 8 payload bits of rate 4
    pw = np.array([s * 2.0 ** k for k in range(-126, 127, 3) for s in (1, -1)], dtype=np.float32)
    for rate in RATES:
        x = np.repeat(pw, 4)
        d = oracle.decompress(oracle.compress(x, rate), x.size, rate)
        assert np.array_equal(d.view(np.uint32), x.view(np.uint32))


def test_error_bound_from_complete_planes(oracle):
    """T = floor((4R-15)/5) planes are always coded completely, so
    |decoded - x| <= (1.5 * 2^(32-T) + 4) * 2^(e-28)."""
    bufs = [workloads.gradient_iid(1 << 14), workloads.activation_gelu(1 << 14),
            workloads.adam_second_moments(1 << 14), workloads.parameters(1 << 14),
            workloads.edge_values(5)]
    for rate in (16, 20, 24, 28, 32):
        T = (4 * rate - 15) // 5
        for x in bufs:
            d = oracle.decompress(oracle.compress(x, rate), x.size, rate).astype(np.float64)
            xb = x.reshape(-1, 4)
            E = np.array([oracle.block_exponent(b) for b in xb[::16]])
            err = np.abs(d.reshape(-1, 4)[::16] - xb[::16].astype(np.float64)).max(axis=1)
            ok = (E > 0) & (E < 250)
            bound = (1.5 * 2.0 ** (32 - T) + 4) * 2.0 ** (E.astype(np.float64) - 127 - 28)
            assert (err[ok] <= bound[ok]).all()
            # subnormal-output rounding can add half an ulp at the bottom of the range
            assert (err[~ok & (E > 0)] <= 2 * bound[~ok & (E > 0)] + 1e-45).all()


@pytest.mark.parametrize("maker", [workloads.gradient_iid, workloads.activation_gelu,
                                   workloads.parameters, workloads.adam_second_moments,
                                   lambda n: workloads.gradient_lowrank(64, n // 64)])
def test_error_decreases_with_rate(oracle, maker):
    """Aggregate RMSE over a buffer falls strictly as the rate rises; the
    largest error never rises (Sec. IV-C/IV-F: a higher rate stays closer to the
    uncompressed run)."""
    x = maker(1 << 16)
    prev_rmse, prev_max = np.inf, np.inf
    for rate in RATES:
        d = oracle.decompress(oracle.compress(x, rate), x.size, rate).astype(np.float64)
        err = d - x.astype(np.float64)
        rmse, mx = np.sqrt(np.mean(err ** 2)), np.abs(err).max()
        assert rmse < prev_rmse and mx <= prev_max, (rate, rmse, mx)
        prev_rmse, prev_max = rmse, mx
    assert prev_rmse < 1e-8 * x.astype(np.float64).std() * 100


def test_relative_error_levels_on_gaussian_data(oracle):
    """Order-of-magnitude anchors for i.i.d. Gaussian data: roughly 4 bits of
    the 4R-bit block are overhead per value, each further bit halves the error."""
    x = workloads.gradient_iid(1 << 16)
    sd = x.astype(np.float64).std()
    rel = {}
    for rate in (8, 16, 24):
        d = oracle.decompress(oracle.compress(x, rate), x.size, rate).astype(np.float64)
        rel[rate] = np.sqrt(np.mean((d - x) ** 2)) / sd
    assert 3e-2 < rel[8] < 1.4e-1
    assert 1.2e-4 < rel[16] < 5.5e-4
    assert 4e-7 < rel[24] < 2.2e-6


def test_ragged_tail_repeats_the_last_value(oracle):
    x = workloads.gradient_iid(64)
    for rate in (4, 8, 16, 24):
        for n in (61, 62, 63, 1, 2, 3):
            padded = np.concatenate([x[:n], np.repeat(x[n - 1], (-n) % 4)])
            assert np.array_equal(oracle.compress(x[:n], rate), oracle.compress(padded, rate))
            d = oracle.decompress(oracle.compress(x[:n], rate), n, rate)
            assert np.array_equal(d, oracle.decompress(oracle.compress(padded, rate), padded.size, rate)[:n])


def test_decoding_arbitrary_bytes_is_defined(oracle):
    rng = np.random.default_rng(33)
    for rate in RATES:
        s = rng.integers(0, 256, size=1024 * (rate // 2), dtype=np.uint8)
        with np.errstate(all="ignore"):
            a = oracle.decompress(s, 4096, rate)
            b = oracle.decompress(s.copy(), 4096, rate)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_reduce_is_decode_add_encode(oracle):
    """reduce(in_0..in_{k-1}) == compress(((d_0 + d_1) + d_2) + ...), with the
    adds done by numpy in fp32."""
    n = 4096 + 2
    peers = [workloads.gradient_lowrank(64, 64, tail=2, config=5, index=p) for p in range(8)]
    for rate in (4, 8, 16, 24):
        comp = [oracle.compress(p, rate) for p in peers]
        dec = [oracle.decompress(c, n, rate) for c in comp]
        for k in (1, 2, 3, 8):
            s = dec[0].copy()
            for j in range(1, k):
                s = (s + dec[j]).astype(np.float32)
            want = oracle.compress(s, rate)
            got = oracle.reduce_compressed(comp[:k], n, rate)
            assert np.array_equal(got, want), (rate, k)
    # ring order: seven pairwise steps
    rate = 4
    comp = [oracle.compress(p, rate) for p in peers]
    acc = comp[0]
    s = oracle.decompress(acc, n, rate)
    for j in range(1, 8):
        acc = oracle.reduce_compressed([acc, comp[j]], n, rate)
        s = oracle.decompress(oracle.compress((s + oracle.decompress(comp[j], n, rate)).astype(np.float32), rate), n, rate)
    assert np.array_equal(oracle.decompress(acc, n, rate), s)


def test_reduce_argument_checks(oracle):
    c = oracle.compress(np.ones(8, dtype=np.float32), 8)
    with pytest.raises(ValueError):
        oracle.reduce_compressed([], 8, 8)
    with pytest.raises(ValueError):
        oracle.reduce_compressed([c] * 17, 8, 8)
    assert np.array_equal(oracle.reduce_compressed([c] * 16, 8, 8),
                          oracle.compress(np.full(8, 16, dtype=np.float32), 8))


def test_ring_hop_variants_are_compositions(oracle):
    """reduce_mixed == compress((sum of decoded chunks) + local) and reduce_decompress ==
    that sum itself, with every add done by numpy in fp32 in the stated order."""
    n = 4096 + 3
    peers = [workloads.gradient_lowrank(64, 64, tail=3, config=5, index=p) for p in range(5)]
    local = workloads.gradient_lowrank(64, 64, tail=3, config=5, index=7)
    for rate in (4, 8, 16, 24):
        comp = [oracle.compress(p, rate) for p in peers]
        dec = [oracle.decompress(c, n, rate) for c in comp]
        for k in (1, 2, 5):
            s = dec[0].copy()
            for j in range(1, k):
                s = (s + dec[j]).astype(np.float32)
            assert np.array_equal(oracle.reduce_decompress(comp[:k], None, n, rate).view(np.uint32), s.view(np.uint32))
            assert np.array_equal(oracle.reduce_mixed(comp[:k], None, n, rate), oracle.reduce_compressed(comp[:k], n, rate))
            t = (s + local).astype(np.float32)
            assert np.array_equal(oracle.reduce_decompress(comp[:k], local, n, rate).view(np.uint32), t.view(np.uint32))
            assert np.array_equal(oracle.reduce_mixed(comp[:k], local, n, rate), oracle.compress(t, rate))
    # a full ring on one rank's share: first hop has only raw data on both sides
    rate, acc = 8, None
    raw = [workloads.gradient_lowrank(64, 64, tail=3, config=5, index=p) for p in range(4)]
    acc = oracle.compress(raw[0], rate)
    ref = raw[0]
    for p in (1, 2):
        acc = oracle.reduce_mixed([acc], raw[p], n, rate)
        ref = (oracle.decompress(oracle.compress(ref, rate), n, rate) + raw[p]).astype(np.float32)
    final = oracle.reduce_decompress([acc], raw[3], n, rate)
    want = (oracle.decompress(oracle.compress(ref, rate), n, rate) + raw[3]).astype(np.float32)
    assert np.array_equal(final.view(np.uint32), want.view(np.uint32))
    with pytest.raises(ValueError):
        oracle.reduce_mixed([], local, n, 8)



def test_requantising_chain_error_per_rate(oracle):
    """A ring that re-encodes the running sum at every hop: with eight payload bits per block
    (rate 4) the error of the running sum about doubles per hop, at rate 8 it grows about
    linearly and stays a fraction of the sum, at rate 16 it is negligible; one 8-way reduce
    of the same chunks re-encodes once and stays close to one compression's error."""
    bufs = [b for _, b in workloads.config_buffers(5, 10)]
    n = bufs[0].size
    total = np.sum([b.astype(np.float64) for b in bufs], axis=0)
    rmse = {}
    for rate in (4, 8, 16):
        comp = [oracle.compress(b, rate) for b in bufs]
        acc, partial, per_hop = comp[0], bufs[0].astype(np.float64), []
        for j in range(1, 8):
            acc = oracle.reduce_compressed([acc, comp[j]], n, rate)
            partial = partial + bufs[j]
            per_hop.append(np.sqrt(np.mean((oracle.decompress(acc, n, rate) - partial) ** 2)))
        direct = oracle.decompress(oracle.reduce_compressed(comp, n, rate), n, rate)
        rmse[rate] = (per_hop, np.sqrt(np.mean((direct - total) ** 2)))
    std = total.std()
    hops4, direct4 = rmse[4]
    assert all(1.7 < b / a < 2.3 for a, b in zip(hops4[:-1], hops4[1:])) and hops4[-1] > 20 * std
    assert direct4 < 2.5 * std
    hops8, direct8 = rmse[8]
    assert hops8[-1] < 6 * hops8[0] and hops8[-1] < 0.3 * std and direct8 < 0.15 * std
    assert all(b > a for a, b in zip(hops8[:-1], hops8[1:]))
    assert rmse[16][0][-1] < 1e-3 * std


@pytest.mark.parametrize("n", [1, 5, 4097, 2, 6, 4098, 3, 4099, 4, 4096])
def test_every_call_on_every_ragged_length(oracle, n):
    """All buffer calls at lengths with every remainder modulo 4, against their definitions
    spelled out with numpy: the last block holds n mod 4 values, its pad repeats the last valid
    value (for the reduce calls: the last valid SUM), and nothing beyond n values is produced."""
    x = [workloads.gradient_iid(4100, index=40 + j) * np.float32(1 + j) for j in range(3)]
    local = workloads.gradient_iid(4100, index=50)[:n]
    blocks = (n + 3) // 4
    for rate in (4, 16):
        comp = [oracle.compress(v[:n], rate) for v in x]
        assert all(c.size == blocks * rate // 2 for c in comp)
        # the last block of the stream is the block of the padded values
        tail = np.concatenate([x[0][4 * (blocks - 1):n], np.repeat(x[0][n - 1], 4 * blocks - n)])
        assert np.array_equal(comp[0][-(rate // 2):], oracle.encode_block(tail, rate))
        dec = [oracle.decompress(c, n, rate) for c in comp]
        assert dec[0].size == n
        assert np.array_equal(dec[0][4 * (blocks - 1):].view(np.uint32),
                              oracle.decode_block(comp[0][-(rate // 2):], rate)[:n - 4 * (blocks - 1)].view(np.uint32))
        for k in (1, 3):
            total = dec[0].copy()
            for j in range(1, k):
                total = (total + dec[j]).astype(np.float32)
            assert np.array_equal(oracle.reduce_compressed(comp[:k], n, rate), oracle.compress(total, rate))
            assert np.array_equal(oracle.reduce_decompress(comp[:k], None, n, rate).view(np.uint32), total.view(np.uint32))
            with_local = (total + local).astype(np.float32)
            assert np.array_equal(oracle.reduce_mixed(comp[:k], local, n, rate), oracle.compress(with_local, rate))
            assert np.array_equal(oracle.reduce_decompress(comp[:k], local, n, rate).view(np.uint32), with_local.view(np.uint32))


def test_what_the_output_buffer_held_before_does_not_matter(oracle):
    """Every bit of every block is written, zeros included: compressing and reducing into a
    buffer full of ones gives the same bytes as into a buffer of zeros."""
    import ctypes
    L = oracle.lib()
    n = 4 * 300 + 1
    x = workloads.gradient_iid(n)
    y = workloads.gradient_iid(n, index=3)
    for rate in (4, 8, 12, 24, 32):
        want = oracle.compress(x, rate)
        out = np.full(want.size, 0xFF, dtype=np.uint8)
        assert L.zc_ref_compress(x.ctypes.data, n, rate, out.ctypes.data, out.size) == 0
        assert np.array_equal(out, want), rate
        other = oracle.compress(y, rate)
        ptrs = (ctypes.c_void_p * 2)(want.ctypes.data, other.ctypes.data)
        out = np.full(want.size, 0xFF, dtype=np.uint8)
        assert L.zc_ref_reduce_compressed(ptrs, 2, n, rate, out.ctypes.data, out.size) == 0
        assert np.array_equal(out, oracle.reduce_compressed([want, other], n, rate)), rate


def test_ring_hop_calls_take_one_to_sixteen_chunks(oracle):
    c = oracle.compress(np.ones(9, dtype=np.float32), 8)
    local = np.full(9, 0.5, dtype=np.float32)
    for call in (lambda chunks: oracle.reduce_mixed(chunks, local, 9, 8), lambda chunks: oracle.reduce_decompress(chunks, local, 9, 8)):
        with pytest.raises(ValueError):
            call([])
        with pytest.raises(ValueError):
            call([c] * 17)
    assert np.array_equal(oracle.reduce_decompress([c] * 16, local, 9, 8), np.full(9, 16.5, dtype=np.float32))
    assert np.array_equal(oracle.reduce_mixed([c] * 16, local, 9, 8), oracle.compress(np.full(9, 16.5, dtype=np.float32), 8))
