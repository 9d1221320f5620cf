"""GPU parity: the HIP library (through its C ABI) against the CPU reference,
bit for bit, on the same seeded inputs.  Compressed streams are compared as bytes,
decoded values as fp32 bit patterns."""
import ctypes

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

pytestmark = pytest.mark.gpu

RATES = (4, 8, 12, 16, 20, 24, 28, 32)
MAIN_RATES = (4, 8, 16, 24)


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_02423_amd import zc
    zc.lib()
    return zc


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _host(t):
    return t.cpu().numpy()


def _assert_bytes_equal(got, want, block_bytes, what):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s: %d bytes differ, first at byte %d (block %d)" %
                             (what, bad.size, bad[0], bad[0] // block_bytes))


def _assert_floats_equal(got, want, what):
    g, w = np.asarray(got).view(np.uint32), np.asarray(want).view(np.uint32)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    if not np.array_equal(g, w):
        bad = np.flatnonzero(g != w)
        raise AssertionError("%s: %d values differ, first at %d: got %08x want %08x" %
                             (what, bad.size, bad[0], g[bad[0]], w[bad[0]]))


# ---- small buffers, whole-buffer comparison ------------------------------------------------

@pytest.mark.parametrize("rate", RATES)
def test_edge_values_round_trip(gpu, oracle, rate):
    print("edge values, rate", rate, flush=True)
    x = workloads.edge_values(21)
    want_c = oracle.compress(x, rate)
    got_c = gpu.zc_compress(_dev(x), rate)
    _assert_bytes_equal(_host(got_c), want_c, rate // 2, "compress edge rate %d" % rate)
    want_d = oracle.decompress(want_c, x.size, rate)
    got_d = gpu.zc_decompress(_dev(want_c), x.size, rate)
    _assert_floats_equal(_host(got_d), want_d, "decompress edge rate %d" % rate)


@pytest.mark.parametrize("rate", RATES)
def test_arbitrary_bytes_decode_alike(gpu, oracle, rate):
    print("arbitrary bytes, rate", rate, flush=True)
    rng = np.random.default_rng(100 + rate)
    n = 4 * 20000
    s = rng.integers(0, 256, size=n // 4 * (rate // 2), dtype=np.uint8)
    s[: s.size // 3] &= rng.integers(0, 256, size=s.size // 3, dtype=np.uint8)  # sparser streams too
    with np.errstate(all="ignore"):
        want = oracle.decompress(s, n, rate)
    got = gpu.zc_decompress(_dev(s), n, rate)
    _assert_floats_equal(_host(got), want, "arbitrary bytes rate %d" % rate)


@pytest.mark.parametrize("rate", RATES)
def test_reduce_on_arbitrary_bytes(gpu, oracle, rate):
    """The three reduce calls on streams of arbitrary bytes (every header byte, every payload):
    wherever the sum defined by decode-then-add is finite, stream bytes and fp32 sums equal the
    reference's; where it is infinite the fp32 sum still does (the rate-4 kernel's fused
    multiply-add must not turn an overflowing decoded value into a finite one); blocks holding
    a NaN (infinity minus infinity) are only required to be written and repeatable."""
    print("reduce on arbitrary bytes, rate", rate, flush=True)
    rng = np.random.default_rng(300 + rate)
    n = 4 * 20000 + 2
    size = oracle.compressed_size(n, rate)
    streams = [rng.integers(0, 256, size=size, dtype=np.uint8) for _ in range(3)]
    streams[1][: size // 2] &= rng.integers(0, 256, size=size // 2, dtype=np.uint8)
    # plenty of blocks at the top of the exponent range, where a decoded value overflows
    for s in streams:
        hdr = s[:: rate // 2]
        sel = rng.random(hdr.size) < 0.05
        hdr[sel] = rng.integers(248, 256, size=int(sel.sum()), dtype=np.uint8)
    local = workloads.gradient_iid(n) * np.float32(1e30)
    dstreams = [_dev(s) for s in streams]
    for k, loc in ((2, None), (3, None), (1, local), (3, local)):
        with np.errstate(all="ignore"):
            sums = oracle.reduce_decompress(streams[:k], loc, n, rate)
            want_c = oracle.reduce_mixed(streams[:k], loc, n, rate)
        dloc = None if loc is None else _dev(loc)
        got_raw = _host(gpu.zc_reduce_decompress(dstreams[:k], dloc, n, rate))
        got_c = _host(gpu.zc_reduce_mixed(dstreams[:k], dloc, n, rate)) if loc is not None else \
            _host(gpu.zc_reduce_compressed(dstreams[:k], n, rate))
        again = _host(gpu.zc_reduce_mixed(dstreams[:k], dloc, n, rate))
        assert np.array_equal(got_c, again)
        not_nan = ~np.isnan(sums)
        assert np.isinf(sums).sum() > 50 and (~not_nan).sum() < n // 4
        _assert_floats_equal(got_raw[not_nan], sums[not_nan], "reduce_decompress arbitrary bytes r%d k%d" % (rate, k))
        assert np.isnan(got_raw[~not_nan]).all()
        padded = np.concatenate([sums, np.repeat(sums[-1:], (-n) % 4)]).reshape(-1, 4)
        finite = np.repeat(np.isfinite(padded).all(axis=1), rate // 2)
        assert finite.sum() > 0.8 * finite.size
        _assert_bytes_equal(got_c[finite], want_c[finite], rate // 2, "reduce arbitrary bytes r%d k%d" % (rate, k))


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_configs_scaled_down_whole_buffer(gpu, oracle, config):
    """Every configuration's distribution at a size the reference finishes in
    seconds, at the configuration's own rate and at the other main rates; sizes
    span many workgroups and end in a ragged block."""
    rate0 = workloads.CONFIGS[config]["rate"]
    shrink = {1: 0, 2: 9, 3: 7, 4: 8, 5: 6}[config]
    for label, x in workloads.config_buffers(config, shrink)[:2]:
        for cut in (0, 3):  # whole, and with a ragged tail of 1 value
            xs = x[: x.size - cut]
            for rate in sorted(set((rate0,) + MAIN_RATES)):
                print("config", config, label, "n", xs.size, "rate", rate, flush=True)
                want_c = oracle.compress(xs, rate)
                got_c = gpu.zc_compress(_dev(xs), rate)
                _assert_bytes_equal(_host(got_c), want_c, rate // 2, "compress cfg%d %s r%d" % (config, label, rate))
                want_d = oracle.decompress(want_c, xs.size, rate)
                got_d = gpu.zc_decompress(got_c, xs.size, rate)
                _assert_floats_equal(_host(got_d), want_d, "decompress cfg%d %s r%d" % (config, label, rate))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 255 * 4 + 1, 256 * 4, 256 * 4 + 7, 1027, 65536 + 2])
def test_small_and_ragged_sizes(gpu, oracle, n):
    x = workloads.gradient_iid(70000)[:n]
    for rate in RATES:
        want_c = oracle.compress(x, rate)
        got_c = gpu.zc_compress(_dev(x), rate)
        assert got_c.numel() == gpu.zc_compressed_size(n, rate) == want_c.size
        _assert_bytes_equal(_host(got_c), want_c, rate // 2, "n=%d r%d" % (n, rate))
        _assert_floats_equal(_host(gpu.zc_decompress(got_c, n, rate)), oracle.decompress(want_c, n, rate),
                             "n=%d r%d" % (n, rate))


def test_only_the_stated_bytes_are_written(gpu, oracle):
    import torch
    x = workloads.gradient_iid(4096 + 2)
    for rate in MAIN_RATES:
        size = gpu.zc_compressed_size(x.size, rate)
        out = torch.full((size + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        rc = gpu.lib().zc_compress(_dev(x).data_ptr(), x.size, rate, out.data_ptr(), size,
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()
        h = _host(out)
        assert (h[size:] == 0xA5).all()
        _assert_bytes_equal(h[:size], oracle.compress(x, rate), rate // 2, "canary r%d" % rate)
        dst = torch.full((x.size + 16,), -77.0, dtype=torch.float32, device="cuda")
        gpu.zc_decompress(out[:size].clone(), x.size, rate, d_out=dst)
        hd = _host(dst)
        assert (hd[x.size:] == -77.0).all()
        _assert_floats_equal(hd[: x.size], oracle.decompress(h[:size], x.size, rate), "canary r%d" % rate)


def test_empty_and_errors_on_device(gpu):
    import torch
    e = torch.empty(0, dtype=torch.float32, device="cuda")
    assert gpu.zc_compress(e, 8).numel() == 0
    assert gpu.zc_decompress(torch.empty(0, dtype=torch.uint8, device="cuda"), 0, 8).numel() == 0
    x = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(gpu.ZcError) as err:
        gpu.zc_compress(x, 8, d_out=torch.empty(63, dtype=torch.uint8, device="cuda"))
    assert err.value.code == gpu.ZC_ERR_CAPACITY
    with pytest.raises(gpu.ZcError):
        gpu.zc_compress(x, 9)
    with pytest.raises(gpu.ZcError) as err:
        gpu.zc_compress(x[1:], 8)  # 4-byte aligned only
    assert err.value.code == gpu.ZC_ERR_ALIGN


def test_runs_on_a_side_stream(gpu, oracle):
    import torch
    x = workloads.activation_gelu(1 << 16)
    s = torch.cuda.Stream()
    dx = _dev(x)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        c = gpu.zc_compress(dx, 16)
        d = gpu.zc_decompress(c, x.size, 16, stream=s)
    s.synchronize()
    want_c = oracle.compress(x, 16)
    _assert_bytes_equal(_host(c), want_c, 8, "side stream")
    _assert_floats_equal(_host(d), oracle.decompress(want_c, x.size, 16), "side stream")


# ---- reduce ---------------------------------------------------------------------------------

@pytest.mark.parametrize("rate", MAIN_RATES + (12, 32))
def test_reduce_matches_reference(gpu, oracle, rate):
    n = 4 * 3000 + 2
    peers = [workloads.gradient_lowrank(50, 240, tail=2, config=5, index=p) for p in range(13)]
    comp = [oracle.compress(p, rate) for p in peers]
    dcomp = [_dev(c) for c in comp]
    for k in (1, 2, 3, 5, 8, 13):   # (the kernel takes the chunks of a tile in groups of four or eight)
        print("reduce rate", rate, "k", k, flush=True)
        want = oracle.reduce_compressed(comp[:k], n, rate)
        got = gpu.zc_reduce_compressed(dcomp[:k], n, rate)
        _assert_bytes_equal(_host(got), want, rate // 2, "reduce r%d k%d" % (rate, k))
    # sixteen chunks, and edge values (subnormal sums, exact cancellation)
    e = workloads.edge_values(5)
    e = e[np.abs(e) < 1e30]
    e = e[: e.size // 4 * 4]
    ce = [oracle.compress(np.roll(e, 4 * i) * np.float32(1 if i % 2 else -1), rate) for i in range(16)]
    want = oracle.reduce_compressed(ce, e.size, rate)
    got = gpu.zc_reduce_compressed([_dev(c) for c in ce], e.size, rate)
    _assert_bytes_equal(_host(got), want, rate // 2, "reduce edge r%d k16" % rate)


def test_ring_chain_in_place(gpu, oracle):
    """One GPU's share of a compressed ring all-reduce at small size: seven pairwise
    steps, each writing over the accumulator, then the final decompress."""
    rate, n = 4, 1 << 17
    peers = [b for _, b in workloads.config_buffers(5, 8)]
    assert peers[0].size == n
    comp = [oracle.compress(p, rate) for p in peers]
    acc_ref = comp[0]
    for j in range(1, 8):
        acc_ref = oracle.reduce_compressed([acc_ref, comp[j]], n, rate)
    acc = _dev(comp[0]).clone()
    for j in range(1, 8):
        gpu.zc_reduce_compressed([acc, _dev(comp[j])], n, rate, d_out=acc)
    _assert_bytes_equal(_host(acc), acc_ref, rate // 2, "ring chain")
    _assert_floats_equal(_host(gpu.zc_decompress(acc, n, rate)), oracle.decompress(acc_ref, n, rate), "ring final")
    # the direct-exchange form: all eight at once
    want8 = oracle.reduce_compressed(comp, n, rate)
    _assert_bytes_equal(_host(gpu.zc_reduce_compressed([_dev(c) for c in comp], n, rate)), want8, 2, "k=8")


@pytest.mark.parametrize("rate", MAIN_RATES)
def test_ring_hop_variants_match_reference(gpu, oracle, rate):
    """Compressed chunks plus raw local values -> compressed sum, and -> fp32 sum."""
    n = 4 * 5000 + 1   # four whole tiles of 1024 blocks, a partial tile, a ragged block
    peers = [workloads.gradient_lowrank(70, 285, tail=n - 70 * 285, config=5, index=p) for p in range(4)]
    local = workloads.gradient_lowrank(70, 285, tail=n - 70 * 285, config=5, index=9)
    comp = [oracle.compress(p, rate) for p in peers]
    dcomp = [_dev(c) for c in comp]
    dlocal = _dev(local)
    for k in (1, 2, 4):
        print("ring hop rate", rate, "k", k, flush=True)
        for loc, dloc in ((local, dlocal), (None, None)):
            want = oracle.reduce_mixed(comp[:k], loc, n, rate)
            got = gpu.zc_reduce_mixed(dcomp[:k], dloc, n, rate)
            _assert_bytes_equal(_host(got), want, rate // 2, "mixed r%d k%d local=%s" % (rate, k, loc is not None))
            want = oracle.reduce_decompress(comp[:k], loc, n, rate)
            got = gpu.zc_reduce_decompress(dcomp[:k], dloc, n, rate)
            _assert_floats_equal(_host(got), want, "to-raw r%d k%d local=%s" % (rate, k, loc is not None))
    # in place: the accumulator chunk is overwritten, the fp32 sum lands in the local buffer
    acc = dcomp[0].clone()
    gpu.zc_reduce_mixed([acc], dlocal, n, rate, d_out=acc)
    _assert_bytes_equal(_host(acc), oracle.reduce_mixed(comp[:1], local, n, rate), rate // 2, "mixed in place")
    buf = dlocal.clone()
    gpu.zc_reduce_decompress(dcomp[:2], buf, n, rate, d_out=buf)
    _assert_floats_equal(_host(buf), oracle.reduce_decompress(comp[:2], local, n, rate), "to-raw in place")


def test_full_ring_on_one_share(gpu, oracle):
    """What one rank does to its share over a whole compressed ring all-reduce with raw
    local gradients: compress, six mixed hops, and a final hop to fp32."""
    rate, n = 8, 1 << 16
    raw = [workloads.gradient_lowrank(256, 256, config=5, index=p) for p in range(8)]
    acc_ref = oracle.compress(raw[0], rate)
    acc = gpu.zc_compress(_dev(raw[0]), rate)
    for p in range(1, 7):
        acc_ref = oracle.reduce_mixed([acc_ref], raw[p], n, rate)
        gpu.zc_reduce_mixed([acc], _dev(raw[p]), n, rate, d_out=acc)
    _assert_bytes_equal(_host(acc), acc_ref, rate // 2, "ring accumulator")
    _assert_floats_equal(_host(gpu.zc_reduce_decompress([acc], _dev(raw[7]), n, rate)),
                         oracle.reduce_decompress([acc_ref], raw[7], n, rate), "ring result")


# ---- half-precision messages ---------------------------------------------------------------

def _half_bits(x, name):
    if name == "f16":
        with np.errstate(over="ignore"):
            return x.astype(np.float16).view(np.uint16)
    return (x.view(np.uint32) >> 16).astype(np.uint16)   # any bf16 pattern is a valid input


@pytest.mark.parametrize("name", ["bf16", "f16"])
def test_half_precision_messages(gpu, oracle, name):
    import torch
    tdtype = torch.bfloat16 if name == "bf16" else torch.float16
    code = oracle.BF16 if name == "bf16" else oracle.F16
    x = np.concatenate([workloads.gradient_iid(40000), workloads.activation_gelu(30000), workloads.parameters(9003),
                        workloads.edge_values(3)])
    x = x[np.abs(x) < 6e4] if name == "f16" else x      # keep fp16 inputs finite
    h = _half_bits(x, name)
    n = h.size
    dh = torch.from_numpy(h.view(np.int16)).cuda().view(tdtype)
    for rate in RATES:
        print("half", name, "rate", rate, flush=True)
        want_c = oracle.compress_half(h, code, rate)
        got_c = gpu.zc_compress_half(dh, rate)
        _assert_bytes_equal(_host(got_c), want_c, rate // 2, "compress %s r%d" % (name, rate))
        want_d = oracle.decompress_half(want_c, n, rate, code)
        got_d = gpu.zc_decompress_half(got_c, n, rate, dtype=tdtype)
        got_bits = _host(got_d.view(torch.int16)).view(np.uint16)
        assert np.array_equal(got_bits, want_d), ("decompress %s r%d" % (name, rate), np.flatnonzero(got_bits != want_d)[:5])
    # the stream is the ordinary format: the fp32 calls read it, and fp32 streams decode to halves
    c32 = gpu.zc_compress(_dev(x), 16)
    want = oracle.decompress_half(oracle.compress(x, 16), x.size, 16, code)
    got = _host(gpu.zc_decompress_half(c32, x.size, 16, dtype=tdtype).view(torch.int16)).view(np.uint16)
    assert np.array_equal(got, want)
    for m in (1, 2, 3, 5, 1027):
        got_c = gpu.zc_compress_half(dh[:m].clone(), 8)
        _assert_bytes_equal(_host(got_c), oracle.compress_half(h[:m], code, 8), 4, "ragged %s %d" % (name, m))
        got = _host(gpu.zc_decompress_half(got_c, m, 8, dtype=tdtype).view(torch.int16)).view(np.uint16)
        assert np.array_equal(got, oracle.decompress_half(_host(got_c), m, 8, code))


# ---- full-size configurations, sampled comparison -------------------------------------------------

def _sample_ranges(blocks, count, length, seed):
    rng = np.random.default_rng(seed)
    starts = set([0, max(0, blocks - length)])
    starts.update(int(s) for s in rng.integers(0, max(1, blocks - length), size=count))
    return sorted(starts)


@pytest.mark.parametrize("config", [1, 2, 3, 4])
def test_full_size_configs_sampled(gpu, oracle, config):
    """The benchmark's own buffers and launch shapes; the reference recomputes
    sampled runs of blocks (blocks are independent, so any run is comparable)."""
    rate = workloads.CONFIGS[config]["rate"]
    bb = rate // 2
    for label, x in workloads.config_buffers(config):
        print("full config", config, label, "n", x.size, flush=True)
        n = x.size
        dx = _dev(x)
        dc = gpu.zc_compress(dx, rate)
        dd = gpu.zc_decompress(dc, n, rate)
        length = 4096
        for b0 in _sample_ranges(n // 4, 48, length, seed=config):
            xs = x[4 * b0: 4 * (b0 + length)]
            want_c = oracle.compress(xs, rate)
            got_c = _host(dc[b0 * bb: b0 * bb + want_c.size])
            _assert_bytes_equal(got_c, want_c, bb, "cfg%d %s blocks from %d" % (config, label, b0))
            got_d = _host(dd[4 * b0: 4 * b0 + xs.size])
            _assert_floats_equal(got_d, oracle.decompress(want_c, xs.size, rate), "cfg%d %s from %d" % (config, label, b0))
        del dx, dc, dd


def test_full_size_ring_share_sampled(gpu, oracle):
    """Configuration 5 at full size: eight chunks of 2^25 values at rate 4, the seven
    ring steps in place, the final decompress, and the single eight-way reduce."""
    rate, bb = 4, 2
    peers = [b for _, b in workloads.config_buffers(5)]
    n = peers[0].size
    assert n == 1 << 25
    dcomp = [gpu.zc_compress(_dev(p), rate) for p in peers]
    acc = dcomp[0].clone()
    for j in range(1, 8):
        gpu.zc_reduce_compressed([acc, dcomp[j]], n, rate, d_out=acc)
    final = gpu.zc_decompress(acc, n, rate)
    all8 = gpu.zc_reduce_compressed(dcomp, n, rate)
    dlocal = _dev(peers[7])
    mixed = gpu.zc_reduce_mixed(dcomp[:2], dlocal, n, rate)
    to_raw = gpu.zc_reduce_decompress(dcomp[:2], dlocal, n, rate)
    length = 2048
    for b0 in _sample_ranges(n // 4, 24, length, seed=5):
        print("ring share blocks from", b0, flush=True)
        sl = slice(4 * b0, 4 * (b0 + length))
        comp = [oracle.compress(p[sl], rate) for p in peers]
        for j in range(8):
            _assert_bytes_equal(_host(dcomp[j][b0 * bb:(b0 + length) * bb]), comp[j], bb, "peer %d" % j)
        ref = comp[0]
        for j in range(1, 8):
            ref = oracle.reduce_compressed([ref, comp[j]], 4 * length, rate)
        _assert_bytes_equal(_host(acc[b0 * bb:(b0 + length) * bb]), ref, bb, "ring from %d" % b0)
        _assert_floats_equal(_host(final[sl]), oracle.decompress(ref, 4 * length, rate), "final from %d" % b0)
        _assert_bytes_equal(_host(all8[b0 * bb:(b0 + length) * bb]),
                            oracle.reduce_compressed(comp, 4 * length, rate), bb, "k=8 from %d" % b0)
        _assert_bytes_equal(_host(mixed[b0 * bb:(b0 + length) * bb]),
                            oracle.reduce_mixed(comp[:2], peers[7][sl], 4 * length, rate), bb, "mixed from %d" % b0)
        _assert_floats_equal(_host(to_raw[sl]), oracle.reduce_decompress(comp[:2], peers[7][sl], 4 * length, rate),
                             "to-raw from %d" % b0)
