"""GPU parity for the 4 x 4 block codec (zc2d_* calls of include/zc.h) against the CPU
reference oracle/zc2d_ref, bit for bit: streams as bytes, matrices as fp32 bit patterns."""
import numpy as np
import pytest

from paper_2409_02423_amd import workloads

pytestmark = pytest.mark.gpu

RATES = (2, 4, 8, 16)


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_02423_amd import zc
    zc.lib()
    return zc


@pytest.fixture(scope="module")
def ref():
    from oracle import zc2d_ref
    zc2d_ref.lib()
    return zc2d_ref


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _host(t):
    return t.cpu().numpy()


def _same_bytes(got, want, rate, what):
    got, want = np.asarray(got).reshape(-1), np.asarray(want).reshape(-1)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s: %d bytes differ, first at byte %d (block %d)" %
                             (what, bad.size, bad[0], bad[0] // (2 * rate)))


def _same_floats(got, want, what):
    g, w = np.asarray(got).view(np.uint32), np.asarray(want).view(np.uint32)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    if not np.array_equal(g, w):
        bad = np.argwhere(g != w)
        raise AssertionError("%s: %d values differ, first at %s: got %08x want %08x" %
                             (what, len(bad), tuple(bad[0]), g[tuple(bad[0])], w[tuple(bad[0])]))


def _round_trip(gpu, ref, x, rate, what):
    rows, cols = x.shape
    want_c = ref.compress(x, rate)
    got_c = gpu.zc2d_compress(_dev(x), rate)
    _same_bytes(_host(got_c), want_c, rate, "compress " + what)
    want_d = ref.decompress(want_c, rows, cols, rate)
    got_d = gpu.zc2d_decompress(got_c, rows, cols, rate)
    _same_floats(_host(got_d), want_d, "decompress " + what)


def _matrix(rows, cols, seed, kind="lowrank"):
    if kind == "lowrank":
        return workloads.gradient_lowrank(rows, cols, config=2, index=seed).reshape(rows, cols)
    if kind == "act":
        return workloads.activation_gelu(rows * cols, config=3, index=seed).reshape(rows, cols)
    return workloads.gradient_iid(rows * cols, config=1, index=seed).reshape(rows, cols)


@pytest.mark.parametrize("rate", RATES)
def test_edge_values(gpu, ref, rate):
    """Zeros, signed zeros, subnormals, extremes and mixed magnitudes, in three shapes so
    that the same values fall into different blocks."""
    v = workloads.edge_values(33)
    for cols in (4, 12, 52):
        rows = v.size // cols
        print("2d edge values rate", rate, "shape", rows, cols, flush=True)
        _round_trip(gpu, ref, v[: rows * cols].reshape(rows, cols).copy(), rate, "edge %dx%d r%d" % (rows, cols, rate))


@pytest.mark.parametrize("rate", RATES)
def test_structured_blocks(gpu, ref, rate):
    """Constant, one-hot, checkerboard, striped, planar, outlier and nearly equal blocks at
    magnitudes over the whole exponent range, laid out as a matrix 36 blocks wide."""
    b = workloads.structured_blocks_4x4(11, 288)            # 8 kinds x 288 blocks
    x = b.reshape(-1, 36, 4, 4).transpose(0, 2, 1, 3).reshape(-1, 144).copy()
    print("2d structured blocks rate", rate, "shape", x.shape, flush=True)
    _round_trip(gpu, ref, x, rate, "structured r%d" % rate)


@pytest.mark.parametrize("rate", RATES)
def test_arbitrary_bytes_decode_alike(gpu, ref, rate):
    print("2d arbitrary bytes rate", rate, flush=True)
    rng = np.random.default_rng(300 + rate)
    rows, cols = 203, 410      # ragged in both directions
    size = ((rows + 3) // 4) * ((cols + 3) // 4) * 2 * rate
    s = rng.integers(0, 256, size=size, dtype=np.uint8)
    s[: size // 3] &= rng.integers(0, 256, size=size // 3, dtype=np.uint8)
    with np.errstate(all="ignore"):
        want = ref.decompress(s, rows, cols, rate)
    got = gpu.zc2d_decompress(_dev(s), rows, cols, rate)
    _same_floats(_host(got), want, "arbitrary bytes r%d" % rate)


SHAPES = [(1, 1), (1, 9), (9, 1), (3, 5), (4, 4), (5, 4), (4, 5), (8, 1024), (7, 1030), (1029, 7), (256, 1024),
          (258, 1026), (1023, 64), (64, 1023), (1025, 1028)]


@pytest.mark.parametrize("shape", SHAPES)
def test_small_and_ragged_shapes(gpu, ref, shape):
    rows, cols = shape
    x = _matrix(rows, cols, seed=rows % 7)
    for rate in RATES:
        print("2d shape", shape, "rate", rate, flush=True)
        _round_trip(gpu, ref, x, rate, "%dx%d r%d" % (rows, cols, rate))


@pytest.mark.parametrize("kind", ["lowrank", "act", "iid"])
def test_more_blocks_than_one_pass_of_the_grid(gpu, ref, kind):
    """4096 x 4100 values = 1.05 M blocks (the widest grid covers 1.05 M lanes only when
    256 * 16 workgroups are resident), and 2052 x 8200 with a ragged last block row."""
    for rows, cols in ((4096, 4100), (2050, 8202)):
        x = _matrix(rows, cols, seed=3, kind=kind)
        for rate in (4, 8):
            print("2d large", kind, rows, cols, "rate", rate, flush=True)
            _round_trip(gpu, ref, x, rate, "%s %dx%d r%d" % (kind, rows, cols, rate))


def test_only_the_stated_bytes_are_written(gpu, ref):
    import torch
    rows, cols, rate = 37, 1021, 4
    x = _matrix(rows, cols, seed=5)
    size = gpu.zc2d_compressed_size(rows, cols, rate)
    out = torch.full((size + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    gpu.zc2d_compress(_dev(x), rate, d_out=out)
    h = _host(out)
    _same_bytes(h[:size], ref.compress(x, rate), rate, "canary compress")
    assert (h[size:] == 0xA5).all()
    dec = torch.full((rows * cols + 64,), float("nan"), dtype=torch.float32, device="cuda")
    gpu.zc2d_decompress(out[:size], rows, cols, rate, d_out=dec)
    hd = _host(dec)
    _same_floats(hd[: rows * cols].reshape(rows, cols), ref.decompress(h[:size], rows, cols, rate), "canary decompress")
    assert np.isnan(hd[rows * cols:]).all()


def test_empty_and_errors_on_device(gpu):
    import torch
    x = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    assert gpu.zc2d_compress(torch.zeros((0, 8), dtype=torch.float32, device="cuda"), 4).numel() == 0
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_compress(x, 12)
    assert e.value.code == gpu.ZC_ERR_RATE
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_compress(x, 4, d_out=torch.zeros(31, dtype=torch.uint8, device="cuda"))
    assert e.value.code == gpu.ZC_ERR_CAPACITY
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_compress(x.reshape(-1)[1:33].reshape(4, 8), 4)
    assert e.value.code == gpu.ZC_ERR_ALIGN
    torch.cuda.synchronize()


def test_runs_on_a_side_stream(gpu, ref):
    import torch
    x = _matrix(512, 2048, seed=2)
    s = torch.cuda.Stream()
    dx = _dev(x)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        c = gpu.zc2d_compress(dx, 8, stream=s)
        d = gpu.zc2d_decompress(c, 512, 2048, 8, stream=s)
    s.synchronize()
    want_c = ref.compress(x, 8)
    _same_bytes(_host(c), want_c, 8, "side stream compress")
    _same_floats(_host(d), ref.decompress(want_c, 512, 2048, 8), "side stream decompress")


@pytest.mark.parametrize("rate", RATES)
def test_reduce_matches_reference(gpu, ref, rate):
    for rows, cols in ((64, 256), (61, 1027), (3, 5), (1030, 7)):
        mats = [_matrix(rows, cols, seed=10 + j) * np.float32(1 + j) for j in range(8)]
        comp = [ref.compress(m, rate) for m in mats]
        dcomp = [_dev(c) for c in comp]
        for k in (1, 2, 3, 8):
            print("2d reduce rate", rate, "shape", rows, cols, "k", k, flush=True)
            want = ref.reduce_compressed(comp[:k], rows, cols, rate)
            got = gpu.zc2d_reduce_compressed(dcomp[:k], rows, cols, rate)
            _same_bytes(_host(got), want, rate, "reduce %dx%d r%d k%d" % (rows, cols, rate, k))
        # in place over the first input, as a ring step does
        acc = dcomp[0].clone()
        gpu.zc2d_reduce_compressed([acc, dcomp[1]], rows, cols, rate, d_out=acc)
        _same_bytes(_host(acc), ref.reduce_compressed(comp[:2], rows, cols, rate), rate, "reduce in place")


@pytest.mark.parametrize("rate", RATES)
def test_reduce_on_arbitrary_bytes(gpu, ref, rate):
    """The three reduce calls on streams of arbitrary bytes, with plenty of exponent bytes at both
    ends of the range (where the scaling of a decoded value rounds to a subnormal or overflows,
    and the kernel's fused scale-and-add must give way to decode-then-add): fp32 sums equal the
    reference's wherever they are not NaN, stream bytes wherever the block's sums are finite."""
    print("2d reduce on arbitrary bytes, rate", rate, flush=True)
    rng = np.random.default_rng(700 + rate)
    rows, cols = 64, 320
    size = ref.compressed_size(rows, cols, rate)
    streams = [rng.integers(0, 256, size=size, dtype=np.uint8) for _ in range(3)]
    streams[1][: size // 2] &= rng.integers(0, 256, size=size // 2, dtype=np.uint8)
    for s in streams:
        hdr = s[:: 2 * rate]
        sel = rng.random(hdr.size)
        hdr[sel < 0.05] = rng.integers(248, 256, size=int((sel < 0.05).sum()), dtype=np.uint8)
        hdr[sel > 0.90] = rng.integers(0, 40, size=int((sel > 0.90).sum()), dtype=np.uint8)
    local = (workloads.gradient_iid(rows * cols) * np.float32(1e30)).reshape(rows, cols)
    dstreams = [_dev(s) for s in streams]
    for k, loc in ((2, None), (3, None), (1, local), (3, local)):
        with np.errstate(all="ignore"):
            sums = ref.reduce_decompress(streams[:k], loc, rows, cols, rate)
            want_c = ref.reduce_mixed(streams[:k], loc, rows, cols, rate)
        dloc = None if loc is None else _dev(loc)
        got_raw = _host(gpu.zc2d_reduce_decompress(dstreams[:k], dloc, rows, cols, rate))
        got_c = _host(gpu.zc2d_reduce_mixed(dstreams[:k], dloc, rows, cols, rate)) if loc is not None else \
            _host(gpu.zc2d_reduce_compressed(dstreams[:k], rows, cols, rate))
        not_nan = ~np.isnan(sums)
        assert np.isinf(sums).sum() > 50 and (~not_nan).sum() < sums.size // 4
        _same_floats(got_raw[not_nan], sums[not_nan], "2d reduce_decompress arbitrary bytes r%d k%d" % (rate, k))
        assert np.isnan(got_raw[~not_nan]).all()
        finite = np.isfinite(sums).reshape(rows // 4, 4, cols // 4, 4).all(axis=(1, 3)).reshape(-1)
        assert finite.sum() > 0.7 * finite.size
        per_byte = np.repeat(finite, 2 * rate)
        _same_bytes(got_c[per_byte], want_c[per_byte], rate, "2d reduce arbitrary bytes r%d k%d" % (rate, k))


@pytest.mark.parametrize("name", ["bf16", "f16"])
def test_half_precision_matrices(gpu, ref, name):
    import torch
    for rows, cols in ((64, 256), (37, 54), (5, 1028), (1026, 6)):
        f = (workloads.activation_gelu(rows * cols, config=3, index=rows) * np.float32(2.5)).reshape(rows, cols)
        if name == "f16":
            bits, code, tdt = f.astype(np.float16).view(np.uint16), ref.F16, torch.float16
        else:
            bits, code, tdt = (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16), ref.BF16, torch.bfloat16
        dbits = _dev(bits.view(np.int16)).view(tdt)
        for rate in RATES:
            print("2d", name, "shape", rows, cols, "rate", rate, flush=True)
            want = ref.compress_half(bits, code, rate)
            got = gpu.zc2d_compress_half(dbits, rate)
            _same_bytes(_host(got), want, rate, "%s compress %dx%d r%d" % (name, rows, cols, rate))
            back = gpu.zc2d_decompress_half(got, rows, cols, rate, dtype=tdt)
            wantd = ref.decompress_half(want, rows, cols, rate, code)
            assert np.array_equal(_host(back.view(torch.int16)).view(np.uint16), wantd), (name, rows, cols, rate)
    with pytest.raises(TypeError):
        gpu.zc2d_compress_half(torch.zeros((4, 4), device="cuda"), 4)
    assert gpu.lib().zc2d_compress_half(0x10000, 0, 4, 4, 4, 0x10000, 100, None) == gpu.ZC_ERR_DTYPE
    assert gpu.lib().zc2d_decompress_half(0x10000, 4, 4, 4, 7, 0x10000, None) == gpu.ZC_ERR_DTYPE


@pytest.mark.parametrize("rate", (4, 16))
def test_ring_hop_variants_match_reference(gpu, ref, rate):
    import torch
    for rows, cols in ((64, 256), (61, 1027), (2, 3)):
        mats = [_matrix(rows, cols, seed=20 + j) for j in range(3)]
        local = _matrix(rows, cols, seed=29)
        comp = [ref.compress(m, rate) for m in mats]
        dcomp = [_dev(c) for c in comp]
        dlocal = _dev(local)
        for k in (1, 2, 3):
            print("2d ring hop rate", rate, "shape", rows, cols, "k", k, flush=True)
            for loc, dloc in ((local, dlocal), (None, None)):
                got = gpu.zc2d_reduce_mixed(dcomp[:k], dloc, rows, cols, rate)
                _same_bytes(_host(got), ref.reduce_mixed(comp[:k], loc, rows, cols, rate), rate, "mixed k%d" % k)
                raw = gpu.zc2d_reduce_decompress(dcomp[:k], dloc, rows, cols, rate)
                _same_floats(_host(raw), ref.reduce_decompress(comp[:k], loc, rows, cols, rate), "to raw k%d" % k)
        # the fp32 output over the local matrix, as the last hop of a ring would do it
        acc = dlocal.clone()
        gpu.zc2d_reduce_decompress(dcomp[:2], acc, rows, cols, rate, d_out=acc)
        _same_floats(_host(acc), ref.reduce_decompress(comp[:2], local, rows, cols, rate), "in place over local")
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_reduce_mixed([], None, 8, 8, 4)
    assert e.value.code == gpu.ZC_ERR_K
    assert gpu.lib().zc2d_reduce_decompress(None, 1, None, 8, 8, 4, None, None) == gpu.ZC_ERR_NULL
    torch.cuda.synchronize()


def test_reduce_errors(gpu):
    import torch
    c = torch.zeros(gpu.zc2d_compressed_size(8, 8, 4), dtype=torch.uint8, device="cuda")
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_reduce_compressed([], 8, 8, 4, d_out=c)
    assert e.value.code == gpu.ZC_ERR_K
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_reduce_compressed([c] * 17, 8, 8, 4)
    assert e.value.code == gpu.ZC_ERR_K
    with pytest.raises(gpu.ZcError) as e:
        gpu.zc2d_reduce_compressed([c, c], 8, 8, 4, d_out=c[:16])
    assert e.value.code == gpu.ZC_ERR_CAPACITY
    torch.cuda.synchronize()


def test_full_size_reduce_sampled(gpu, ref):
    """Two 8192 x 32768 matrices reduced at rate 4, checked on sampled bands of block rows."""
    rows, cols, rate = 8192, 32768, 4
    bc = cols // 4
    mats = [workloads.gradient_lowrank(rows, cols, config=2, index=j).reshape(rows, cols) for j in range(2)]
    dcomp = [gpu.zc2d_compress(_dev(m), rate) for m in mats]
    out = gpu.zc2d_reduce_compressed(dcomp, rows, cols, rate)
    rng = np.random.default_rng(78)
    for bi in sorted(set([0, rows // 4 - 1] + [int(b) for b in rng.integers(0, rows // 4, size=4)])):
        print("2d full size reduce, block row", bi, flush=True)
        comp = [ref.compress(m[4 * bi: 4 * bi + 4], rate) for m in mats]
        want = ref.reduce_compressed(comp, 4, cols, rate)
        _same_bytes(_host(out[bi * bc * 2 * rate: (bi + 1) * bc * 2 * rate]), want, rate, "full reduce block row %d" % bi)


def test_full_size_gradient_matrix_sampled(gpu, ref):
    """The matrix the benchmark times the 2-D calls on (8192 x 32768 = 2^28 values with the
    low-rank structure of configuration 2), at the rates it is timed at; the reference
    recomputes sampled bands of block rows."""
    rows, cols = 8192, 32768
    x = workloads.gradient_lowrank(rows, cols, config=2, index=0).reshape(rows, cols)
    dx = _dev(x)
    bc = (cols + 3) // 4
    rng = np.random.default_rng(77)
    bands = sorted(set([0, rows // 4 - 1] + [int(b) for b in rng.integers(0, rows // 4, size=6)]))
    for rate in (2, 4, 8):
        dc = gpu.zc2d_compress(dx, rate)
        dd = gpu.zc2d_decompress(dc, rows, cols, rate)
        for bi in bands:
            print("2d full size rate", rate, "block row", bi, flush=True)
            xs = x[4 * bi: 4 * bi + 4]
            want_c = ref.compress(xs, rate)
            got_c = _host(dc[bi * bc * 2 * rate: (bi + 1) * bc * 2 * rate])
            _same_bytes(got_c, want_c, rate, "full r%d block row %d" % (rate, bi))
            _same_floats(_host(dd[4 * bi: 4 * bi + 4]), ref.decompress(want_c, 4, cols, rate),
                         "full r%d rows from %d" % (rate, 4 * bi))
        del dc, dd
