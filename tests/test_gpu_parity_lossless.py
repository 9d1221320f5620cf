"""GPU parity for the lossless codec (zl_* calls of include/zc.h) against the CPU reference
oracle/zl_ref: streams byte for byte (header, table and payload), decoded words bit for bit."""
import numpy as np
import pytest

from paper_2409_02423_amd import workloads

pytestmark = pytest.mark.gpu
C = 8192


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_02423_amd import zc
    zc.lib()
    return zc


@pytest.fixture(scope="module")
def ref():
    from oracle import zl_ref
    zl_ref.lib()
    return zl_ref


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _host(t):
    return t.cpu().numpy()


def _same(got, want, what):
    got, want = np.asarray(got).reshape(-1), np.asarray(want).reshape(-1)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s: %d items differ, first at %d: got %r want %r" % (what, bad.size, bad[0], got[bad[0]], want[bad[0]]))


def _round_trip(gpu, ref, x, what):
    """x: numpy array of 32-bit items."""
    import torch
    w = np.ascontiguousarray(x).reshape(-1).view(np.int32)
    n = w.size
    want = ref.compress(w)
    cap = gpu.zl_max_compressed_size(n)
    out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    gpu.zl_compress(_dev(w), d_out=out[:cap])
    size = gpu.zl_stream_bytes(out)
    assert size == want.size, (what, size, want.size)
    h = _host(out)
    _same(h[:size], want, "stream " + what)
    assert (h[cap:] == 0xA5).all(), "wrote beyond the capacity: " + what
    back = gpu.zl_decompress(out[:size], n, dtype=torch.int32)
    _same(_host(back), w, "round trip " + what)
    # the reference's stream decodes alike on the GPU, from a buffer longer than the stream
    padded = np.concatenate([want, np.full(40, 0x5A, dtype=np.uint8)])
    _same(_host(gpu.zl_decompress(_dev(padded), n, dtype=torch.int32)), w, "decode of reference stream " + what)
    return size


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 1023, 1024, 1025, C - 1, C, C + 1, 3 * C + 4097, 64 * C + 17])
def test_sizes_and_ragged_tails(gpu, ref, n):
    print("lossless n", n, flush=True)
    _round_trip(gpu, ref, workloads.gradient_iid(max(n, 1))[:n], "gradient n=%d" % n)


def test_every_kind_of_bit_pattern(gpu, ref):
    rng = np.random.default_rng(4242)
    cases = {
        "edge": workloads.edge_values(9),
        "nan_inf": np.array([np.nan, -np.nan, np.inf, -np.inf, 0.0, -0.0] * 3000, dtype=np.float32),
        "random_bits": rng.integers(0, 1 << 32, size=5 * C + 77, dtype=np.uint64).astype(np.uint32),
        "zeros": np.zeros(4 * C + 5, dtype=np.float32),
        "constant": np.full(3 * C, -3.25, dtype=np.float32),
        "bf16_content": (workloads.activation_gelu(6 * C).view(np.uint32) & np.uint32(0xFFFF0000)),
        "smooth": np.cumsum(workloads.gradient_iid(7 * C + 3, std=1e-6)).astype(np.float32) + np.float32(1.0),
        "activation": workloads.activation_gelu(9 * C + 100),
        "moments": workloads.adam_second_moments(5 * C),
        "small_ints": rng.integers(0, 1000, size=3 * C + 1, dtype=np.int64).astype(np.int32),
    }
    for name, x in cases.items():
        print("lossless case", name, flush=True)
        _round_trip(gpu, ref, x, name)


def test_many_chunks_of_uneven_size(gpu, ref):
    """8192 chunks whose sizes change from chunk to chunk (runs of zeros, half-precision
    content, full-entropy words, smooth runs): every running total in the table is checked
    by the byte-for-byte comparison."""
    rng = np.random.default_rng(99)
    chunks = 8192
    x = workloads.gradient_iid(chunks * C, config=1, index=5).view(np.uint32).copy().reshape(chunks, C)
    kind = rng.integers(0, 5, size=chunks)
    x[kind == 0] = 0
    x[kind == 1] &= np.uint32(0xFFFF0000)
    x[kind == 2] = rng.integers(0, 1 << 32, size=(int((kind == 2).sum()), C), dtype=np.uint64).astype(np.uint32)
    x[kind == 3] = (np.float32(1.0) + np.cumsum(x[kind == 3].view(np.float32) * np.float32(1e-3), axis=1)).astype(np.float32).view(np.uint32)
    size = _round_trip(gpu, ref, x, "uneven chunks")
    print("uneven chunks: stream is %.3f of the message" % (size / (4.0 * x.size)), flush=True)


def test_errors_and_side_stream(gpu, ref):
    import torch
    x = _dev(workloads.gradient_iid(2 * C + 5))
    with pytest.raises(gpu.ZcError) as e:
        gpu.zl_compress(x, d_out=torch.zeros(gpu.zl_max_compressed_size(x.numel()) - 1, dtype=torch.uint8, device="cuda"))
    assert e.value.code == gpu.ZC_ERR_CAPACITY
    with pytest.raises(gpu.ZcError) as e:
        gpu.zl_stream_bytes(torch.zeros(64, dtype=torch.uint8, device="cuda"))
    assert e.value.code == gpu.ZC_ERR_STREAM
    with pytest.raises(gpu.ZcError) as e:
        gpu.zl_decompress(torch.zeros(32, dtype=torch.uint8, device="cuda"), 100)
    assert e.value.code == gpu.ZC_ERR_CAPACITY
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        c = gpu.zl_compress(x, stream=s)
        size = gpu.zl_stream_bytes(c, stream=s)
        y = gpu.zl_decompress(c[:size], x.numel(), stream=s)
    s.synchronize()
    _same(_host(c[:size]), ref.compress(_host(x)), "side stream")
    _same(_host(y).view(np.uint32), _host(x).view(np.uint32), "side stream round trip")


@pytest.mark.parametrize("n", [0, 1, 5, C - 3, C, 5 * C + 1234, 65536])
def test_16_bit_messages(gpu, ref, n):
    """bf16 activations, fp16 activations and arbitrary 16-bit patterns: stream and round trip
    against the reference, and the stream read back as 32-bit words."""
    import torch
    rng = np.random.default_rng(n + 1)
    f = workloads.activation_gelu(max(n, 1), config=3, index=2)[:n]
    cases = {"bf16": (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16),
             "fp16": f.astype(np.float16).view(np.uint16),
             "bits": np.arange(n, dtype=np.uint32).astype(np.uint16) if n == 65536 else rng.integers(0, 65536, size=n, dtype=np.uint16)}
    for name, h in cases.items():
        print("lossless 16-bit", name, "n", n, flush=True)
        want = ref.compress16(h)
        cap = gpu.zl_max_compressed_size(n)
        out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        gpu.zl_compress16(_dev(h.view(np.int16)), d_out=out[:cap])
        size = gpu.zl_stream_bytes(out)
        hh = _host(out)
        _same(hh[:size], want, "16-bit stream %s n=%d" % (name, n))
        assert (hh[cap:] == 0xA5).all()
        back = torch.full((n + 32,), -7, dtype=torch.int16, device="cuda")
        gpu.zl_decompress16(out[:size], n, d_out=back[:n])
        _same(_host(back[:n]).view(np.uint16), h, "16-bit round trip %s n=%d" % (name, n))
        assert (_host(back[n:]) == -7).all()
        words = gpu.zl_decompress(out[:size], n, dtype=torch.int32)
        _same(_host(words).view(np.uint32), h.astype(np.uint32) << np.uint32(16), "16-bit stream as words %s" % name)


def test_16_bit_decoder_on_streams_of_full_words(gpu, ref):
    """A stream whose words use all 32 bits, decoded as a 16-bit message: the decoder's short form
    (only the upper 16 planes, which is all a stream made from 16-bit words has) does not apply,
    and the result is the upper halves of the decoded words, as in the reference.  Chunks of both
    kinds side by side in one stream as well."""
    import torch
    n = 6 * C + 77
    full = workloads.gradient_iid(n, config=1, index=3).view(np.uint32)
    mixed = full.copy()
    mixed[C:3 * C] &= np.uint32(0xFFFF0000)          # two chunks that look as if made from 16-bit words
    for name, w in (("full words", full), ("mixed chunks", mixed)):
        print("lossless 16-bit decoder,", name, flush=True)
        stream = ref.compress(w)
        want = ref.decompress16(stream, n)
        assert np.array_equal(want, (w >> np.uint32(16)).astype(np.uint16))
        back = torch.full((n + 32,), -7, dtype=torch.int16, device="cuda")
        gpu.zl_decompress16(_dev(stream), n, d_out=back[:n])
        _same(_host(back[:n]).view(np.uint16), want, "16-bit decode of %s" % name)
        assert (_host(back[n:]) == -7).all()


def test_two_compressions_at_once(gpu, ref):
    """Two messages compressed on two streams at the same time (each kernel alone would fill
    the chip): both streams must come out as the reference's, several times over."""
    import torch
    a = workloads.gradient_iid(600 * C + 11, config=1, index=8)
    b = workloads.activation_gelu(500 * C + 7, config=3, index=8)
    want_a, want_b = ref.compress(a), ref.compress(b)
    da, db = _dev(a), _dev(b)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(5):
        print("two compressions at once, repetition", rep, flush=True)
        with torch.cuda.stream(s1):
            ca = gpu.zl_compress(da, stream=s1)
        with torch.cuda.stream(s2):
            cb = gpu.zl_compress(db, stream=s2)
        s1.synchronize()
        s2.synchronize()
        _same(_host(ca[:gpu.zl_stream_bytes(ca)]), want_a, "stream a, repetition %d" % rep)
        _same(_host(cb[:gpu.zl_stream_bytes(cb)]), want_b, "stream b, repetition %d" % rep)


def test_arbitrary_bytes_stay_in_bounds(gpu):
    """Streams that no encoder produced: the output is unspecified, but nothing outside the
    output buffer is written and the call returns."""
    import torch
    rng = np.random.default_rng(5)
    n = 5 * C + 9
    for trial in range(4):
        s = rng.integers(0, 256, size=60000 + 1000 * trial, dtype=np.uint8)
        if trial >= 2:   # plausible table: increasing ends, the right marks
            ends = np.sort(rng.integers(0, 70000, size=6).astype(np.uint64)) | (np.uint64(2) << np.uint64(62))
            s[32:32 + 48] = ends.view(np.uint8)
        out = torch.full((n + 64,), -7, dtype=torch.int32, device="cuda")
        gpu.zl_decompress(_dev(s), n, d_out=out[:n])
        torch.cuda.synchronize()
        assert (_host(out[n:]) == -7).all()


def test_full_size_messages_sampled(gpu, ref):
    """The sizes bench.py times (2^28 words): the GPU stream must decode to the message on the
    GPU, agree with the reference in its header, in the table entries and payload of sampled
    runs of chunks (chunks are independent, so a run can be recomputed alone)."""
    import torch
    for label, x in (("gradient", workloads.config_buffers(2)[0][1]),):
        n = x.size
        dx = _dev(x)
        c = gpu.zl_compress(dx)
        size = gpu.zl_stream_bytes(c)
        y = gpu.zl_decompress(c[:size], n)
        assert torch.equal(y.view(torch.int32), dx.view(torch.int32)), label
        chunks = n // C
        head = _host(c[:32]).view(np.uint32)
        assert head[0] == 0x31304C5A and head[1] == chunks and head[2] == n and head[6] == 0 and head[7] == 0
        table = _host(c[32:32 + 8 * chunks]).view(np.uint64)
        assert (table >> np.uint64(62) == 2).all()
        ends = (table & np.uint64((1 << 62) - 1)).astype(np.int64)
        assert size == 32 + 8 * chunks + ends[-1]
        rng = np.random.default_rng(31)
        for c0 in sorted(set([0, chunks - 16] + [int(v) for v in rng.integers(0, chunks - 16, size=6)])):
            print("lossless full size", label, "chunks from", c0, flush=True)
            want = ref.compress(x[c0 * C:(c0 + 16) * C])
            wt = want[32:32 + 128].view(np.uint64) & np.uint64((1 << 62) - 1)
            start = int(ends[c0 - 1]) if c0 else 0
            _same(ends[c0:c0 + 16] - start, wt.astype(np.int64), "table from chunk %d" % c0)
            p0 = 32 + 8 * chunks + start
            _same(_host(c[p0:p0 + int(wt[-1])]), want[32 + 128:], "payload from chunk %d" % c0)
        print("lossless full size", label, "stream is %.4f of the message" % (size / (4.0 * n)), flush=True)
        del dx, c, y
