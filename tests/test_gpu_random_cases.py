"""Seeded random cases: sizes, shapes, rates and value kinds drawn at random, every call of the
library against the reference on the whole result."""
import numpy as np
import pytest

from paper_2409_02423_amd import workloads

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _host(t):
    return t.cpu().numpy()


def _values(rng, n, kind):
    if kind == 0:
        return workloads.gradient_iid(n, std=float(10.0 ** rng.uniform(-6, 2)), config=1, index=int(rng.integers(0, 1000)))
    if kind == 1:
        return workloads.activation_gelu(n, config=3, index=int(rng.integers(0, 1000)))
    if kind == 2:      # mixed magnitudes, some exact zeros
        x = rng.standard_normal(n).astype(np.float32) * np.exp2(rng.integers(-40, 40, size=n)).astype(np.float32)
        x[rng.random(n) < 0.2] = 0
        return x
    return np.cumsum(rng.standard_normal(n).astype(np.float32) * np.float32(1e-3)).astype(np.float32)


@pytest.mark.parametrize("seed", range(6))
def test_one_dimensional(oracle, seed):
    from paper_2409_02423_amd import zc
    rng = np.random.default_rng(9100 + seed)
    for _ in range(6):
        n = int(rng.integers(1, 300000))
        rate = int(rng.choice([4, 8, 12, 16, 20, 24, 28, 32]))
        k = int(rng.choice([1, 2, 3, 4, 6, 9, 16]))
        xs = [_values(rng, n, int(rng.integers(0, 4))) for _ in range(k)]
        print("random 1-D: n", n, "rate", rate, "k", k, flush=True)
        comp = [oracle.compress(x, rate) for x in xs]
        dcomp = [zc.zc_compress(_dev(x), rate) for x in xs]
        for a, b in zip(dcomp, comp):
            assert np.array_equal(_host(a), b), (n, rate)
        assert np.array_equal(_host(zc.zc_decompress(dcomp[0], n, rate)).view(np.uint32),
                              oracle.decompress(comp[0], n, rate).view(np.uint32)), (n, rate)
        assert np.array_equal(_host(zc.zc_reduce_compressed(dcomp, n, rate)), oracle.reduce_compressed(comp, n, rate)), (n, rate, k)
        assert np.array_equal(_host(zc.zc_reduce_mixed(dcomp, _dev(xs[0]), n, rate)),
                              oracle.reduce_mixed(comp, xs[0], n, rate)), (n, rate, k)
        assert np.array_equal(_host(zc.zc_reduce_decompress(dcomp, _dev(xs[0]), n, rate)).view(np.uint32),
                              oracle.reduce_decompress(comp, xs[0], n, rate).view(np.uint32)), (n, rate, k)


@pytest.mark.parametrize("seed", range(4))
def test_matrices(seed):
    from oracle import zc2d_ref
    from paper_2409_02423_amd import zc
    rng = np.random.default_rng(9200 + seed)
    for _ in range(5):
        rows, cols = int(rng.integers(1, 400)), int(rng.integers(1, 700))
        rate = int(rng.choice([2, 4, 8, 16]))
        k = int(rng.integers(1, 4))
        ms = [_values(rng, rows * cols, int(rng.integers(0, 4))).reshape(rows, cols) for _ in range(k)]
        print("random 2-D:", rows, cols, "rate", rate, "k", k, flush=True)
        comp = [zc2d_ref.compress(m, rate) for m in ms]
        dcomp = [zc.zc2d_compress(_dev(m), rate) for m in ms]
        for a, b in zip(dcomp, comp):
            assert np.array_equal(_host(a), b), (rows, cols, rate)
        assert np.array_equal(_host(zc.zc2d_decompress(dcomp[0], rows, cols, rate)).view(np.uint32),
                              zc2d_ref.decompress(comp[0], rows, cols, rate).view(np.uint32)), (rows, cols, rate)
        assert np.array_equal(_host(zc.zc2d_reduce_compressed(dcomp, rows, cols, rate)),
                              zc2d_ref.reduce_compressed(comp, rows, cols, rate)), (rows, cols, rate, k)


@pytest.mark.parametrize("seed", range(4))
def test_lossless(seed):
    import torch
    from oracle import zl_ref
    from paper_2409_02423_amd import zc
    rng = np.random.default_rng(9300 + seed)
    for _ in range(5):
        n = int(rng.integers(1, 200000))
        kind = int(rng.integers(0, 6))
        if kind < 4:
            w = _values(rng, n, kind).view(np.uint32)
        elif kind == 4:
            w = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
        else:
            w = (rng.integers(0, 1 << 16, size=n, dtype=np.uint64).astype(np.uint32)) << np.uint32(16)
        print("random lossless: n", n, "kind", kind, flush=True)
        want = zl_ref.compress(w)
        c = zc.zl_compress(_dev(w.view(np.int32)))
        size = zc.zl_stream_bytes(c)
        assert size == want.size and np.array_equal(_host(c[:size]), want), (n, kind)
        assert np.array_equal(_host(zc.zl_decompress(c[:size], n, dtype=torch.int32)).view(np.uint32), w), (n, kind)
        h = (w >> np.uint32(16)).astype(np.uint16)
        c16 = zc.zl_compress16(_dev(h.view(np.int16)))
        size16 = zc.zl_stream_bytes(c16)
        assert np.array_equal(_host(c16[:size16]), zl_ref.compress16(h)), (n, kind)
        assert np.array_equal(_host(zc.zl_decompress16(c16[:size16], n, dtype=torch.int16)).view(np.uint16), h), (n, kind)
