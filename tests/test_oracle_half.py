"""Pins for the reference's half-precision entry points: widening against numpy's
float16 and the bf16 bit layout (all 65536 patterns), narrowing against numpy's
round-to-nearest-even cast and a closed form on bits, and the buffer calls as
compositions with the pinned fp32 codec."""
import numpy as np

from paper_2409_02423_amd import workloads

ALL16 = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def _widen_all(oracle, dtype):
    return np.array([oracle.widen(int(h), dtype) for h in ALL16], dtype=np.float32)


def test_widen_fp16_is_numpys(oracle):
    got = _widen_all(oracle, oracle.F16)
    want = ALL16.view(np.float16).astype(np.float32)
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok].view(np.uint32), want[ok].view(np.uint32))
    assert np.isnan(got[~ok]).all()


def test_widen_bf16_is_the_upper_half_of_fp32(oracle):
    got = _widen_all(oracle, oracle.BF16)
    want = (ALL16.astype(np.uint32) << 16).view(np.float32)
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok].view(np.uint32), want[ok].view(np.uint32))


def _float_samples():
    rng = np.random.default_rng(41)
    bits = rng.integers(0, 1 << 32, size=60000, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    f = f[np.isfinite(f)]
    h = ALL16.view(np.float16).astype(np.float32)
    h = h[np.isfinite(h)]
    ties = ((h[:-1].astype(np.float64) + h[1:].astype(np.float64)) / 2).astype(np.float32)  # exact midpoints
    b = (ALL16.astype(np.uint32) << 16).view(np.float32)
    b = b[np.isfinite(b)]
    bties = (b.view(np.uint32) | 0x8000).view(np.float32)      # midpoints between neighbouring bf16 values
    near = np.concatenate([np.nextafter(ties, np.float32(np.inf)), np.nextafter(ties, np.float32(-np.inf)),
                           np.nextafter(bties, np.float32(np.inf)), np.nextafter(bties, np.float32(-np.inf))])
    small = np.array([0.0, -0.0, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -26, 65504.0, 65519.9, 65520.0,
                      65536.0, 1e10, -1e10, np.inf, -np.inf, 3.3895314e38, 3.4e38], dtype=np.float32)
    return np.concatenate([f, h, ties, b, bties, near, small, workloads.edge_values(2)]).astype(np.float32)


def test_narrow_fp16_is_numpys_rounding(oracle):
    x = _float_samples()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.narrow(v, oracle.F16) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want), np.flatnonzero(got != want)[:5]


def test_narrow_bf16_closed_form_on_bits(oracle):
    """Round to nearest even on the bit pattern: add 0x7FFF plus the lowest kept bit,
    drop 16 bits (a carry into the exponent is the correct next binade or infinity)."""
    x = _float_samples()
    b = x.view(np.uint32).astype(np.uint64)
    want = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    got = np.array([oracle.narrow(v, oracle.BF16) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want), np.flatnonzero(got != want)[:5]


def test_narrow_inverts_widen(oracle):
    for dtype in (oracle.BF16, oracle.F16):
        w = _widen_all(oracle, dtype)
        ok = ~np.isnan(w)
        back = np.array([oracle.narrow(v, dtype) for v in w[ok]], dtype=np.uint16)
        assert np.array_equal(back, ALL16[ok])


def _half_inputs(dtype_name):
    x = np.concatenate([workloads.gradient_iid(4099), workloads.activation_gelu(4096), workloads.parameters(2048)])
    if dtype_name == "f16":
        return x.astype(np.float16).view(np.uint16)
    return (x.view(np.uint32) >> 16).astype(np.uint16)          # truncation: any bf16 pattern is a valid input


def test_buffer_calls_are_compositions(oracle):
    for name, dtype in (("bf16", oracle.BF16), ("f16", oracle.F16)):
        h = _half_inputs(name)
        wide = h.view(np.float16).astype(np.float32) if name == "f16" else (h.astype(np.uint32) << 16).view(np.float32)
        for rate in (4, 8, 16, 24):
            for n in (h.size, h.size - 1, 5, 1):
                c = oracle.compress_half(h[:n], dtype, rate)
                assert np.array_equal(c, oracle.compress(wide[:n], rate))
                d = oracle.decompress(c, n, rate)
                got = oracle.decompress_half(c, n, rate, dtype)
                if name == "f16":
                    with np.errstate(over="ignore"):
                        want = d.astype(np.float16).view(np.uint16)
                else:
                    b = d.view(np.uint32).astype(np.uint64)
                    want = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
                assert np.array_equal(got, want)


def test_narrowing_a_nan_gives_the_formats_quiet_nan(oracle):
    """Not-a-number narrows to one fixed pattern per format, the positive quiet NaN with an empty
    payload: 0x7FC0 (bf16), 0x7E00 (fp16), whatever the sign and payload of the fp32 NaN."""
    for bits in (0x7FC00000, 0xFFC00000, 0x7F800001, 0xFFFFFFFF, 0x7FC12345):
        v = np.array([bits], dtype=np.uint32).view(np.float32)[0]
        assert oracle.narrow(v, oracle.BF16) == 0x7FC0
        assert oracle.narrow(v, oracle.F16) == 0x7E00
