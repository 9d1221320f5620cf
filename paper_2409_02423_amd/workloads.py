"""Seeded synthetic message buffers (host numpy fp32).

These stand in for the collective messages of a GPT-NeoX-20B training run with
3D parallelism and ZeRO stage 1 (Sec. III, Table I; Sec. IV-B: PP=6, TP=4,
micro-batch 4, up to 192 GPUs, so 8 data-parallel replicas): data-parallel
gradient buckets, tensor-parallel activations, parameters and optimizer
states.  The training data and weights themselves are not available; only the
shapes, sizes and value distributions are reproduced.

This module holds input generation only: no step of the codec lives here, so
both the GPU tests and the CPU reference may draw their inputs from it.
Every generator is a pure function of its arguments (numpy PCG64 streams).
"""
import numpy as np
from scipy.special import ndtr

BASE_SEED = 20240902


def _rng(config, index):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 100 * config + index))


def gradient_iid(n, std=1e-3, config=1, index=0):
    """i.i.d. Gaussian gradient buffer (std given)."""
    r = _rng(config, index)
    x = r.standard_normal(n, dtype=np.float32)
    x *= np.float32(std)
    return x


def gradient_lowrank(rows, cols, tail=0, rank=8, std=1e-3, noise_std=1e-5, config=2, index=0):
    """Gradient bucket with low-rank structure.

    The first rows*cols values are, row-major, (std/sqrt(rank)) * U @ V with
    U (rows x rank) and V (rank x cols) standard normal, plus Gaussian noise of
    std noise_std; `tail` further values carry the noise term alone.
    """
    ru = _rng(config, 10 * index + 0)
    rv = _rng(config, 10 * index + 1)
    rn = _rng(config, 10 * index + 2)
    U = ru.standard_normal((rows, rank)).astype(np.float32)
    V = rv.standard_normal((rank, cols)).astype(np.float32)
    scale = np.float32(std / np.sqrt(rank))
    out = np.empty(rows * cols + tail, dtype=np.float32)
    step = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = (U[r0:r1] * scale) @ V
        noise = rn.standard_normal(blk.shape, dtype=np.float32)
        noise *= np.float32(noise_std)
        blk += noise
        out[r0 * cols:r1 * cols] = blk.reshape(-1)
    if tail:
        t = rn.standard_normal(tail, dtype=np.float32)
        t *= np.float32(noise_std)
        out[rows * cols:] = t
    return out


def activation_gelu(n, outlier_frac=0.01, outlier_gain=20.0, config=3, index=0):
    """GELU(z), z ~ N(0,1) (exact erf form, evaluated in fp64), with a fraction
    of the entries scaled up as outliers."""
    rz = _rng(config, 10 * index + 0)
    rm = _rng(config, 10 * index + 1)
    out = np.empty(n, dtype=np.float32)
    step = 1 << 23
    for a in range(0, n, step):
        b = min(n, a + step)
        z = rz.standard_normal(b - a)
        x = z * ndtr(z)
        mask = rm.random(b - a) < outlier_frac
        x[mask] *= outlier_gain
        out[a:b] = x.astype(np.float32)
    return out


def parameters(n, std=0.02, config=4, index=0):
    """Model parameters at initialisation scale."""
    r = _rng(config, 10 * index + 0)
    x = r.standard_normal(n, dtype=np.float32)
    x *= np.float32(std)
    return x


def adam_second_moments(n, grad_std=1e-6, config=4, index=1):
    """Adam second-moment estimates: squares of Gaussian gradients."""
    r = _rng(config, 10 * index + 0)
    g = r.standard_normal(n, dtype=np.float32)
    g *= np.float32(grad_std)
    return g * g


def edge_values(seed=7):
    """A buffer (multiple of 4 values) of blocks at the float edges: zeros,
    signed zeros, subnormals, the smallest normals, huge finite values, mixed
    magnitudes inside one block, exact constants, powers of two, and random
    bit patterns restricted to finite values."""
    r = np.random.Generator(np.random.PCG64(BASE_SEED + 9000 + seed))
    f = np.float32
    tiny = np.float32(1.401298464324817e-45)  # smallest subnormal
    fmin = np.float32(1.1754943508222875e-38)  # smallest normal
    fmax = np.float32(3.4028234663852886e38)
    blocks = [
        [0, 0, 0, 0], [-0.0, 0.0, 0.0, -0.0], [tiny, 0, 0, 0], [0, 0, 0, -tiny],
        [tiny, -tiny, 3 * tiny, 1000 * tiny], [fmin, fmin / f(2), 0, -fmin],
        [fmin, fmin, fmin, fmin], [fmin * f(1.5), -fmin / f(4), tiny, fmin * f(3)],
        [1, 1e-30, 0, 0], [1, 2, 3, 4], [0.001, -0.002, 0.0005, 0],
        [-1 / 3, -1 / 3, -1 / 3, -1 / 3], [fmax / f(4), -fmax / f(8), fmax / f(16), 1],
        [f(2.0) ** 126, -(f(2.0) ** 126), f(2.0) ** 100, 0],
        [f(2.0) ** 126 * f(1.9999), f(2.0) ** 126 * f(1.5), -(f(2.0) ** 126), f(2.0) ** 125],
        [1, 1, 1, 1], [-2, -2, -2, -2], [0.5, 0.5, 0.5, 0.5], [3, 3, 3, 3],
        [1, -1, 1, -1], [-1, 1, -1, 1], [1e-3, 1e3, 1e-3, 1e3],
        [f(1.0) - f(2.0) ** -24, 1, f(1.0) + f(2.0) ** -23, 1],
        [16777215, -16777215, 16777216, 1], [0, 0, 0, 1], [1, 0, 0, 0], [0, -1, 0, 0],
        [0, 0, 7, 0],
    ]
    fixed = np.array(blocks, dtype=np.float32).reshape(-1)
    # random finite bit patterns, whole exponent range below 2^127
    bits = r.integers(0, 1 << 32, size=4096, dtype=np.uint64).astype(np.uint32)
    expo = (bits >> 23) & 0xFF
    bits = np.where(expo >= 254, bits & np.uint32(0x807FFFFF) | np.uint32(100 << 23), bits)
    rnd = bits.astype(np.uint32).view(np.float32)
    # blocks whose values share a magnitude (typical of real messages)
    loc = r.standard_normal(4096).astype(np.float32) * np.repeat(
        np.exp2(r.integers(-140, 120, size=1024)).astype(np.float32), 4)
    sub = (r.integers(0, 1 << 23, size=1024, dtype=np.uint64).astype(np.uint32)
           | (r.integers(0, 2, size=1024, dtype=np.uint64).astype(np.uint32) << 31)).view(np.float32)
    return np.concatenate([fixed, rnd, loc, sub]).astype(np.float32)


def structured_blocks_4x4(seed=7, count=512):
    """4 x 4 blocks (an array of shape [blocks, 16], row-major blocks) with the shapes
    that stress a block coder: constant blocks, one non-zero value per block, pure
    checkerboards and stripes, ramps, a smooth block plus one outlier, and blocks whose
    values differ only in their last bits; each kind `count` times at magnitudes spread
    over the whole exponent range."""
    r = np.random.Generator(np.random.PCG64(BASE_SEED + 9500 + seed))
    mag = lambda: np.exp2(r.integers(-130, 120, size=(count, 1))).astype(np.float32)
    base = lambda: (1.0 + r.random((count, 1))).astype(np.float32) * np.where(r.random((count, 1)) < 0.5, -1, 1).astype(np.float32)
    ii, jj = np.meshgrid(np.arange(4), np.arange(4), indexing="ij")
    kinds = []
    kinds.append(np.repeat(base() * mag(), 16, axis=1))                                  # constant
    one = np.zeros((count, 16), dtype=np.float32)
    one[np.arange(count), r.integers(0, 16, size=count)] = (base() * mag())[:, 0]
    kinds.append(one)                                                                    # one value
    checker = ((-1.0) ** (ii + jj)).reshape(1, 16).astype(np.float32)
    kinds.append(checker * base() * mag())                                               # checkerboard
    kinds.append(((-1.0) ** ii).reshape(1, 16).astype(np.float32) * base() * mag())      # row stripes
    kinds.append(((-1.0) ** jj).reshape(1, 16).astype(np.float32) * base() * mag())      # column stripes
    ramp = (r.standard_normal((count, 1)) * ii.reshape(1, 16) + r.standard_normal((count, 1)) * jj.reshape(1, 16)
            + r.standard_normal((count, 1))).astype(np.float32)
    kinds.append(ramp * mag())                                                           # planes
    smooth = np.repeat(base(), 16, axis=1) * mag()
    smooth[np.arange(count), r.integers(0, 16, size=count)] *= np.float32(-37.0)
    kinds.append(smooth)                                                                 # outlier
    near = (np.repeat(base(), 16, axis=1).view(np.uint32) ^ r.integers(0, 4, size=(count, 16)).astype(np.uint32))
    kinds.append(near.view(np.float32) * mag())                                          # last bits differ
    out = np.concatenate(kinds).astype(np.float32)
    return np.where(np.isfinite(out), out, np.float32(1.0)).astype(np.float32)


# --- the five benchmark configurations ------------------------------------

CONFIGS = {
    1: dict(name="dp_gradient_iid_2^20", rate=8, n=1 << 20),
    2: dict(name="dp_gradient_bucket_lowrank_2^28", rate=4, n=1 << 28),
    3: dict(name="tp_activation_4x2048x6144", rate=16, n=4 * 2048 * 6144),
    4: dict(name="zero_params_and_adam_moments_1.5e8", rate=16, n=150_000_000),
    5: dict(name="ring_allreduce_share_8x2^25", rate=4, n=1 << 25, peers=8),
}


def config_buffers(config, scale_log2=0):
    """Host buffers of one benchmark configuration.

    scale_log2 > 0 shrinks every buffer by that power of two (same
    distributions and structure) for tests that run the CPU reference on the
    whole buffer.  Returns a list of (label, array).
    """
    s = scale_log2
    if config == 1:
        return [("grad", gradient_iid((1 << 20) >> s))]
    if config == 2:
        rows, cols = 6144 >> (s // 2), 43690 >> (s - s // 2)
        n = (1 << 28) >> s
        return [("grad", gradient_lowrank(rows, cols, tail=n - rows * cols))]
    if config == 3:
        return [("act", activation_gelu((4 * 2048 * 6144) >> s))]
    if config == 4:
        n = (150_000_000 >> s) // 4 * 4
        return [("param", parameters(n)), ("adam_v", adam_second_moments(n))]
    if config == 5:
        rows, cols = 4096 >> (s // 2), 8192 >> (s - s // 2)
        return [("peer%d" % p, gradient_lowrank(rows, cols, config=5, index=p)) for p in range(8)]
    raise ValueError("config must be 1..5")
