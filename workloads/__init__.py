"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random integers and describes shapes; it holds none of the method's
arithmetic, so both the oracle-side tests and the HIP-side harness may use it.

The paper evaluates on randomly generated feature and kernel vectors with p = q
(Section "Convolution layer evaluation") and on the layer shapes of a 4-bit detection CNN
whose trained weights and data set are not available here; uniform random quantised values
of the same shapes stand in for them.

Generator: numpy PCG64 seeded with crc32 of the case key, so every case is independent and
reproducible.  Value ranges: unsigned b-bit U{0..2^b-1}; signed b-bit
U{-2^(b-1)..2^(b-1)-1} (so signed 1-bit is {-1,0}); bipolar layers U{-1,+1}.
"""
import zlib

import numpy as np


def case_seed(*key) -> int:
    return zlib.crc32(repr(key).encode())


def rng_for(*key) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(case_seed(*key)))


def value_range(bits: int, signed: bool):
    if signed:
        return -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    return 0, (1 << bits) - 1


def uniform_values(rng, shape, bits: int, signed: bool) -> np.ndarray:
    """int8 array for signed values, uint8 array for unsigned ones (one value per byte)."""
    lo, hi = value_range(bits, signed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int8 if signed else np.uint8)


def bipolar_values(rng, shape) -> np.ndarray:
    return (rng.integers(0, 2, size=shape, dtype=np.int8) * 2 - 1).astype(np.int8)


# ---------------------------------------------------------------------------------------
# The five configurations.  Signed operands are int8 arrays, unsigned operands uint8 arrays.
# ---------------------------------------------------------------------------------------

def conv1d_case(bits: int, signed: bool, taps: int, rows: int, length: int, tag="c2"):
    """One case of the 1-D sweep: x[rows][length], one kernel g[taps] shared by all rows."""
    rng = rng_for(tag, bits, signed, taps, rows, length)
    x = uniform_values(rng, (rows, length), bits, signed)
    g = uniform_values(rng, (taps,), bits, signed)
    return x, g


def config1():
    """4096 uint4 inputs, 3 uint4 taps, valid padding, seed 0."""
    rng = np.random.Generator(np.random.PCG64(0))
    x = uniform_values(rng, (1, 4096), 4, False)
    g = uniform_values(rng, (3,), 4, False)
    return x, g


def conv2d_case(bits, a_signed, w_signed, n, c, h, w, co, kh, kw, tag="c3"):
    rng = rng_for(tag, bits, a_signed, w_signed, n, c, h, w, co, kh, kw)
    x = uniform_values(rng, (n, c, h, w), bits, a_signed)
    wt = uniform_values(rng, (co, c, kh, kw), bits, w_signed)
    return x, wt


def config3(scale: int = 1):
    """4-bit signed layer 1x64x56x56 -> 64 channels, 3x3, stride 1, pad 1."""
    return conv2d_case(4, True, True, 1, 64 // scale, 56 // scale, 56 // scale, 64 // scale, 3, 3)


def bipolar_case(n, c, h, w, co, kh, kw, tag="c4"):
    rng = rng_for(tag, n, c, h, w, co, kh, kw)
    return bipolar_values(rng, (n, c, h, w)), bipolar_values(rng, (co, c, kh, kw))


def config4(scale: int = 1):
    """Binarised layer 8x256x28x28 -> 256 channels, 3x3, stride 1, pad 1, values in {-1,+1}."""
    return bipolar_case(8 // min(scale, 8) or 1, 256 // scale, 28, 28, 256 // scale, 3, 3)


CNN_CHANNELS = [3, 16, 32, 64, 64, 64, 64, 64, 64]   # eight 3x3 layers ...
CNN_HEAD = 36                                         # ... then one 1x1 layer to 36 channels
CNN_POOL_AFTER = 4                                    # 2x2 max-pool after each of the first 4


def config5(height: int = 160, width: int = 320):
    """Complete 4-bit CNN: input 1x3xHxW uint4, nine conv layers with int4 weights.

    Returns (x, [weights...], [spec...]) where spec = dict(k, pad, pool).
    """
    rng = rng_for("c5", height, width)
    x = uniform_values(rng, (1, 3, height, width), 4, False)
    weights, specs = [], []
    for i in range(8):
        weights.append(uniform_values(rng, (CNN_CHANNELS[i + 1], CNN_CHANNELS[i], 3, 3), 4, True))
        specs.append(dict(k=3, pad=1, pool=i < CNN_POOL_AFTER))
    weights.append(uniform_values(rng, (CNN_HEAD, CNN_CHANNELS[-1], 1, 1), 4, True))
    specs.append(dict(k=1, pad=0, pool=False))
    return x, weights, specs
