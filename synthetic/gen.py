"""Counter-based seeded generators (numpy Philox) and bfloat16 storage helpers.

Values are drawn in fp32 and, for the bf16 workloads, rounded once to bfloat16
(round-to-nearest-even) on the host; both the oracle and the GPU path consume
exactly these rounded values.
"""
import numpy as np


def normal_f32(seed, stream, shape, std=1.0):
    """N(0, std) samples, fp32.  `seed` names the workload, `stream` the tensor
    inside it, so every tensor of a workload has its own Philox key."""
    rng = np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def to_bf16_bits(x_f32):
    """fp32 -> bfloat16 bit patterns (uint16), round-to-nearest-even.
    Inputs are finite (generated normals); NaN handling is not needed."""
    u = np.ascontiguousarray(x_f32, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits_u16):
    u = bits_u16.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def bf16_bits_to_f64(bits_u16):
    return bf16_bits_to_f32(bits_u16).astype(np.float64)
