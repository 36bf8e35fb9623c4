"""Counter-based seeded generators (splitmix64, Steele/Lea/Flood 2014).

One generator per tensor: the 64-bit state starts at ``seed * 2**32 +
tensor_id`` and advances by the golden-ratio increment once per element, in
row-major logical order (NCHW for activations, [out][in][kh][kw] for
weights).  Element i therefore depends only on (seed, tensor_id, i), which
lets numpy evaluate all elements at once.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _draws(seed: int, tensor_id: int, count: int) -> np.ndarray:
    """The first ``count`` 64-bit outputs of the tensor's generator."""
    s0 = np.uint64(((int(seed) << 32) + int(tensor_id)) & 0xFFFFFFFFFFFFFFFF)
    with np.errstate(over="ignore"):
        z = s0 + _GAMMA * np.arange(1, count + 1, dtype=np.uint64)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed, tensor_id, count):
    """Uniform on [0,1) with 24 random bits (exactly representable in fp32)."""
    return (_draws(seed, tensor_id, count) >> np.uint64(40)).astype(np.float64) * (2.0 ** -24)


def splitmix64_uniform(seed, tensor_id, shape, lo=-1.0, hi=1.0):
    """U[lo, hi) samples of the given shape, float64."""
    n = int(np.prod(shape))
    return (lo + (hi - lo) * _unit(seed, tensor_id, n)).reshape(shape)


def splitmix64_normal(seed, tensor_id, shape, std=1.0):
    """N(0, std^2) samples by Box-Muller on consecutive pairs of uniforms."""
    n = int(np.prod(shape))
    m = (n + 1) // 2
    u = _unit(seed, tensor_id, 2 * m)
    u1 = 1.0 - u[0::2]          # (0,1], keeps the log finite
    u2 = u[1::2]
    r = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(2.0 * np.pi * u2)
    out[1::2] = r * np.sin(2.0 * np.pi * u2)
    return (std * out[:n]).reshape(shape)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned
    as float32.  Used once, on the host, to fix the bytes both sides consume
    in the bf16 configurations; it is a storage-format conversion."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    bias = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        r = (bits + bias) & np.uint32(0xFFFF0000)
    nan = np.isnan(a)
    r = np.where(nan, bits | np.uint32(0x00400000), r).astype(np.uint32)
    return r.view(np.float32).reshape(a.shape)
