"""Counter-based random numbers keyed by (seed, tensor id, logical index).

Values depend only on the logical index of an element, never on a memory layout,
so a change of device layout cannot change any input.  The mixer is the public
splitmix64 finaliser; normals come from Box-Muller on two derived uniforms.
"""
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix(z):
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def _key(seed, tensor_id):
    k = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
    with np.errstate(over="ignore"):
        k = _splitmix(np.asarray(k, dtype=np.uint64))
        k = _splitmix(k ^ np.uint64(tensor_id & 0xFFFFFFFFFFFFFFFF))
    return k


def _bits(seed, tensor_id, count, stream):
    with np.errstate(over="ignore"):
        idx = np.arange(count, dtype=np.uint64)
        k = _key(seed, tensor_id * 4 + stream)
        return _splitmix(idx * np.uint64(0xD6E8FEB86659FD93) + k)


def uniform(seed, tensor_id, shape, lo=0.0, hi=1.0):
    """float64 uniforms in [lo, hi), element i of the flattened logical tensor from counter i."""
    count = int(np.prod(shape, dtype=np.int64))
    u = (_bits(seed, tensor_id, count, 0) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return (lo + (hi - lo) * u).reshape(shape)


def normal(seed, tensor_id, shape, mean=0.0, std=1.0):
    """float64 normals (Box-Muller), element i from counter i."""
    count = int(np.prod(shape, dtype=np.int64))
    u1 = ((_bits(seed, tensor_id, count, 1) >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / (1 << 53))
    u2 = (_bits(seed, tensor_id, count, 2) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + std * g).reshape(shape)


def integers(seed, tensor_id, shape, n):
    """int32 uniform over 0..n-1."""
    count = int(np.prod(shape, dtype=np.int64))
    return (_bits(seed, tensor_id, count, 3) % np.uint64(n)).astype(np.int32).reshape(shape)


def round_to_bf16(a):
    """Round float64/float32 values to the nearest bfloat16 (ties to even); returns float64.

    Used so that, for the bf16 workloads, both the oracle and the GPU path start from
    inputs and initial weights that are exactly representable in bf16.
    """
    f = np.ascontiguousarray(a, dtype=np.float32)
    b = f.view(np.uint32).astype(np.uint64)
    b = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return b.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))
