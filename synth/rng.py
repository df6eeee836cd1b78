"""Counter-based random arrays.

Element i of the array with id `array_id` under master seed `master` depends
only on (master, array_id, i), so any slice can be generated independently and
the CPU and GPU sides always see the same bytes.
"""
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(x):
    """One splitmix64 output step applied to every element of a uint64 array."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def stream_seed(master, array_id):
    """Per-array stream start: splitmix64(master xor array_id)."""
    return int(splitmix64(np.array([(int(master) ^ int(array_id)) & 0xFFFFFFFFFFFFFFFF],
                                   dtype=np.uint64))[0])


def _raw(master, array_id, n, lane):
    """n raw 64-bit words; `lane` (0 or 1) selects one of two independent words per element."""
    base = np.uint64(stream_seed(master, array_id))
    with np.errstate(over="ignore"):
        ctr = base + (np.arange(n, dtype=np.uint64) * np.uint64(2) + np.uint64(lane))
    return splitmix64(ctr)


def uniform01(master, array_id, n, lane=0):
    """fp64 uniforms in (0, 1): top 53 bits, offset by half an ulp so 0 never occurs."""
    r = _raw(master, array_id, n, lane)
    return ((r >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(master, array_id, n, mean=0.0, std=1.0):
    """fp64 normals by Box-Muller from two uniforms per element."""
    u1 = uniform01(master, array_id, n, 0)
    u2 = uniform01(master, array_id, n, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return mean + std * z


def uniform(master, array_id, n, lo, hi):
    return lo + (hi - lo) * uniform01(master, array_id, n, 0)


def integers(master, array_id, n, hi):
    """Integers uniform over [0, hi)."""
    return (_raw(master, array_id, n, 0) % np.uint64(hi)).astype(np.int64)


def f32_to_bf16_bits(a):
    """Round fp32 to bf16 bit patterns (uint16), ties to even; NaN stays NaN."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), r)
    return r


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
