"""Counter-based random numbers for synthetic tensors.

Element i of the stream with seed s is a pure function of (s, i): a 64-bit
mixing function of the splitmix family turns the counter into uniform bits,
and a Box-Muller transform in fp64 turns two uniforms into one standard
normal.  Every consumer (oracle or GPU path) receives the values as host
arrays, so neither has to re-implement the generator.
"""
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(z):
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def _bits(seed, stream, n):
    with np.errstate(over="ignore"):
        ctr = np.arange(n, dtype=np.uint64)
        key = _mix64(np.uint64(seed) ^ (np.uint64(stream) << np.uint64(32)))
        return _mix64(ctr * np.uint64(0xD1342543DE82EF95) + key)


def _uniform01(seed, stream, n):
    # 53 random bits -> (0, 1): never exactly 0 so log() below is finite
    return ((_bits(seed, stream, n) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, shape, std=1.0):
    """N(0, std^2) samples in fp64, shape `shape`, fully determined by `seed`."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for lo in range(0, n, step):
        m = min(step, n - lo)
        # distinct sub-streams per block keep memory bounded for large tensors
        u1 = _uniform01(seed, 2 * (lo // step), m)
        u2 = _uniform01(seed, 2 * (lo // step) + 1, m)
        out[lo:lo + m] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (out * std).reshape(shape)


def uniform_int(seed, shape, high):
    """Integers uniform on {0, ..., high-1} (int32)."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.int32)
    step = 1 << 22
    for lo in range(0, n, step):
        m = min(step, n - lo)
        out[lo:lo + m] = (_bits(seed, 1000003 + lo // step, m) % np.uint64(high)).astype(np.int32)
    return out.reshape(shape)


def bf16_bits(x):
    """Round fp64/fp32 values to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return r.astype(np.uint16).reshape(f.shape)


def bits_to_f32(b):
    """bfloat16 bit patterns (uint16) -> fp32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """Values of x rounded once to bfloat16, returned as fp64 (exactly representable)."""
    return bits_to_f32(bf16_bits(x)).astype(np.float64)
