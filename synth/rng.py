"""Counter-based random numbers: splitmix64 -> (0,1) uniforms -> Box-Muller normals."""
import numpy as np

SEED = 181112174  # default seed for every synthetic tensor in this repository

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _key(seed, stream):
    s = np.array([np.uint64(seed)], dtype=np.uint64)
    t = np.array([np.uint64(stream)], dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_mix(s + _GOLDEN) ^ (t * _GOLDEN + _GOLDEN))[0]


def _raw(seed, stream, start, count):
    """`count` 64-bit words: word i is mix(key + (start+i+1)*golden)."""
    idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_key(seed, stream) + idx * _GOLDEN)


def uniform(seed, stream, count, start=0):
    """float64 uniforms in the open interval (0,1), 53 bits each."""
    r = _raw(seed, stream, start, count)
    return ((r >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, stream, shape, dtype=np.float32, chunk=1 << 22):
    """Standard normals of the given shape; element i uses uniforms 2i and 2i+1."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        u = uniform(seed, stream, 2 * m, start=2 * lo)
        z = np.sqrt(-2.0 * np.log(u[0::2])) * np.cos(2.0 * np.pi * u[1::2])
        out[lo:lo + m] = z.astype(dtype)
    return out.reshape(shape)


def f32_to_bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 array (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """float32 array rounded to the nearest bf16 value, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))
