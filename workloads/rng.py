"""Counter-based random numbers: value = f(seed, index), no hidden state.

The 64-bit mixer is the SplitMix64 output function (Steele, Lea & Flood,
"Fast splittable pseudorandom number generators", OOPSLA 2014) applied to the
counter ``seed * GOLDEN + index``; any element of any input can therefore be
regenerated on its own, which is what sampled verification of large tasks
needs.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def raw64(seed, index):
    """64 random bits for every entry of ``index`` (array of counters)."""
    index = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        ctr = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _GOLDEN + (index + np.uint64(1)) * _GOLDEN
    return _mix64(ctr)


def task_seed(seed_mix, task_id):
    """Per-task seed derived from the mix seed and the task id."""
    return int(raw64(int(seed_mix) ^ 0x5DEECE66D, np.uint64(task_id)))


def _chunks(n, offset):
    start = 0
    while start < n:
        m = min(_CHUNK, n - start)
        yield start, np.arange(offset + start, offset + start + m, dtype=np.uint64)
        start += m


def uniform01(seed, n, offset=0):
    """float32 U[0,1): top 24 bits of the 64-bit word / 2**24 (exact in fp32)."""
    out = np.empty(n, dtype=np.float32)
    for s, idx in _chunks(n, offset):
        out[s:s + idx.size] = (raw64(seed, idx) >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)
    return out


def normal(seed, n, offset=0, sigma=1.0):
    """float32 N(0, sigma^2) by Box-Muller on two 24-bit uniforms per value."""
    out = np.empty(n, dtype=np.float32)
    for s, idx in _chunks(n, offset):
        a = (raw64(seed, idx * np.uint64(2)) >> np.uint64(40)).astype(np.float64)
        b = (raw64(seed, idx * np.uint64(2) + np.uint64(1)) >> np.uint64(40)).astype(np.float64)
        u1 = (a + 1.0) * 2.0 ** -24          # (0, 1]
        u2 = b * 2.0 ** -24                  # [0, 1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + idx.size] = (sigma * z).astype(np.float32)
    return out


def exponential(seed, n, mean, offset=0):
    """float64 exponential gaps with the given mean (inverse-CDF)."""
    idx = np.arange(offset, offset + n, dtype=np.uint64)
    u = (raw64(seed, idx) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    return -mean * np.log1p(-u)


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        r = ((b + rnd) >> np.uint32(16)).astype(np.uint16)
    return r


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
