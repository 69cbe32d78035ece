"""Counter-based generator: every value is a pure function of (seed, stream, index).

splitmix64's output mixer is applied to a per-stream key plus a Weyl step per index,
so any sub-range of any buffer can be regenerated alone (rows of a large batch can be
re-made on the host for spot checks without generating the whole batch).
"""
import numpy as np

BASE_SEED = 221115023

# stream ids: one per kind of buffer
STREAM = {
    "weights_teacher": 1,
    "weights_student": 2,
    "calibration": 3,
    "states": 4,
    "uniforms": 5,
    "done": 6,
    "hc": 7,
    "rectangles": 8,
    "monitor_logits": 9,
    "trajectory": 10,
}

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def u64(seed, stream, start, count):
    """count 64-bit words for indices start .. start+count-1 of (seed, stream)."""
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * _GOLD + np.uint64(stream))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(key + (idx + np.uint64(1)) * _GOLD)


def uniform01(seed, stream, start, count):
    """float32 in [0, 1): top 24 bits / 2**24 (exactly representable)."""
    return ((u64(seed, stream, start, count) >> np.uint64(40)).astype(np.float32)
            * np.float32(1.0 / 16777216.0))


def _uniform01_f64(seed, stream, start, count):
    return (u64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(seed, stream, start, count):
    """float32 N(0,1) by Box-Muller in double; value i uses words 2i and 2i+1."""
    w = _uniform01_f64(seed, stream, 2 * start, 2 * count)
    u1 = 1.0 - w[0::2]          # (0, 1]
    u2 = w[1::2]
    return (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)


def randint(seed, stream, start, count, lo, hi):
    """integers uniform in lo..hi inclusive (modulo reduction of the 64-bit word)."""
    span = np.uint64(hi - lo + 1)
    return (u64(seed, stream, start, count) % span).astype(np.int64) + lo
