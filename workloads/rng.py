"""Counter-based integer generator: element i of tensor t under seed s is a pure
function of (s, t, i), so any slice of any tensor can be regenerated anywhere.

    r(s, t, i) = splitmix64_mix((s XOR t*GOLDEN) + i)        (all mod 2**64)
    value      = lo + (r mod (hi - lo + 1))

splitmix64_mix is the published SplitMix64 output function (Steele, Lea, Flood,
"Fast splittable pseudorandom number generators", 2014): add the golden-ratio
increment, then two xor-shift-multiply rounds and a final xor-shift.
"""
import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1


def splitmix64(x):
    """SplitMix64 output function on a uint64 numpy array (wraps mod 2**64)."""
    x = np.asarray(x, dtype=np.uint64)
    z = x + np.uint64(GOLDEN)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
    return z ^ (z >> np.uint64(31))


def splitmix64_scalar(x):
    """Same function on one Python int (used by tests to pin the array form)."""
    z = (x + GOLDEN) & _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def uniform_int(seed, tensor_id, count, lo, hi, dtype=np.int64, start=0):
    """`count` integers uniform on [lo, hi], elements start..start+count-1 of
    tensor `tensor_id` under `seed`, returned as a flat array of `dtype`."""
    if hi < lo:
        raise ValueError("empty range")
    base = ((int(seed) & _MASK) ^ ((int(tensor_id) * GOLDEN) & _MASK)) & _MASK
    out = np.empty(count, dtype=dtype)
    span = np.uint64(hi - lo + 1)
    chunk = 1 << 22
    with np.errstate(over="ignore"):
        for c0 in range(0, count, chunk):
            c1 = min(count, c0 + chunk)
            idx = np.arange(start + c0, start + c1, dtype=np.uint64) + np.uint64(base)
            r = splitmix64(idx) % span
            out[c0:c1] = (r.astype(np.int64) + lo).astype(dtype)
    return out
