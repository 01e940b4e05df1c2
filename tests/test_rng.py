"""Pins of the seeded input generator (workloads.rng)."""
import numpy as np

from workloads import rng


def test_splitmix64_published_vectors():
    # First five outputs of SplitMix64 seeded with 1234567 (the widely published
    # check values of the public-domain reference generator).
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    got = [rng.splitmix64_scalar((1234567 + i * rng.GOLDEN) & ((1 << 64) - 1)) for i in range(5)]
    assert got == want


def test_array_form_matches_scalar_form():
    xs = np.array([0, 1, 2**63, 2**64 - 1, 1234567, 0xDEADBEEF], dtype=np.uint64)
    with np.errstate(over="ignore"):
        got = rng.splitmix64(xs)
    assert [int(g) for g in got] == [rng.splitmix64_scalar(int(x)) for x in xs]


def test_uniform_int_range_prefix_and_chunking():
    a = rng.uniform_int(3, 7, 10000, -127, 127, np.int8)
    assert a.min() >= -127 and a.max() <= 127 and a.min() < -100 and a.max() > 100
    b = rng.uniform_int(3, 7, 100, -127, 127, np.int8)
    assert (a[:100] == b).all()                       # a prefix is a prefix
    c = rng.uniform_int(3, 7, 50, -127, 127, np.int8, start=50)
    assert (a[50:100] == c).all()                     # any slice can be regenerated
    d = rng.uniform_int(4, 7, 100, -127, 127, np.int8)
    e = rng.uniform_int(3, 8, 100, -127, 127, np.int8)
    assert (b != d).any() and (b != e).any()          # seed and tensor id both matter
    big = rng.uniform_int(0, 1, (1 << 22) + 5, 0, 127, np.uint8)   # crosses a chunk border
    tail = rng.uniform_int(0, 1, 10, 0, 127, np.uint8, start=(1 << 22) - 5)
    assert (big[(1 << 22) - 5:] == tail).all()
    assert abs(float(big.mean()) - 63.5) < 0.1
