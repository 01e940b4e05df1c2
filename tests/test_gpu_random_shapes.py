"""Seeded random shapes through the kernels for few-channel layers on pictures (two-dimensional tiles, twin launches,
first layers straight off the picture) against the oracle, bit for bit: picture sizes that are no multiples of any tile,
channel counts with tails, every epilogue kind."""
import numpy as np
import pytest

from oracle import oracle as O

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_layers_on_the_two_dimensional_tile_kernel(seed):
    from gpu_util import gpu_conv2d
    from paper_2006_11735_amd import binding as B
    g = np.random.default_rng(seed)
    B.icnn_set_tuning("plane_always", 1)
    try:
        for it in range(12):
            k, cin = [(3, 48), (3, 64), (5, 64)][it % 3]
            cout = int(g.choice([16, 32] if k == 5 else [1, 3, 16, 24, 32, 48, 64]))
            n, h, w = int(g.integers(1, 3)), int(g.integers(1, 70)), int(g.integers(1, 110))
            x = g.integers(0, 128, size=(n, h, w, cin), dtype=np.uint8)
            wt = g.integers(-127, 128, size=(cout, k, k, cin), dtype=np.int8)
            b = g.integers(-4096, 4097, size=cout).astype(np.int32)
            sigma = 37.0 * 74 * (k * k * cin) ** 0.5
            kw = dict(pad=k // 2, mul=max(1, int(round(127 / (3.0 * sigma) * (1 << 25)))), shift=25)
            mode = it % 4
            if mode == 1:
                kw.update(out_mode="raw_s32")
            elif mode == 2:
                kw.update(res=g.integers(0, 128, size=(n, h, w, cout), dtype=np.uint8), res_mode="pre", res_mul=int(3 * sigma / 127),
                          res_shift=0)
            elif mode == 3:
                kw.update(res=g.integers(0, 256, size=(n, h, w, cout), dtype=np.uint8), res_mode="post", res_mul=3, res_shift=1,
                          out_mode="clamp_u8", lo=0, hi=255)
            want = O.conv2d(x, wt, b, **kw)
            got = gpu_conv2d(x, wt, b, **kw)
            assert (got == want).all(), (k, cin, cout, n, h, w, mode)
    finally:
        B.icnn_set_tuning("reset")


@pytest.mark.parametrize("seed", [4, 5])
def test_random_first_layers_off_the_picture(seed):
    from gpu_util import gpu_conv2d
    g = np.random.default_rng(seed)
    for _ in range(14):
        k, cin, cout = int(g.integers(1, 9)), int(g.integers(1, 5)), int(g.choice([32, 64]))
        pad = int(g.integers(0, k // 2 + 1))
        n, h, w = int(g.integers(1, 3)), int(g.integers(k, 50)), int(g.integers(k, 90))
        cbuf = cin + int(g.integers(0, 3))
        x = g.integers(0, 256, size=(n, h, w, cbuf), dtype=np.uint8)
        wt = g.integers(-127, 128, size=(cout, k, k, cin), dtype=np.int8)
        b = g.integers(-4096, 4097, size=cout).astype(np.int32)
        sigma = 74.0 * 74 * (k * k * cin) ** 0.5
        kw = dict(pad=pad, mul=max(1, int(round(127 / (3.0 * sigma) * (1 << 25)))), shift=25, in_sub128=True, cin=cin)
        want = O.conv2d(x, wt, b, **kw)
        got = gpu_conv2d(x, wt, b, **kw)
        assert (got == want).all(), (k, cin, cout, pad, n, h, w, cbuf)


@pytest.mark.parametrize("seed", [6, 7])
def test_random_twin_launches(seed):
    from test_gpu_twin import run_twin
    g = np.random.default_rng(seed)
    for it in range(9):
        ka, cin = [(5, 64), (3, 48), (3, 64)][it % 3]
        ca, cb = int(g.integers(1, 33)), int(g.integers(1, 33))
        n, h, w = int(g.integers(1, 3)), int(g.integers(1, 50)), int(g.integers(1, 80))
        got, want = run_twin(100 * seed + it, n, h, w, cin, ka, ca, cb, off_a=int(g.integers(0, 9)), xbuf=cin + 16 * int(g.integers(0, 2)))
        assert (got == want).all(), (ka, cin, ca, cb, n, h, w)
