"""Seeded random layer shapes through the dispatcher (whatever kernel family and tile the
planners pick) against the oracle: the planners' rules are data-driven and route shapes to
many (kernel, tile) combinations that no hand-written list covers."""
import numpy as np
import pytest

import oracle
from helpers import TOL_F32, rel_err
from paper_2006_09791_amd import workloads as wl
from test_gpu_parity import gpu, run_conv  # noqa: F401  (gpu is the fixture the tests below use)

pytestmark = pytest.mark.gpu


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 3, 3, 3]))
        stride = int(rng.choice([1, 1, 2]))
        pad = k // 2 if rng.random() < 0.85 else int(rng.integers(0, 3))
        g = int(rng.choice([1, 2, 4, 8, 16, 32]))
        cpg = int(rng.choice([1, 2, 3, 4, 8, 16, 24, 32, 64]))
        kpg = int(rng.choice([1, 2, 4, 8, 12, 16, 32, 48, 64]))
        if rng.random() < 0.15:       # depthwise, sometimes with a channel multiplier
            g, cpg, kpg = int(rng.choice([8, 32, 96, 256])), 1, int(rng.choice([1, 1, 2]))
        h = int(rng.choice([4, 7, 8, 9, 12, 14, 16, 20, 28, 32, 56]))
        w = h if rng.random() < 0.7 else int(rng.choice([4, 6, 8, 10, 12, 16, 24, 28]))
        n = int(rng.choice([1, 1, 2, 3, 5, 16, 37, 64, 130, 300]))
        cin, cout = g * cpg, g * kpg
        ho, wo = wl.out_size(h, k, stride, pad), wl.out_size(w, k, stride, pad)
        if ho <= 0 or wo <= 0:
            continue
        macs = n * cout * cpg * k * k * ho * wo
        elems = n * (cin * h * w + cout * ho * wo)
        if macs > 150e6 or elems > 12e6:
            continue
        out.append(wl.ConvShape(n, cin, h, w, cout, k, k, stride, pad, g))
    return out


SHAPES = _random_shapes(140, 20260611)


@pytest.mark.parametrize("i", range(len(SHAPES)), ids=lambda i: "x".join(map(str, SHAPES[i])))
def test_random_shape_fp32(gpu, i):
    s = SHAPES[i]
    y, x, w, name = run_conv(gpu, s, seed=1000 + i)
    ref = oracle.conv2d_grouped(x, w, s.stride, s.pad, s.groups, threads=8)
    assert not np.isnan(y).any(), f"{name}: output not fully written for {s}"
    assert rel_err(y, ref) < TOL_F32, f"{name} for {s}"


@pytest.mark.parametrize("i", range(0, len(SHAPES), 4), ids=lambda i: "x".join(map(str, SHAPES[i])))
def test_random_shape_bf16(gpu, i):
    torch, b = gpu
    s = SHAPES[i]
    y, x, w, name = run_conv(gpu, s, seed=2000 + i, dtype=b.GSPC_BF16)
    _, xr = wl.round_to_bf16(x)
    _, wr = wl.round_to_bf16(w)
    ref = oracle.conv2d_grouped(xr, wr, s.stride, s.pad, s.groups, threads=8)
    assert not np.isnan(y).any(), f"{name}: output not fully written for {s}"
    assert rel_err(y, ref) < 1e-4, f"{name} for {s}"
