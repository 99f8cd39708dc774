"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
without reference to the oracle's own formula and without any GPU.

Each test names the mistake it would catch.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape)


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


# --------------------------------------------------------------------------
# P1: brute force.  A grouped conv is a standard conv whose dense weights are
# zero outside the block diagonal (Section II, Fig. 2).  The standard routine
# has no group logic and pads by copying, so a wrong group->channel mapping,
# stride or border rule in the grouped routine shows up here.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 0), (2, 1), (3, 2)])
@pytest.mark.parametrize("N,Cin,Cout,H,W,g,KH,KW", [
    (2, 6, 4, 5, 4, 2, 3, 3),
    (1, 8, 8, 6, 7, 4, 3, 2),
    (2, 6, 9, 7, 5, 3, 1, 3),
    (1, 4, 4, 5, 5, 4, 3, 3),     # depthwise
    (1, 4, 8, 5, 6, 4, 2, 2),     # depthwise with channel multiplier 2
])
def test_p1_block_diagonal_dense(N, Cin, Cout, H, W, g, KH, KW, stride, pad):
    if H + 2 * pad < KH or W + 2 * pad < KW:
        pytest.skip("kernel larger than padded input")
    x = _rand((N, Cin, H, W), 1)
    w = _rand((Cout, Cin // g, KH, KW), 2)
    CPG, KPG = Cin // g, Cout // g
    dense = np.zeros((Cout, Cin, KH, KW))
    for oc in range(Cout):
        j = oc // KPG
        dense[oc, j * CPG:(j + 1) * CPG] = w[oc]
    ref = oracle.conv2d_standard(x, dense, stride, pad)
    got = oracle.conv2d_grouped(x, w, stride, pad, g)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# P2: g = 1 is the standard convolution.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad,K", [(1, 1, 3), (2, 3, 7), (1, 0, 1), (2, 0, 1)])
def test_p2_g1_is_standard(stride, pad, K):
    x = _rand((2, 5, 9, 8), 3)
    w = _rand((7, 5, K, K), 4)
    np.testing.assert_allclose(oracle.conv2d_grouped(x, w, stride, pad, 1),
                               oracle.conv2d_standard(x, w, stride, pad),
                               rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# P3: the instrumented MAC counter equals Eq. 2 exactly (loop bounds, output
# size formula).  The right-hand side is typed out here, not taken from the
# oracle.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("N,Cin,Cout,H,W,g,K,stride,pad", [
    (1, 64, 64, 32, 32, 4, 3, 1, 1),
    (2, 6, 4, 5, 4, 2, 3, 2, 1),
    (1, 16, 16, 7, 7, 16, 3, 2, 1),
    (1, 3, 8, 15, 15, 1, 7, 2, 3),
])
def test_p3_mac_count(N, Cin, Cout, H, W, g, K, stride, pad):
    x = _rand((N, Cin, H, W), 5)
    w = _rand((Cout, Cin // g, K, K), 6)
    y, macs = oracle.conv2d_grouped(x, w, stride, pad, g, return_macs=True)
    Hout = (H + 2 * pad - K) // stride + 1
    Wout = (W + 2 * pad - K) // stride + 1
    assert y.shape == (N, Cout, Hout, Wout)
    expect = N * Cin * Cout * K * K * Hout * Wout // g
    assert macs == expect
    assert oracle.macs(N, Cin, Cout, K, K, Hout, Wout, g) == expect


def test_p3_config1_macs():
    # The small benchmark case is quoted at about 9.4 M MACs.
    assert oracle.macs(1, 64, 64, 3, 3, 32, 32, 4) == 9437184


def test_depthwise_7x7_stride2_output_is_4x4():
    assert oracle.out_dim(7, 3, 2, 1) == 4
    assert oracle.out_dim(224, 7, 2, 3) == 112
    assert oracle.out_dim(112, 3, 2, 1) == 56


# --------------------------------------------------------------------------
# P4: worked example of Fig. 3 (hand-derived sequences in tests/golden).
# --------------------------------------------------------------------------
def test_p4_fig3_worked_example():
    gold = _read_golden("fig3_worked_example.txt")
    x = np.arange(16.0).reshape(1, 4, 2, 2)
    w = np.arange(32.0).reshape(4, 2, 2, 2)
    y = oracle.conv2d_grouped(x, w, 1, 0, 2)
    assert y.shape == (1, 4, 1, 1)
    assert y.ravel().tolist() == gold["Y"]
    wp = oracle.alg1_pack_kernels(w, 2, 2, 2)
    assert wp.shape == (2, 1, 1, 2, 2, 2, 2)
    assert wp.ravel().tolist() == gold["W_packed"]
    xp = oracle.alg1_pack_inputs(x, 0, 2, 2)
    assert xp.shape == (2, 1, 1, 2, 2, 2)
    assert xp.ravel().tolist() == gold["X_packed"]
    # output reshape is the identity in flat memory
    yp = np.arange(4.0).reshape(2, 1, 1, 1, 1, 2)
    assert oracle.alg1_unpack_outputs(yp, 4, 2, 2).ravel().tolist() == gold["Y_unpack"]
    # full pipeline
    assert oracle.gspc_alg1(x, w, 1, 0, 2, 2, 2).ravel().tolist() == gold["Y"]


def test_p4_each_input_value_used_twice():
    # d(sum Y)/dX[i] = number of MACs that read X[i] when W == 1.
    w = np.ones((4, 2, 2, 2))
    base = oracle.conv2d_grouped(np.zeros((1, 4, 2, 2)), w, 1, 0, 2).sum()
    for i in range(16):
        x = np.zeros(16)
        x[i] = 1.0
        uses = oracle.conv2d_grouped(x.reshape(1, 4, 2, 2), w, 1, 0, 2).sum() - base
        assert uses == 2.0


# --------------------------------------------------------------------------
# P5: impulse response.  A single 1 in the input stamps the (un-flipped read,
# hence 180-degree rotated stamp) kernel, only in its own group's outputs.
# Catches a kernel flip, a transposed kh/kw, leakage between groups.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0), (2, 2)])
def test_p5_impulse(stride, pad):
    N, Cin, Cout, H, W, g, KH, KW = 2, 6, 6, 6, 7, 3, 3, 2
    CPG, KPG = Cin // g, Cout // g
    w = _rand((Cout, CPG, KH, KW), 7)
    n0, c0, h0, w0 = 1, 3, 2, 4
    x = np.zeros((N, Cin, H, W))
    x[n0, c0, h0, w0] = 1.0
    y = oracle.conv2d_grouped(x, w, stride, pad, g)
    Hout = (H + 2 * pad - KH) // stride + 1
    Wout = (W + 2 * pad - KW) // stride + 1
    expect = np.zeros((N, Cout, Hout, Wout))
    j = c0 // CPG
    for oc in range(j * KPG, (j + 1) * KPG):
        for oh in range(Hout):
            for ow in range(Wout):
                kh = h0 + pad - oh * stride
                kw = w0 + pad - ow * stride
                if 0 <= kh < KH and 0 <= kw < KW:
                    expect[n0, oc, oh, ow] = w[oc, c0 % CPG, kh, kw]
    assert np.array_equal(y, expect)


# --------------------------------------------------------------------------
# P6: all ones.  Y = CPG * (number of taps inside the image): zero padding.
# --------------------------------------------------------------------------
def test_p6_all_ones():
    Cin, Cout, g, H, W = 8, 4, 2, 5, 6
    CPG = Cin // g
    y = oracle.conv2d_grouped(np.ones((1, Cin, H, W)), np.ones((Cout, CPG, 3, 3)), 1, 1, g)
    assert y.shape == (1, Cout, H, W)
    assert np.all(y[0, :, 1:-1, 1:-1] == 9 * CPG)
    for c in ((0, 0), (0, -1), (-1, 0), (-1, -1)):
        assert np.all(y[0, :, c[0], c[1]] == 4 * CPG)
    assert np.all(y[0, :, 0, 1:-1] == 6 * CPG)
    assert np.all(y[0, :, 1:-1, 0] == 6 * CPG)


# --------------------------------------------------------------------------
# P7: depthwise with a rank-1 kernel separates into a column pass and a row
# pass of 1-D correlations (numpy.correlate is the library routine here).
# --------------------------------------------------------------------------
def test_p7_depthwise_separable():
    C, H, W = 5, 9, 11
    x = _rand((1, C, H, W), 8)
    u = _rand((C, 3), 9)
    v = _rand((C, 3), 10)
    w = np.einsum("ci,cj->cij", u, v).reshape(C, 1, 3, 3)
    y = oracle.conv2d_grouped(x, w, 1, 1, C)
    for c in range(C):
        rows = np.stack([np.correlate(np.pad(x[0, c, h], 1), v[c], "valid") for h in range(H)])
        cols = np.stack([np.correlate(np.pad(rows[:, i], 1), u[c], "valid") for i in range(W)], axis=1)
        np.testing.assert_allclose(y[0, c], cols, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# P8: linearity and equivariance under a permutation of whole groups.
# --------------------------------------------------------------------------
def test_p8_linearity_and_group_permutation():
    N, Cin, Cout, g = 2, 8, 12, 4
    x1, x2 = _rand((N, Cin, 6, 5), 11), _rand((N, Cin, 6, 5), 12)
    w = _rand((Cout, Cin // g, 3, 3), 13)
    a, b = 0.75, -1.5
    lhs = oracle.conv2d_grouped(a * x1 + b * x2, w, 2, 1, g)
    rhs = a * oracle.conv2d_grouped(x1, w, 2, 1, g) + b * oracle.conv2d_grouped(x2, w, 2, 1, g)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-13)
    perm = [2, 0, 3, 1]
    CPG, KPG = Cin // g, Cout // g
    xperm = np.concatenate([x1[:, p * CPG:(p + 1) * CPG] for p in perm], axis=1)
    wperm = np.concatenate([w[p * KPG:(p + 1) * KPG] for p in perm], axis=0)
    y = oracle.conv2d_grouped(x1, w, 2, 1, g)
    yperm = np.concatenate([y[:, p * KPG:(p + 1) * KPG] for p in perm], axis=1)
    assert np.array_equal(oracle.conv2d_grouped(xperm, wperm, 2, 1, g), yperm)


# --------------------------------------------------------------------------
# P9: Algorithm 1 taken literally equals the 7-loop definition bit for bit
# (same c, kh, kw summation order) for every legal pair of tile sizes.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("N,Cin,Cout,H,W,g,K,stride,pad", [
    (2, 8, 12, 6, 5, 2, 3, 1, 1),
    (1, 12, 6, 7, 7, 3, 3, 2, 1),
    (2, 4, 4, 5, 5, 4, 3, 1, 1),      # depthwise
    (1, 6, 6, 8, 8, 1, 1, 2, 0),
])
def test_p9_algorithm1_equals_definition(N, Cin, Cout, H, W, g, K, stride, pad):
    x = _rand((N, Cin, H, W), 14)
    w = _rand((Cout, Cin // g, K, K), 15)
    ref = oracle.conv2d_grouped(x, w, stride, pad, g)
    CPG, KPG = Cin // g, Cout // g
    for T_I, T_O in itertools.product(range(1, CPG + 1), range(1, KPG + 1)):
        if CPG % T_I or KPG % T_O:
            with pytest.raises(ValueError):
                oracle.gspc_alg1(x, w, stride, pad, g, T_I, T_O)
            continue
        assert np.array_equal(oracle.gspc_alg1(x, w, stride, pad, g, T_I, T_O), ref)


@pytest.mark.parametrize("N,Cin,Cout,H,W,g,K,stride,pad,T_I,T_O", [
    (2, 8, 16, 6, 5, 2, 3, 1, 1, 2, 8),
    (3, 12, 12, 7, 7, 3, 3, 2, 1, 4, 4),
    (2, 6, 6, 5, 5, 6, 3, 1, 1, 1, 1),       # depthwise
    (1, 4, 32, 9, 8, 1, 1, 1, 0, 4, 16),
    (1, 3, 24, 11, 11, 1, 7, 2, 3, 1, 3),    # a vector length that is not a power of two
])
def test_p9_vectorised_schedule_has_the_same_bits(N, Cin, Cout, H, W, g, K, stride, pad, T_I, T_O):
    # The timed "paper's method on the host" baseline: T_O filters as one vector,
    # (group, image) pairs over threads.  Same (c, kh, kw) order per output, so the
    # same bits as the plain stage (and hence as the definition, by the test above).
    x = _rand((N, Cin, H, W), 28)
    w = _rand((Cout, Cin // g, K, K), 29)
    ref = oracle.conv2d_grouped(x, w, stride, pad, g)
    for threads in (1, 3):
        got = oracle.gspc_alg1(x, w, stride, pad, g, T_I, T_O, vectorised=True, threads=threads)
        assert np.array_equal(got, ref)
    with pytest.raises(ValueError):
        oracle.gspc_alg1(x, w, stride, pad, g, T_I, T_O + 1 if (Cout // g) % (T_O + 1) else 65, vectorised=True)


def test_p9_depthwise_output_reshape_identity_for_batch_one():
    # Section III-B: for depthwise the output reshape is the identity (N = 1).
    yp = _rand((6, 1, 1, 4, 3, 1), 16)
    y = oracle.alg1_unpack_outputs(yp, 6, 6, 1)
    assert np.array_equal(y.ravel(), yp.ravel())


# --------------------------------------------------------------------------
# P10: third-party library cross-check (PyTorch CPU, float64).
# --------------------------------------------------------------------------
@pytest.mark.parametrize("N,Cin,Cout,H,W,g,KH,KW,stride,pad", [
    (2, 16, 24, 13, 9, 4, 3, 3, 1, 1),
    (1, 16, 16, 14, 14, 16, 3, 3, 2, 1),
    (1, 3, 8, 20, 20, 1, 7, 7, 2, 3),
    (2, 6, 6, 8, 9, 3, 2, 3, 2, 2),
    (1, 8, 16, 6, 6, 1, 1, 1, 1, 0),
])
def test_p10_torch_cpu_float64(N, Cin, Cout, H, W, g, KH, KW, stride, pad):
    torch = pytest.importorskip("torch")
    x = _rand((N, Cin, H, W), 17)
    w = _rand((Cout, Cin // g, KH, KW), 18)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w),
                                     stride=stride, padding=pad, groups=g).numpy()
    got, a = oracle.conv2d_grouped(x, w, stride, pad, g, return_abs=True)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert np.all(np.abs(got) <= a + 1e-15)
    sel = [Cout - 1, 0, Cout // 2]
    sub = oracle.conv2d_grouped_channels(x, w, sel, stride, pad, g)
    np.testing.assert_allclose(sub, ref[:, sel], rtol=0, atol=1e-12)


def test_threads_do_not_change_result():
    x = _rand((3, 8, 9, 9), 19)
    w = _rand((8, 2, 3, 3), 20)
    y1, m1 = oracle.conv2d_grouped(x, w, 1, 1, 4, return_macs=True, threads=1)
    y4, m4 = oracle.conv2d_grouped(x, w, 1, 1, 4, return_macs=True, threads=4)
    assert np.array_equal(y1, y4) and m1 == m4


# --------------------------------------------------------------------------
# P11: MAC column of Table II.  WRN-40-2 rebuilt layer by layer (stem 3->16,
# widths 32/64/128, six basic blocks per stage, 1x1 shortcut at each stage
# entry, 128->10 classifier), G(g) = grouped 3x3 a->a at the conv's output
# resolution followed by pointwise a->b.  The printed totals sit a constant
# 0.70 M above the convolution-only count in every row, so the row-to-row
# differences, which isolate the grouped layers and the 1/g scaling of Eq. 2,
# must match to the table's 0.01 M print precision.
# --------------------------------------------------------------------------
def _wrn40x2_macs(g):
    total = 0

    def conv3(a, b, hw_out):
        nonlocal total
        if g is None:
            total += oracle.macs(1, a, b, 3, 3, hw_out, hw_out, 1)
        else:
            gg = a if g == "N" else g
            total += oracle.macs(1, a, a, 3, 3, hw_out, hw_out, gg)
            total += oracle.macs(1, a, b, 1, 1, hw_out, hw_out, 1)

    total += oracle.macs(1, 3, 16, 3, 3, 32, 32, 1)
    cin, hw = 16, 32
    for width, stride in ((32, 1), (64, 2), (128, 2)):
        hw_out = hw // stride
        for b in range(6):
            a = cin if b == 0 else width
            conv3(a, width, hw_out)
            conv3(width, width, hw_out)
            if b == 0:
                total += oracle.macs(1, a, width, 1, 1, hw_out, hw_out, 1)
        cin, hw = width, hw_out
    return total + 128 * 10


def test_p11_table2_mac_differences():
    gold = _read_golden("table2_wrn40x2_macs.txt")
    keys = ["S", "G2", "G4", "G8", "G16", "GN"]
    ours = [_wrn40x2_macs(g) / 1e6 for g in (None, 2, 4, 8, 16, "N")]
    printed = [gold[k][0] for k in keys]
    for i in range(len(keys) - 1):
        assert abs((ours[i] - ours[i + 1]) - (printed[i] - printed[i + 1])) < 0.0101
    offsets = [p - o for p, o in zip(printed, ours)]
    assert max(offsets) - min(offsets) < 0.0101      # one constant offset
    assert 0.6 < offsets[0] < 0.8


# --------------------------------------------------------------------------
# Chain helpers, pinned with numpy alone (no optional import decides whether
# these run).
# --------------------------------------------------------------------------
def test_relu_and_add():
    x = _rand((2, 3, 9, 8), 21)
    assert np.array_equal(oracle.relu(x), np.maximum(x, 0))
    assert np.array_equal(oracle.add(x, 2 * x), x + 2 * x)


@pytest.mark.parametrize("H,W,k,stride,pad", [(9, 8, 3, 2, 1), (7, 7, 3, 2, 1), (6, 5, 2, 2, 0),
                                              (5, 6, 3, 1, 1), (112, 112, 3, 2, 1)])
def test_maxpool_against_windows_of_a_padded_copy(H, W, k, stride, pad):
    # Independent construction: pad a copy with -inf, take every k x k window
    # with numpy's sliding-window view, subsample by the stride.  Catches a
    # wrong window origin, a zero (instead of ignored) border, a stride slip.
    N, C = (1, 2) if H > 50 else (2, 3)
    x = _rand((N, C, H, W), 24)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)), constant_values=-np.inf)
    win = np.lib.stride_tricks.sliding_window_view(xp, (k, k), axis=(2, 3))
    ref = win[:, :, ::stride, ::stride].max(axis=(4, 5))
    got = oracle.maxpool2d(x, k, stride, pad)
    assert got.shape == (N, C, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1)
    assert np.array_equal(got, ref)


def test_maxpool_closed_forms():
    # 1x1 windows: the identity.  A plane that increases along both axes: the
    # maximum of a window is its last in-image corner, also at the borders.
    x = _rand((1, 2, 5, 4), 25)
    assert np.array_equal(oracle.maxpool2d(x, 1, 1, 0), x)
    H = W = 8
    ramp = (np.arange(H)[:, None] * 10.0 + np.arange(W)[None, :]).reshape(1, 1, H, W)
    got = oracle.maxpool2d(-ramp, 3, 2, 1)      # all negative: a zero border would win
    for oh in range(4):
        for ow in range(4):
            h0, w0 = max(2 * oh - 1, 0), max(2 * ow - 1, 0)
            assert got[0, 0, oh, ow] == -(h0 * 10.0 + w0)
    got = oracle.maxpool2d(ramp, 3, 2, 1)
    for oh in range(4):
        for ow in range(4):
            h1, w1 = min(2 * oh + 1, H - 1), min(2 * ow + 1, W - 1)
            assert got[0, 0, oh, ow] == h1 * 10.0 + w1


@pytest.mark.parametrize("N,Cin,Cout,H,W,g,K,stride,pad", [
    (2, 8, 12, 7, 6, 4, 3, 1, 1),
    (1, 6, 6, 9, 9, 6, 3, 2, 1),
    (2, 4, 8, 5, 5, 1, 1, 2, 0),
    (1, 6, 4, 12, 11, 2, 7, 2, 3),
])
def test_channel_subset_is_a_slice_of_the_full_result(N, Cin, Cout, H, W, g, K, stride, pad):
    # The sampled-channel routine (used at full batch sizes) must give exactly
    # the planes the pinned full routine gives: same sum, same order.  Catches
    # a wrong group for a selected filter, a selection / position mix-up,
    # a border rule that differs from the full routine's.
    x = _rand((N, Cin, H, W), 26)
    w = _rand((Cout, Cin // g, K, K), 27)
    full = oracle.conv2d_grouped(x, w, stride, pad, g)
    for sel in ([Cout - 1, 0, Cout // 2], list(range(Cout)), [1, 1], [Cout // g - 1]):
        sub = oracle.conv2d_grouped_channels(x, w, sel, stride, pad, g, threads=3)
        assert np.array_equal(sub, full[:, sel])
    with pytest.raises(ValueError):
        oracle.conv2d_grouped_channels(x, w, [Cout], stride, pad, g)


# --------------------------------------------------------------------------
# The chain executor against a chain worked out by hand (tests/golden):
# residual added before the ReLU, buffer routing, overwriting a buffer, the
# stand-alone add / ReLU / max-pool steps.
# --------------------------------------------------------------------------
def _hand_chain():
    from paper_2006_09791_amd.workloads import Layer
    L = Layer
    return [
        L("conv", 0, -1, 1, 1, 2, 2, 2, 2, 1, 1, 1, 0, 2, True, 0),
        L("conv", 1, 0, 2, 1, 2, 2, 2, 2, 1, 1, 1, 0, 1, True, 1),
        L("maxpool", 2, -1, 3, 1, 2, 2, 2, 2, 3, 3, 2, 1, 1, False, -1),
        L("add", 1, 2, 4, 1, 2, 2, 2, 2, 1, 1, 1, 0, 1, False, -1),
        L("relu", 0, -1, 5, 1, 2, 2, 2, 2, 1, 1, 1, 0, 1, False, -1),
        L("conv", 5, -1, 1, 1, 2, 2, 2, 2, 3, 3, 1, 1, 2, False, 2),
    ]


def test_run_chain_hand_example():
    gold = _read_golden("chain_hand_example.txt")
    x0 = np.array(gold["x0"]).reshape(1, 2, 2, 2)
    weights = [np.array(gold["w1"]).reshape(2, 1, 1, 1), np.array(gold["w2"]).reshape(2, 2, 1, 1),
               np.array(gold["w6"]).reshape(2, 1, 3, 3)]
    layers = _hand_chain()
    # after the first step buffer 1 holds step 1's result ...
    first = oracle.run_chain(layers[:1], 6, x0, weights)
    assert first[1].ravel().tolist() == gold["buf1_after_step1"]
    assert all(first[i] is None for i in (2, 3, 4, 5))
    # ... and at the end it holds step 6's
    bufs = oracle.run_chain(layers, 6, x0, weights, threads=2)
    assert bufs[0].ravel().tolist() == gold["x0"]
    for i in (1, 2, 3, 4, 5):
        assert bufs[i].ravel().tolist() == gold[f"buf{i}"], i
    assert bufs[3].shape == (1, 2, 1, 1) and bufs[2].shape == (1, 2, 2, 2)


def test_run_chain_add_with_relu_and_unknown_op():
    from paper_2006_09791_amd.workloads import Layer
    x0 = np.array([1.0, -5.0, 2.0, -1.0]).reshape(1, 1, 2, 2)
    w = [np.array([-1.0]).reshape(1, 1, 1, 1)]
    layers = [Layer("conv", 0, -1, 1, 1, 1, 2, 2, 1, 1, 1, 1, 0, 1, False, 0),     # -x
              Layer("add", 0, 1, 2, 1, 1, 2, 2, 1, 1, 1, 1, 0, 1, True, -1),       # relu(x - x) = 0
              Layer("add", 0, 0, 3, 1, 1, 2, 2, 1, 1, 1, 1, 0, 1, True, -1)]       # relu(2x)
    bufs = oracle.run_chain(layers, 4, x0, w)
    assert bufs[1].ravel().tolist() == [-1.0, 5.0, -2.0, 1.0]
    assert bufs[2].ravel().tolist() == [0.0] * 4
    assert bufs[3].ravel().tolist() == [2.0, 0.0, 4.0, 0.0]
    with pytest.raises(ValueError):
        oracle.run_chain([Layer("pool", 0, -1, 1, 1, 1, 2, 2, 1, 1, 1, 1, 0, 1, False, -1)], 2, x0, w)


def test_bad_arguments_rejected():
    x = _rand((1, 6, 4, 4), 22)
    w = _rand((4, 3, 3, 3), 23)
    with pytest.raises(ValueError):
        oracle.conv2d_grouped(x, w, 1, 1, 4)       # 6 % 4 != 0
    with pytest.raises(ValueError):
        oracle.conv2d_grouped(x, _rand((4, 3, 5, 5), 1), 1, 0, 2)   # kernel > input
