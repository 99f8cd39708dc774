"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times (same dispatcher, same tiles): the oracle recomputes sampled output
channels of sampled images, whole planes at a time."""
import numpy as np
import pytest

import oracle
from helpers import TOL_BF16, TOL_F32, rel_err
from paper_2006_09791_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _sampled_check(s, seed, dtype_bf16, n_img, n_oc, tol_same, tol_unrounded=None):
    import torch
    from paper_2006_09791_amd import binding as b
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    b.gspc_force_path(b.PATH_AUTO)
    x = wl.make_input((s.N, s.Cin, s.H, s.W), seed)
    w = wl.make_weight(s.Cout, s.Cin // s.groups, s.KH, s.KW, seed)
    dt = b.GSPC_BF16 if dtype_bf16 else b.GSPC_F32
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), s.groups, dt)
    xd = torch.from_numpy(x).to(dev)
    if dtype_bf16:
        xd = b.gspc_pack_input_bf16(xd)
    y = b.gspc_conv2d_grouped(xd, pw, s.N, s.Cin, s.H, s.W, s.Cout, s.KH, s.KW, s.stride, s.pad,
                              s.groups)
    name = b.gspc_last_kernel()
    torch.cuda.synchronize()
    rng = np.random.default_rng(seed + 1)
    imgs = np.unique(np.concatenate([[0, s.N - 1], rng.choice(s.N, size=min(n_img, s.N), replace=False)]))
    # sampled filters: first, last, and random ones (hits several groups and tile positions)
    ocs = np.unique(np.concatenate([[0, s.Cout - 1], rng.choice(s.Cout, size=n_oc, replace=False)]))
    got = y[torch.from_numpy(imgs).to(dev)][:, torch.from_numpy(ocs).to(dev)].cpu().numpy()
    assert np.isfinite(got).all()
    xs, ws = x[imgs], w
    if dtype_bf16:
        _, xs_r = wl.round_to_bf16(xs)
        _, ws_r = wl.round_to_bf16(ws)
        ref = oracle.conv2d_grouped_channels(xs_r, ws_r, ocs, s.stride, s.pad, s.groups, threads=16)
        assert rel_err(got, ref) < tol_same, (name, s)
        if tol_unrounded:
            ref2 = oracle.conv2d_grouped_channels(xs, ws, ocs, s.stride, s.pad, s.groups, threads=16)
            assert rel_err(got, ref2) < tol_unrounded, (name, s)
    else:
        ref = oracle.conv2d_grouped_channels(xs, ws, ocs, s.stride, s.pad, s.groups, threads=16)
        assert rel_err(got, ref) < tol_same, (name, s)
    return name


@pytest.mark.parametrize("g", [1, 2, 4, 8, 16])
def test_wrn_layers_batch64_fp32(g):
    for i, s in enumerate(wl.wrn_grouped_shapes(64, g)):
        _sampled_check(s, wl.make_seed(2, 100 + i, g), False, n_img=3, n_oc=4, tol_same=TOL_F32)


@pytest.mark.parametrize("g", [1, 2])
def test_wrn_layers_batch256_fp32(g):
    """More blocks than the chip holds at once: the resident-filter kernel walks
    over several pixel tiles per block (first, last and random images sampled)."""
    from paper_2006_09791_amd import binding as b
    names = []
    b.gspc_set_winograd(0)   # the direct kernels; the automatic choice at this size is the next test
    try:
        for i, s in enumerate(wl.wrn_grouped_shapes(256, g)):
            names.append(_sampled_check(s, wl.make_seed(2, 300 + i, g), False, n_img=3, n_oc=4, tol_same=TOL_F32))
            # stride-1 layers: the resident-filter kernel; stride-2 layers at this batch: the same from 64
            # channels per group on, else the plain one
            want_w = s.stride == 1 or s.Cin // g >= 64
            assert ("conv_mfma16w" if want_w else "conv_mfma16<") in names[-1], names[-1]
    finally:
        b.gspc_set_winograd(None)
    assert any(",true," in n for n in names), names   # the multi-tile instantiation ran


@pytest.mark.parametrize("g", [1, 2, 4])
def test_wrn_layers_batch256_automatic_choice(g):
    """At this size the stride-1 layers with at least 8 channels and 16 filters per group go
    through Winograd F(2x2, 3x3) by default (sampled images and filters against the oracle)."""
    for i, s in enumerate(wl.wrn_grouped_shapes(256, g)):
        name = _sampled_check(s, wl.make_seed(2, 400 + i, g), False, n_img=3, n_oc=4, tol_same=TOL_F32)
        eligible = s.stride == 1 and (s.Cin // g) >= 8 and (s.Cin // g) % 4 == 0 and (s.Cout // g) % 16 == 0
        assert name.startswith("conv_wino<") == eligible, (s, name)


def test_winograd_forms_by_launch_size():
    """One product tile per wave: V is transformed in registers (last template argument true) up to
    sixteen blocks per compute unit, through the LDS buffer beyond that; both against the oracle on
    sampled images and filters."""
    S = wl.ConvShape
    small = _sampled_check(S(64, 32, 32, 32, 32, 3, 3, 1, 1, 1), wl.make_seed(2, 500, 1), False, n_img=3, n_oc=4,
                           tol_same=TOL_F32)
    assert small.startswith("conv_wino<1,1,") and small.endswith(",true>"), small
    large = _sampled_check(S(512, 32, 32, 32, 32, 3, 3, 1, 1, 1), wl.make_seed(2, 501, 1), False, n_img=3, n_oc=4,
                           tol_same=TOL_F32)
    assert large.startswith("conv_wino<1,1,") and large.endswith(",false>"), large


def test_residual_chain_batch256_fp32():
    """Residual and ReLU epilogue of the multi-tile form, whole tensors."""
    import torch
    from helpers import gpu_chain, oracle_chain
    from paper_2006_09791_amd import binding as b
    N, C, hw = 256, 64, 16
    ch = wl.Chain("big", (N, C, hw, hw))
    ch.conv(0, 1, N, C, hw, hw, C, 3, 1, 1, 1, relu=True)
    ch.conv(1, 2, N, C, hw, hw, C, 3, 1, 1, 1, relu=True, residual=0)
    x0 = wl.make_input(ch.input_shape, 41)
    weights = ch.make_weights(9)
    lc, bufs = gpu_chain(ch, x0, weights)
    b.gspc_set_winograd(0)
    try:
        b.gspc_run_layer_chain(lc)
        torch.cuda.synchronize()
    finally:
        b.gspc_set_winograd(None)
    assert "conv_mfma16w" in b.gspc_last_kernel() and ",true," in b.gspc_last_kernel()
    ref = oracle_chain(ch, x0, weights, threads=16)[2]
    got = bufs[2][:ref.size].cpu().numpy().reshape(ref.shape)
    assert rel_err(got, ref) < TOL_F32


def test_wrn_stem_and_shortcuts_batch64_fp32():
    S = wl.ConvShape
    for i, s in enumerate([S(64, 3, 32, 32, 32, 3, 3, 1, 1, 1), S(64, 32, 32, 32, 64, 1, 1, 2, 0, 1),
                           S(64, 64, 16, 16, 128, 1, 1, 2, 0, 1)]):
        _sampled_check(s, wl.make_seed(2, 200 + i, 1), False, n_img=3, n_oc=4, tol_same=TOL_F32)


@pytest.mark.parametrize("g", [2, 8, 32])
def test_resnet34_layers_batch256_bf16(g):
    for i, s in enumerate(wl.resnet34_grouped_shapes(256, g)):
        _sampled_check(s, wl.make_seed(5, i, g), True, n_img=2, n_oc=4, tol_same=1e-4,
                       tol_unrounded=TOL_BF16)


@pytest.mark.parametrize("idx,g", [(0, 2), (0, 8), (0, 32), (1, 32), (2, 8), (2, 32), (4, 32), (6, 32)])
def test_resnet34_layers_batch256_bf16_whole_images(idx, g):
    """Every output channel of a block of images at the batch-256 size (the other
    test samples a few filters): the wide-store epilogues are compared element by
    element over whole images, first and last of the batch included, and a second run
    must give the same bits over the whole tensor."""
    import torch
    from paper_2006_09791_amd import binding as b
    s = wl.resnet34_grouped_shapes(256, g)[idx]
    seed = wl.make_seed(5, 50 + idx, g)
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    b.gspc_force_path(b.PATH_AUTO)
    x = wl.make_input((s.N, s.Cin, s.H, s.W), seed)
    w = wl.make_weight(s.Cout, s.Cin // s.groups, s.KH, s.KW, seed)
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), s.groups, b.GSPC_BF16)
    xd = b.gspc_pack_input_bf16(torch.from_numpy(x).to(dev))
    ys = []
    for rep in range(2):
        y = torch.full((s.N, s.Cout) + tuple(b.gspc_output_dims(s.H, s.W, 3, 3, s.stride, 1)), float("nan"),
                       dtype=torch.float32, device=dev)
        b.gspc_conv2d_grouped(xd, pw, s.N, s.Cin, s.H, s.W, s.Cout, 3, 3, s.stride, 1, s.groups, y)
        torch.cuda.synchronize()
        ys.append(y)
    name = b.gspc_last_kernel()
    assert torch.equal(ys[0], ys[1]), name             # no NaN left, same bits
    imgs = [0, 1, 2, 3, 100, 101, 254, 255]
    got = ys[0][imgs].cpu().numpy()
    _, xr = wl.round_to_bf16(x[imgs])
    _, wr = wl.round_to_bf16(w)
    ref = oracle.conv2d_grouped(xr, wr, s.stride, s.pad, s.groups, threads=16)
    assert rel_err(got, ref) < 1e-4, (name, s)


def test_depthwise_batched_fp32():
    # batched re-run of the MobileNet-shaped depthwise layers (HBM-bound kernel at a size that fills the GPU)
    for i, (dw, _) in enumerate(wl.depthwise_pairs(32)):
        _sampled_check(dw, wl.make_seed(4, 300 + i, dw.groups), False, n_img=2, n_oc=6, tol_same=TOL_F32)
