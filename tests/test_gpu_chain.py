"""GPU parity of whole layer chains (gspc_run_layer_chain) against the oracle."""
import numpy as np
import pytest

from helpers import TOL_F32, gpu_chain, oracle_chain, rel_err, side_stream
from paper_2006_09791_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(chain, config_id, seed):
    import torch
    from paper_2006_09791_amd import binding as b
    x0 = wl.make_input(chain.input_shape, seed)
    weights = chain.make_weights(config_id)
    lc, bufs = gpu_chain(chain, x0, weights)
    ms = b.gspc_run_layer_chain(lc, per_layer_ms=True)
    assert len(ms) == len(chain.layers) and all(m >= 0 for m in ms)
    n_out = int(np.prod(chain.out_shape))
    timed = bufs[chain.out_buf][:n_out].cpu().numpy().reshape(chain.out_shape)
    # The untimed form may evaluate runs of grouped layers in one kernel, which
    # changes the summation order: same values within the tolerance, and the
    # reference for the bit-exactness of the replays below.
    bufs[chain.out_buf].zero_()
    b.gspc_run_layer_chain(lc)
    torch.cuda.synchronize()
    got = bufs[chain.out_buf][:n_out].cpu().numpy().reshape(chain.out_shape)
    assert rel_err(timed, got) < TOL_F32
    # The asynchronous form on a side stream is recorded into a HIP graph on
    # its first call and replayed afterwards: every replay must give the same
    # bits as the eager run, with unrelated eager work in between.
    with torch.cuda.stream(side_stream()):
        b.gspc_set_stream()
        for rep in range(4):
            bufs[chain.out_buf].zero_()
            b.gspc_run_layer_chain(lc)
            torch.cuda.synchronize()
            again = bufs[chain.out_buf][:n_out].cpu().numpy().reshape(chain.out_shape)
            assert np.array_equal(got, again), f"graph replay {rep} differs from the eager run"
            scratch = torch.randn(1 << 16, device="cuda")
            (scratch * 2).sum().item()
    b.gspc_set_stream()
    ref = oracle_chain(chain, x0, weights)[chain.out_buf]
    return got, ref


@pytest.mark.parametrize("g", [1, 2, 4, 8, 16])
def test_wrn_chain_n1(g):
    chain = wl.wrn_chain(1, g)
    got, ref = _run(chain, 2, wl.make_seed(2, 999, g))
    assert np.abs(ref).max() > 0
    assert rel_err(got, ref) < TOL_F32


def test_wrn_chain_n3_g4():
    chain = wl.wrn_chain(3, 4)
    got, ref = _run(chain, 2, 77)
    assert rel_err(got, ref) < TOL_F32


@pytest.mark.parametrize("g", [2, 4, 8, 16, 32])
def test_resnet34_chain_n1(g):
    chain = wl.resnet34_chain(1, g)
    got, ref = _run(chain, 3, wl.make_seed(3, 999, g))
    assert np.abs(ref).max() > 0
    assert rel_err(got, ref) < TOL_F32


@pytest.mark.parametrize("C,hw,stride", [(32, 112, 1), (64, 112, 2), (256, 28, 1), (1024, 7, 2)])
def test_depthwise_pointwise_chain(C, hw, stride):
    chain = wl.mobilenet_dw_chain(1, C, hw, stride)
    got, ref = _run(chain, 4, wl.make_seed(4, C, stride))
    assert rel_err(got, ref) < TOL_F32


def test_chain_validation_precedes_launch():
    import torch
    from paper_2006_09791_amd import binding as b
    chain = wl.mobilenet_dw_chain(1, 8, 10, 1)
    x0 = wl.make_input(chain.input_shape, 1)
    weights = chain.make_weights(4)
    lc, bufs = gpu_chain(chain, x0, weights)
    bufs[1].fill_(123.0)
    lc.bytes[2] = 16       # last layer's output buffer too small
    torch.cuda.synchronize()
    with pytest.raises(b.GspcError) as e:
        b.gspc_run_layer_chain(lc)
    assert e.value.code == -6
    torch.cuda.synchronize()
    assert float(bufs[1].min()) == 123.0    # first layer was not launched either


def test_graph_mode_off_matches():
    import torch
    from paper_2006_09791_amd import binding as b
    chain = wl.wrn_chain(2, 8)
    x0 = wl.make_input(chain.input_shape, 5)
    weights = chain.make_weights(2)
    lc, bufs = gpu_chain(chain, x0, weights)
    n_out = int(np.prod(chain.out_shape))
    outs = []
    with torch.cuda.stream(side_stream()):
        b.gspc_set_stream()
        for on in (1, 0, 1):
            b.gspc_set_graph_mode(on)
            bufs[chain.out_buf].zero_()
            b.gspc_run_layer_chain(lc)
            b.gspc_run_layer_chain(lc)
            torch.cuda.synchronize()
            outs.append(bufs[chain.out_buf][:n_out].cpu().numpy())
    b.gspc_set_graph_mode(1)
    b.gspc_set_stream()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[1], outs[2])


@pytest.mark.parametrize("s", [
    wl.ConvShape(300, 64, 14, 14, 64, 3, 3, 1, 1, 2),   # more tiles than resident blocks, 16-byte stores
    wl.ConvShape(40, 64, 7, 7, 64, 3, 3, 1, 1, 2),      # odd width: several images per tile, 4-byte stores
    wl.ConvShape(3, 64, 56, 56, 64, 3, 3, 1, 1, 2),     # 16-byte loads, row bands with a ragged tail
    wl.ConvShape(2, 64, 28, 28, 128, 3, 3, 2, 1, 2),    # stride 2
    wl.ConvShape(5, 256, 12, 12, 256, 3, 3, 1, 1, 2),   # four chunks of channels per group
], ids=lambda s: "x".join(map(str, s)))
def test_bf16_conv_with_residual_and_relu(s):
    """A bf16 convolution step with the residual operand and the ReLU of a
    basic block (Section IV-A networks), against the oracle on the same
    rounded operands."""
    import torch
    import oracle
    from paper_2006_09791_amd import binding as b
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    x = wl.make_input((s.N, s.Cin, s.H, s.W), 41)
    w = wl.make_weight(s.Cout, s.Cin // s.groups, 3, 3, 42)
    ho, wo = b.gspc_output_dims(s.H, s.W, 3, 3, s.stride, s.pad)
    res = wl.make_input((s.N, s.Cout, ho, wo), 43)
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), s.groups, b.GSPC_BF16)
    xb = b.gspc_pack_input_bf16(torch.from_numpy(x).to(dev))
    rd = torch.from_numpy(res).to(dev).reshape(-1)
    yd = torch.full((res.size,), float("nan"), dtype=torch.float32, device=dev)
    layer = wl.Layer("conv", 0, 1, 2, s.N, s.Cin, s.H, s.W, s.Cout, 3, 3, s.stride, s.pad, s.groups, True, 0)
    lc = b.LayerChain([layer], [pw], [xb.reshape(-1), rd, yd])
    b.gspc_run_layer_chain(lc)
    torch.cuda.synchronize()
    assert "mfma16b" in b.gspc_last_kernel()
    got = yd.cpu().numpy().reshape(res.shape)
    _, xr = wl.round_to_bf16(x)
    _, wr = wl.round_to_bf16(w)
    ref = oracle.relu(oracle.add(oracle.conv2d_grouped(xr, wr, s.stride, s.pad, s.groups, threads=8), res))
    assert rel_err(got, ref) < 1e-4, b.gspc_last_kernel()


@pytest.mark.parametrize("N,g", [(1, None), (1, 8), (8, None)], ids=["n1-depthwise", "n1-g8", "n8-depthwise"])
def test_mobilenet_chain(N, g):
    """MobileNet-shaped stack in the paper's block form (grouped 3x3 a -> a, pointwise
    a -> b), depthwise extreme and a G(8) variant; at N = 8 the first blocks run as fused
    depthwise + pointwise kernels."""
    chain = wl.mobilenet_chain(N, g)
    got, ref = _run(chain, 5, wl.make_seed(5, N, 0 if g is None else g))
    assert np.abs(ref).max() > 0
    assert rel_err(got, ref) < TOL_F32


@pytest.mark.parametrize("N,g", [(1, None), (1, 8), (3, None), (2, 16)], ids=["n1-depthwise", "n1-g8", "n3-depthwise", "n2-g16"])
def test_mobilenetv2_chain(N, g):
    """MobileNetV2-shaped stack (Section IV-A): inverted-residual blocks with the 3x3
    convolution depthwise (the original, G(N)) or with g groups; 52 convolutions with
    residual additions on the linear projections."""
    chain = wl.mobilenetv2_chain(N, g, hw=224 if N == 1 else 96)
    got, ref = _run(chain, 6, wl.make_seed(6, N, 0 if g is None else g))
    assert np.abs(ref).max() > 0
    assert rel_err(got, ref) < TOL_F32


@pytest.mark.parametrize("net,N,g", [("wrn", 1, 2), ("wrn", 2, 4), ("wrn", 1, 16), ("resnet34", 1, 8)])
def test_pointwise_form_chain(net, N, g):
    """The form of the paper's trained networks (Section IV-A): every 3x3 convolution of
    a basic block replaced by a grouped 3x3 a -> a followed by a pointwise a -> b."""
    chain = wl.wrn_chain(N, g, pointwise=True) if net == "wrn" else wl.resnet34_chain(N, g, pointwise=True)
    got, ref = _run(chain, 7, wl.make_seed(7, N, g))
    assert np.abs(ref).max() > 0
    assert rel_err(got, ref) < TOL_F32


@pytest.mark.parametrize("s", [
    wl.ConvShape(3, 96, 7, 7, 40, 1, 1, 1, 0, 1),      # 40 filters, 49-element planes: 4-byte stores
    wl.ConvShape(2, 144, 12, 12, 144, 3, 3, 1, 1, 8),  # 18 filters per group: 16-byte stores
    wl.ConvShape(2, 120, 10, 10, 120, 3, 3, 2, 1, 2),  # 60 filters per group, stride 2, 25-element planes
], ids=lambda s: "x".join(map(str, s)))
def test_padded_filter_tile_with_residual_and_relu(s):
    """Residual operand and ReLU on a layer whose last filter tile is partly padding: the
    padding filters must neither read nor write (the buffers end right after the tensor)."""
    import torch
    import oracle
    from paper_2006_09791_amd import binding as b
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    x = wl.make_input((s.N, s.Cin, s.H, s.W), 51)
    w = wl.make_weight(s.Cout, s.Cin // s.groups, s.KH, s.KW, 52)
    ho, wo = b.gspc_output_dims(s.H, s.W, s.KH, s.KW, s.stride, s.pad)
    res = wl.make_input((s.N, s.Cout, ho, wo), 53)
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), s.groups)
    xd = torch.from_numpy(x).to(dev).reshape(-1)
    rd = torch.from_numpy(res).to(dev).reshape(-1)
    # the output sits in the middle of a NaN-filled buffer: nothing around it may change
    guard = 4096
    yd = torch.full((res.size + 2 * guard,), float("nan"), dtype=torch.float32, device=dev)
    layer = wl.Layer("conv", 0, 1, 2, s.N, s.Cin, s.H, s.W, s.Cout, s.KH, s.KW, s.stride, s.pad, s.groups, True, 0)
    lc = b.LayerChain([layer], [pw], [xd, rd, yd[guard:guard + res.size]])
    b.gspc_run_layer_chain(lc)
    torch.cuda.synchronize()
    assert b.gspc_last_kernel().startswith("conv_mfma16<"), b.gspc_last_kernel()
    out = yd.cpu().numpy()
    assert np.isnan(out[:guard]).all() and np.isnan(out[guard + res.size:]).all()
    got = out[guard:guard + res.size].reshape(res.shape)
    ref = oracle.relu(oracle.add(oracle.conv2d_grouped(x, w, s.stride, s.pad, s.groups, threads=8), res))
    assert rel_err(got, ref) < TOL_F32
