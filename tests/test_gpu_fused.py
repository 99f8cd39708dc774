"""Depth-fused runs of grouped 3x3 layers (one kernel per run, activations kept
on chip) against the oracle and against the step-by-step execution."""
import numpy as np
import pytest

from helpers import TOL_F32, gpu_chain, oracle_chain, rel_err, side_stream
from paper_2006_09791_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(ch, x0, weights, fusion):
    """Runs the chain untimed; returns (all buffers as numpy, kernel name of the last step)."""
    import torch
    from paper_2006_09791_amd import binding as b
    lc, bufs = gpu_chain(ch, x0, weights)
    for t in bufs[1:]:
        t.zero_()
    torch.cuda.synchronize()
    b.gspc_set_chain_fusion(fusion)
    try:
        b.gspc_run_layer_chain(lc)
        torch.cuda.synchronize()
        name = b.gspc_last_kernel()
    finally:
        b.gspc_set_chain_fusion(1)
    return [t.cpu().numpy().copy() for t in bufs], name


def _out(ch, bufs):
    n_out = int(np.prod(ch.out_shape))
    return bufs[ch.out_buf][:n_out].reshape(ch.out_shape)


@pytest.mark.parametrize("N,g", [(64, 4), (4, 8), (2, 16), (16, 16), (1, 16)])
def test_wrn_fused_vs_oracle(N, g):
    ch = wl.wrn_chain(N, g)
    weights = ch.make_weights(5)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(5, N, g))
    ref = oracle_chain(ch, x0, weights)[ch.out_buf]
    fused, name = _run(ch, x0, weights, 1)
    assert "conv_fused_run" in name, name
    assert rel_err(_out(ch, fused), ref) < TOL_F32
    plain, name2 = _run(ch, x0, weights, 0)
    assert "conv_fused_run" not in name2
    # every activation buffer holds what the step-by-step execution leaves in it
    for k, (a, c) in enumerate(zip(fused, plain)):
        n = ch.buf_elems[k]
        assert rel_err(a[:n], c[:n]) < TOL_F32, f"buffer {k}"


def test_odd_width_and_buffer_reuse():
    """Width not a multiple of 4 (scalar global accesses, one-pixel strips) and a
    buffer that is overwritten inside the run."""
    N, C, g, hw = 6, 24, 6, 7
    ch = wl.Chain("odd", (N, C, hw, hw))
    ch.conv(0, 1, N, C, hw, hw, C, 3, 1, 1, g, relu=True)
    ch.conv(1, 2, N, C, hw, hw, C, 3, 1, 1, g, relu=True, residual=0)
    ch.conv(2, 3, N, C, hw, hw, C, 3, 1, 1, g, relu=False, residual=1)
    ch.conv(3, 1, N, C, hw, hw, C, 3, 1, 1, g, relu=True)
    weights = ch.make_weights(7)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(7, 1, 1))
    ref = oracle_chain(ch, x0, weights)
    fused, name = _run(ch, x0, weights, 1)
    assert "conv_fused_run" in name, name
    for k in (1, 2, 3):
        n = ch.buf_elems[k]
        assert rel_err(fused[k][:n], np.asarray(ref[k]).reshape(-1)[:n]) < TOL_F32, f"buffer {k}"


def test_replays_are_stable():
    """The fused run is part of the recorded graph: replays with eager work in
    between reproduce the eager result bit for bit."""
    import torch
    from paper_2006_09791_amd import binding as b
    N, g = 8, 8
    ch = wl.wrn_chain(N, g)
    weights = ch.make_weights(8)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(8, N, g))
    eager, _ = _run(ch, x0, weights, 1)
    lc, bufs = gpu_chain(ch, x0, weights)
    n_out = int(np.prod(ch.out_shape))
    with torch.cuda.stream(side_stream()):
        b.gspc_set_stream()
        for rep in range(4):
            bufs[ch.out_buf].zero_()
            b.gspc_run_layer_chain(lc)
            torch.cuda.synchronize()
            again = bufs[ch.out_buf][:n_out].cpu().numpy()
            assert np.array_equal(eager[ch.out_buf][:n_out], again), f"replay {rep}"
            (torch.randn(1 << 16, device="cuda") * 2).sum().item()
    b.gspc_set_stream()


# ---- depthwise 3x3 + pointwise 1x1 as one kernel ------------------------------------

def _dwpw_chain(N, C, C2, hw, stride, relu_dw=True, relu_pw=True, residual=False, reuse=False):
    """dw 3x3 (buffer 0 -> 1), pw 1x1 (1 -> 2); optionally a residual operand for the
    pointwise step (buffer 3, filled by an extra step) and a last step that overwrites the
    depthwise buffer, so that its contents after the pair cannot be observed."""
    ch = wl.Chain(f"dwpw{N}_{C}_{C2}_{hw}_{stride}", (N, C, hw, hw))
    ho = wl.out_size(hw, 3, stride, 1)
    res = -1
    if residual:
        ch.conv(0, 3, N, C, hw, hw, C2, 1, stride, 0, 1)          # any tensor of the output's shape
        res = 3
    ch.conv(0, 1, N, C, hw, hw, C, 3, stride, 1, C, relu=relu_dw)
    ch.conv(1, 2, N, C, ho, ho, C2, 1, 1, 0, 1, relu=relu_pw, residual=res)
    if reuse:
        ch.conv(2, 1, N, C2, ho, ho, C, 1, 1, 0, 1)
    return ch


# The pair is only fused when the launch has at least one block per compute unit, hence the
# batch sizes (the planes are small, the oracle stays within a second or two).
@pytest.mark.parametrize("N,C,C2,hw,stride,kw", [
    (3, 32, 64, 112, 1, {}),                          # first MobileNet block, one-row bands
    (10, 64, 128, 56, 2, {}),                         # stride 2, four filter tiles recompute the tile
    (2098, 32, 64, 8, 1, dict(relu_dw=False)),        # four images per tile, ragged last tile, many tiles per block
    (24, 128, 128, 28, 1, dict(relu_pw=False, residual=True)),
    (300, 64, 64, 16, 2, dict(reuse=True)),           # depthwise buffer overwritten later: not stored
    (600, 16, 32, 8, 1, dict(reuse=True, residual=True)),
    (2, 32, 64, 16, 1, {}),                           # too small a launch: stays two kernels
], ids=lambda v: str(v) if not isinstance(v, dict) else "-".join(v) or "plain")
def test_depthwise_pointwise_fused(N, C, C2, hw, stride, kw):
    ch = _dwpw_chain(N, C, C2, hw, stride, **kw)
    weights = ch.make_weights(6)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(6, C, hw))
    ref = oracle_chain(ch, x0, weights)
    fused, name = _run(ch, x0, weights, 1)
    plain, name2 = _run(ch, x0, weights, 0)
    assert "conv_dwpw" not in name2
    if not kw.get("reuse"):
        assert ("conv_dwpw" in name) == (N > 2), name
    # every buffer ends up as the step-by-step execution (and the oracle) leaves it
    for k, (a, c) in enumerate(zip(fused, plain)):
        n = ch.buf_elems[k]
        assert rel_err(a[:n], c[:n]) < TOL_F32, f"buffer {k}"
        assert rel_err(a[:n], np.asarray(ref[k]).reshape(-1)[:n]) < TOL_F32, f"buffer {k} vs oracle"



# ---- grouped 3x3 + pointwise 1x1 as one kernel (the block of the paper's networks) ------------

def _gpw_chain(N, C, C2, hw, g, stride, relu_a=False, relu_b=True, residual=False, reuse=False):
    """grouped 3x3 C -> C (buffer 0 -> 1), pointwise 1x1 C -> C2 (1 -> 2); optionally a residual
    operand for the pointwise step (buffer 3) and a last step that overwrites the grouped
    layer's buffer, so that its contents after the pair cannot be observed."""
    ch = wl.Chain(f"gpw{N}_{C}_{C2}_{hw}_{g}_{stride}", (N, C, hw, hw))
    ho = wl.out_size(hw, 3, stride, 1)
    res = -1
    if residual:
        ch.conv(0, 3, N, C, hw, hw, C2, 1, stride, 0, 1)
        res = 3
    ch.conv(0, 1, N, C, hw, hw, C, 3, stride, 1, g, relu=relu_a)
    ch.conv(1, 2, N, C, ho, ho, C2, 1, 1, 0, 1, relu=relu_b, residual=res)
    if reuse:
        ch.conv(2, 1, N, C2, ho, ho, C, 1, 1, 0, 1)
    return ch


# The pair is fused when the launch has at least one wave (16 pixels) per SIMD, hence the batches.
@pytest.mark.parametrize("N,C,C2,hw,g,stride,kw", [
    (16, 32, 32, 32, 2, 1, {}),                                   # WRN-style first stage, two-row tiles
    (70, 32, 64, 32, 4, 2, dict(relu_a=True)),                    # stage entry: stride 2, 8 filters per group (pairs merged)
    (70, 64, 64, 16, 16, 1, dict(residual=True)),                 # 4 filters per group: four groups merged; residual
    (260, 128, 128, 8, 2, 1, dict(reuse=True)),                   # whole 8x8 images, 64 filters per group; result not kept
    (6, 64, 64, 56, 8, 1, dict(relu_a=True, relu_b=False)),       # ResNet-34-shaped first stage, one-row tiles with idle lanes
    (23, 128, 128, 28, 32, 1, dict(residual=True, reuse=True)),   # ragged last tile
    (90, 32, 64, 32, 1, 2, {}),                                   # g = 1 followed by a pointwise layer
    (300, 32, 32, 7, 2, 1, {}),                                   # width not a multiple of 4: stays two kernels
    (2, 32, 32, 32, 2, 1, {}),                                    # too small a launch: stays two kernels
], ids=lambda v: str(v) if not isinstance(v, dict) else "-".join(v) or "plain")
def test_grouped_pointwise_fused(N, C, C2, hw, g, stride, kw, monkeypatch):
    monkeypatch.setenv("GSPC_GPW", "1")     # the pair kernel is opt-in (it does not beat the two kernels yet)
    ch = _gpw_chain(N, C, C2, hw, g, stride, **kw)
    weights = ch.make_weights(12)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(12, C, hw))
    ref = oracle_chain(ch, x0, weights)
    fused, name = _run(ch, x0, weights, 1)
    plain, name2 = _run(ch, x0, weights, 0)
    assert "conv_gpw" not in name2
    if not kw.get("reuse"):
        assert ("conv_gpw" in name) == (N > 2 and hw % 4 == 0), name
    for k, (a, c) in enumerate(zip(fused, plain)):
        n = ch.buf_elems[k]
        assert rel_err(a[:n], c[:n]) < TOL_F32, f"buffer {k}"
        assert rel_err(a[:n], np.asarray(ref[k]).reshape(-1)[:n]) < TOL_F32, f"buffer {k} vs oracle"


def test_pointwise_form_wrn_chain_uses_the_fused_pairs(monkeypatch):
    """The paper-form WRN stack (every 3x3 a grouped 3x3 a -> a plus a pointwise a -> b) at a batch
    that fills the chip: pairs run fused, the result matches the oracle, replays are stable."""
    monkeypatch.setenv("GSPC_GPW", "1")
    import torch
    from paper_2006_09791_amd import binding as b
    N, g = 16, 4
    ch = wl.wrn_chain(N, g, pointwise=True)
    weights = ch.make_weights(13)
    x0 = wl.make_input(ch.input_shape, wl.make_seed(13, N, g))
    ref = oracle_chain(ch, x0, weights)[ch.out_buf]
    lc, bufs = gpu_chain(ch, x0, weights)
    n_out = int(np.prod(ch.out_shape))
    names = set()
    b.gspc_set_stream()
    b.gspc_run_layer_chain(lc)
    torch.cuda.synchronize()
    eager = bufs[ch.out_buf][:n_out].cpu().numpy().copy()
    assert rel_err(eager.reshape(ch.out_shape), ref) < TOL_F32
    with torch.cuda.stream(side_stream()):
        b.gspc_set_stream()
        for rep in range(3):
            bufs[ch.out_buf].zero_()
            b.gspc_run_layer_chain(lc)
            torch.cuda.synchronize()
            assert np.array_equal(eager, bufs[ch.out_buf][:n_out].cpu().numpy()), f"replay {rep}"
    b.gspc_set_stream()
    # a single pair of the first stage reports the fused kernel
    pair = wl.Chain("pair", (N, 32, 32, 32))
    pair.conv(0, 1, N, 32, 32, 32, 32, 3, 1, 1, g)
    pair.conv(1, 2, N, 32, 32, 32, 32, 1, 1, 0, 1, relu=True)
    lc2, _ = gpu_chain(pair, wl.make_input(pair.input_shape, 3), pair.make_weights(14))
    b.gspc_run_layer_chain(lc2)
    torch.cuda.synchronize()
    assert b.gspc_last_kernel().startswith("conv_gpw<"), b.gspc_last_kernel()
