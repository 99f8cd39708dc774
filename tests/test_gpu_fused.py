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
