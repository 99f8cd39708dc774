"""GPU parity: libgspc (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from helpers import TOL_BF16, TOL_F32, err_metrics, rel_err
from paper_2006_09791_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2006_09791_amd import binding as b
    assert torch.cuda.is_available()
    b.load()
    b.gspc_set_stream()
    b.gspc_force_path(b.PATH_AUTO)
    return torch, b


def run_conv(gpu, s, seed, path=None, dtype=None, poison=True):
    """Runs one layer on the GPU; returns (y_gpu float32 ndarray, x, w, kernel name)."""
    torch, b = gpu
    dev = torch.device("cuda:0")
    x = wl.make_input((s.N, s.Cin, s.H, s.W), seed)
    w = wl.make_weight(s.Cout, s.Cin // s.groups, s.KH, s.KW, seed)
    dt = dtype if dtype is not None else b.GSPC_F32
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), s.groups, dt)
    xd = torch.from_numpy(x).to(dev)
    if dt == b.GSPC_BF16:
        xd = b.gspc_pack_input_bf16(xd)
    ho, wo = b.gspc_output_dims(s.H, s.W, s.KH, s.KW, s.stride, s.pad)
    y = torch.full((s.N, s.Cout, ho, wo), float("nan"), dtype=torch.float32, device=dev)
    b.gspc_force_path(path if path is not None else b.PATH_AUTO)
    try:
        b.gspc_conv2d_grouped(xd, pw, s.N, s.Cin, s.H, s.W, s.Cout, s.KH, s.KW, s.stride, s.pad,
                              s.groups, y)
        name = b.gspc_last_kernel()
    finally:
        b.gspc_force_path(b.PATH_AUTO)
    torch.cuda.synchronize()
    return y.cpu().numpy(), x, w, name


def check(gpu, s, seed, path=None, tol=TOL_F32):
    y, x, w, name = run_conv(gpu, s, seed, path)
    ref, absum = oracle.conv2d_grouped(x, w, s.stride, s.pad, s.groups, return_abs=True, threads=8)
    assert not np.isnan(y).any(), f"{name}: output not fully written for {s}"
    m = err_metrics(y, ref, absum)
    print(f"{name}: floored {m['floored']:.2e} scaled {m['scaled']:.2e} |g-r|/sum|xw| {m['bound']:.2e} for {s}")
    # fp32 accumulation of K products: |g - r| <= about K * 2^-24 * sum|x*w| (Winograd's transforms a few times that)
    assert tol > TOL_F32 or m["bound"] < 1e-4, f"{name}: |g-r|/sum|xw| {m['bound']:.3e} for {s}"
    assert m["floored"] < tol, f"{name}: rel err {m['floored']:.3e} for {s}"
    assert m["scaled"] < tol, f"{name}: max|g-r|/max|r| {m['scaled']:.3e} for {s}"
    return name


def test_config1(gpu):
    name = check(gpu, wl.config1(), seed=0)
    print("config1 ran on", name)


S = wl.ConvShape
SWEEP = [
    # N Cin H W Cout KH KW stride pad groups
    S(2, 8, 9, 7, 8, 3, 3, 1, 1, 1),
    S(1, 6, 5, 4, 4, 3, 3, 2, 1, 2),       # KPG = 2: direct only
    S(3, 12, 11, 13, 24, 3, 3, 1, 1, 3),   # KPG = 8
    S(2, 16, 10, 10, 16, 3, 3, 2, 1, 4),   # KPG = 4
    S(1, 32, 17, 19, 32, 3, 3, 1, 1, 2),   # KPG = 16
    S(2, 32, 16, 16, 64, 3, 3, 2, 1, 2),   # KPG = 32, CPG = 16
    S(1, 64, 8, 8, 64, 3, 3, 1, 1, 1),     # KPG = 64
    S(3, 128, 8, 8, 128, 3, 3, 1, 1, 1),   # KPG = 128, odd batch vs images per block
    S(3, 32, 12, 20, 48, 3, 3, 1, 1, 1),   # resident-filter kernel: rows wider than a 16-pixel run, ragged row blocks
    S(5, 64, 10, 12, 64, 3, 3, 2, 1, 2),   # the same, stride 2, odd output plane (5x6)
    S(2, 16, 6, 8, 16, 3, 3, 1, 0, 1),     # no padding
    S(1, 32, 4, 4, 32, 3, 3, 1, 1, 1),     # several images per wave tile, fewer images than that
    S(9, 32, 4, 4, 64, 3, 3, 1, 2, 2),     # pad 2, images per tile not dividing the batch
    S(1, 3, 32, 32, 32, 3, 3, 1, 1, 1),    # stem: CPG = 3 padded to the MFMA k extent
    S(1, 3, 40, 40, 64, 7, 7, 2, 3, 1),    # 7x7 stride 2
    S(2, 32, 32, 32, 64, 1, 1, 2, 0, 1),   # 1x1 stride 2 shortcut
    S(1, 16, 14, 14, 32, 1, 1, 1, 0, 1),   # pointwise
    S(3, 64, 14, 14, 128, 1, 1, 1, 0, 1),  # pointwise on planes whose rows are not a multiple of 4 wide
    S(2, 32, 6, 10, 32, 1, 1, 1, 0, 2),    # grouped pointwise, 60-element planes
    S(5, 32, 7, 7, 64, 1, 1, 1, 0, 1),     # pointwise, odd plane size (no re-pitch possible)
    S(300, 32, 16, 16, 32, 3, 3, 1, 1, 8),  # 4 filters per group, several waves of blocks
    S(520, 16, 9, 12, 32, 3, 3, 2, 1, 4),   # 8 filters per group, stride 2, odd height, large batch
    S(700, 16, 7, 7, 16, 3, 3, 1, 1, 4),    # 7x7 planes: scalar staging, several images per tile, ragged tail
    S(1, 8, 12, 12, 8, 3, 3, 1, 1, 8),     # depthwise
    S(2, 8, 7, 7, 8, 3, 3, 2, 1, 8),       # depthwise stride 2, odd size
    S(1, 8, 9, 9, 16, 3, 3, 1, 1, 8),      # depthwise, channel multiplier 2
    S(3, 37, 14, 14, 37, 3, 3, 1, 1, 37),  # depthwise on whole small planes, plane count not a multiple of 4
    S(5, 13, 7, 7, 13, 3, 3, 2, 1, 13),    # the same, stride 2, odd plane size (tail of the last block)
    S(2, 6, 28, 28, 6, 3, 3, 2, 1, 6),     # 28x28 stride 2
    S(1, 10, 9, 8, 15, 2, 3, 1, 0, 5),     # KH != KW, no padding
    S(1, 4, 6, 6, 4, 5, 5, 1, 2, 2),       # 5x5
    S(1, 8, 5, 5, 8, 3, 3, 3, 2, 2),       # stride 3, pad 2
    S(1, 64, 56, 56, 64, 3, 3, 1, 1, 2),   # ResNet-like row blocks with ragged tail
    S(1, 128, 28, 28, 128, 3, 3, 1, 1, 32),
    S(1, 512, 7, 7, 512, 3, 3, 1, 1, 32),
]


@pytest.mark.parametrize("s", SWEEP, ids=lambda s: "x".join(map(str, s)))
def test_sweep_auto(gpu, s):
    check(gpu, s, seed=11)


@pytest.mark.parametrize("s", SWEEP, ids=lambda s: "x".join(map(str, s)))
def test_sweep_direct(gpu, s):
    _, b = gpu
    name = check(gpu, s, seed=12, path=b.PATH_DIRECT)
    assert "direct" in name or "depthwise" in name


@pytest.mark.parametrize("s", SWEEP, ids=lambda s: "x".join(map(str, s)))
def test_sweep_mfma(gpu, s):
    _, b = gpu
    try:
        name = check(gpu, s, seed=13, path=b.PATH_MFMA)
    except b.GspcError as e:
        assert e.code == -8      # family has no instance for this layer
        pytest.skip("no matrix-core instance for this shape")
    assert "mfma" in name


@pytest.mark.parametrize("g", [1, 2, 4, 8, 16])
def test_wrn_layers_n4(gpu, g):
    for i, s in enumerate(wl.wrn_grouped_shapes(4, g)):
        check(gpu, s, seed=wl.make_seed(2, i, g))


@pytest.mark.parametrize("g", [2, 4, 8, 16, 32])
def test_resnet_layers_n1(gpu, g):
    for i, s in enumerate(wl.resnet34_grouped_shapes(1, g)):
        check(gpu, s, seed=wl.make_seed(3, i, g))


def test_depthwise_pairs(gpu):
    for i, (dw, pw) in enumerate(wl.depthwise_pairs(1)):
        check(gpu, dw, seed=wl.make_seed(4, 2 * i, dw.groups))
        check(gpu, pw, seed=wl.make_seed(4, 2 * i + 1, 1))


DW_WAVE = [   # (N, C, plane edge, stride): enough planes for the whole-planes-per-wavefront kernel, ragged last wavefront
    (3, 101, 112, 1), (17, 129, 56, 1), (33, 129, 28, 1), (63, 131, 28, 2), (37, 521, 14, 1), (33, 521, 14, 2), (129, 1031, 7, 1), (129, 1031, 7, 2),
]


@pytest.mark.parametrize("N,C,hw,stride", DW_WAVE, ids=lambda v: str(v))
def test_depthwise_whole_planes_per_wavefront(gpu, N, C, hw, stride):
    """Depthwise 3x3 at batches that fill the chip, on 56x56 to 7x7 planes (whole planes per wavefront) and on
    112x112 planes (a band of rows per wavefront): whole tensors against the oracle, plane count not a
    multiple of a wavefront's share; then the same layer with residual and ReLU in a chain."""
    torch, b = gpu
    from helpers import gpu_chain, oracle_chain
    s = S(N, C, hw, hw, C, 3, 3, stride, 1, C)
    name = check(gpu, s, seed=wl.make_seed(4, 700 + hw, stride))
    assert name.startswith((f"conv_dw_wave<{stride},{hw},{hw},", f"conv_dw_band<{stride},{hw},{hw},")), name
    ho = (hw - 1) // stride + 1
    ch = wl.Chain("dwres", (N, C, hw, hw))
    ch.conv(0, 1, N, C, hw, hw, C, 3, stride, 1, C, relu=True)
    ch.conv(0, 2, N, C, hw, hw, C, 3, stride, 1, C, relu=True, residual=1)
    ch.conv(0, 3, N, C, hw, hw, C, 3, stride, 1, C, residual=2)
    x0 = wl.make_input(ch.input_shape, 91)
    weights = ch.make_weights(17)
    ref = oracle_chain(ch, x0, weights, threads=8)
    lc, bufs = gpu_chain(ch, x0, weights)
    for bf in bufs[1:]:
        bf.fill_(float("nan"))
    b.gspc_run_layer_chain(lc)
    torch.cuda.synchronize()
    assert b.gspc_last_kernel().startswith(("conv_dw_wave<", "conv_dw_band<")), b.gspc_last_kernel()
    for i in (1, 2, 3):
        got = bufs[i][:N * C * ho * ho].cpu().numpy().reshape(ref[i].shape)
        assert rel_err(got, ref[i]) < TOL_F32, i


def test_pack_is_a_permutation(gpu):
    torch, b = gpu
    dev = torch.device("cuda:0")
    for (Cout, Cin, K, g) in [(64, 64, 3, 4), (24, 12, 3, 3), (6, 4, 3, 2), (128, 128, 1, 1),
                              (32, 3, 7, 1), (16, 16, 3, 16)]:
        w = wl.make_weight(Cout, Cin // g, K, K, 5)
        pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), g)
        back = b.gspc_unpack_weights(pw, b.PATH_DIRECT).cpu().numpy()
        assert np.array_equal(back, w)
        if pw.info()["has_mfma"]:
            back = b.gspc_unpack_weights(pw, b.PATH_MFMA).cpu().numpy()
            assert np.array_equal(back, w)
        # padding lanes are zero and nothing else was invented: the packed
        # bytes hold every weight at least once and otherwise only zeros
        n = b.gspc_packed_weight_bytes(Cin, Cout, K, K, g)
        if K == 3 and Cout // g >= 12 and (Cin // g) % 4 == 0 and Cin // g >= 8:
            # the trailing Winograd section holds transformed filters (checked in test_gpu_winograd.py)
            n -= g * (Cin // g // 4) * ((Cout // g + 15) // 16) * 4096
        off = (-pw.storage.data_ptr()) % 256
        flat = pw.storage[off:off + n].view(torch.float32).cpu().numpy()
        vals = set(np.unique(flat).tolist())
        assert vals <= set(np.unique(w).tolist()) | {0.0}


def test_bf16_cast_matches_host_rounding(gpu):
    torch, b = gpu
    x = wl.make_input((3, 5, 7, 11), 6)
    x[0, 0, 0, :4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]   # ties
    bits, _ = wl.round_to_bf16(x)
    got = b.gspc_pack_input_bf16(torch.from_numpy(x).cuda()).view(torch.int16).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), bits)


@pytest.mark.parametrize("s", [
    S(2, 64, 14, 14, 64, 3, 3, 1, 1, 2),
    S(2, 64, 14, 14, 128, 3, 3, 2, 1, 8),
    S(1, 64, 12, 12, 64, 3, 3, 1, 1, 32),
    S(2, 128, 7, 7, 128, 3, 3, 1, 1, 2),      # two chunks of 32 channels, odd width (2-byte loads)
    S(1, 64, 56, 56, 64, 3, 3, 1, 1, 2),      # row blocks with a ragged tail, 8-byte loads
    S(3, 32, 9, 12, 64, 3, 3, 2, 1, 2),       # 16 channels per group, stride 2, odd height
    S(2, 48, 10, 10, 32, 3, 3, 1, 1, 2),      # 24 channels per group: chunks of 8
    S(1, 256, 8, 8, 512, 3, 3, 2, 1, 2),      # four chunks, 256 filters per group
    S(2, 64, 14, 14, 64, 3, 3, 1, 1, 8),      # 8 filters per group: half of the filter tile is padding
    S(1, 48, 10, 10, 144, 3, 3, 1, 1, 6),     # 24 filters per group: ragged last filter tile
], ids=lambda s: "x".join(map(str, s)))
def test_bf16_layers(gpu, s):
    torch, b = gpu
    for path in (b.PATH_AUTO, b.PATH_DIRECT):
        y, x, w, name = run_conv(gpu, s, seed=21, path=path, dtype=b.GSPC_BF16)
        _, xr = wl.round_to_bf16(x)
        _, wr = wl.round_to_bf16(w)
        # primary: same rounded operands on both sides, only accumulation differs
        ref_r = oracle.conv2d_grouped(xr, wr, s.stride, s.pad, s.groups, threads=8)
        assert rel_err(y, ref_r) < 1e-4, name
        # secondary: against the un-rounded data, the stated bf16 tolerance
        ref = oracle.conv2d_grouped(x, w, s.stride, s.pad, s.groups, threads=8)
        assert rel_err(y, ref) < TOL_BF16, name


# bf16 layers with few channels per group: the row-product kernel (groups of fewer than 8
# channels are merged into block-diagonal groups of 8 by the pack step).
ROW_BF16 = [
    S(2, 64, 56, 56, 64, 3, 3, 1, 1, 8),      # 8 channels, 8 filters per group; 14 windows per row
    S(3, 64, 56, 56, 64, 3, 3, 1, 1, 32),     # 2 and 2: four groups merged
    S(5, 128, 28, 28, 128, 3, 3, 1, 1, 32),   # 4 and 4: two groups merged; two images per wave, odd batch
    S(3, 128, 28, 28, 128, 3, 3, 1, 1, 8),    # 16 and 16: two waves share a group's input
    S(2, 16, 12, 12, 32, 3, 3, 1, 1, 2),      # 8 channels, 16 filters; three windows per row, four images per wave
    S(9, 8, 9, 8, 8, 3, 3, 1, 1, 8),          # depthwise, all eight groups merged; two windows per row
    S(2, 32, 7, 64, 32, 3, 3, 1, 1, 4),       # sixteen windows per row, fewer rows than a band
    S(1, 16, 40, 20, 24, 3, 3, 1, 1, 2),      # 12 filters per group: three filter quads
    S(3, 48, 16, 16, 48, 3, 3, 1, 1, 3),      # 16 and 16, three groups
    S(1, 24, 33, 36, 24, 3, 3, 1, 1, 12),     # 2 and 2, twelve groups in three merged ones; odd height
]


@pytest.mark.parametrize("s", ROW_BF16, ids=lambda s: "x".join(map(str, s)))
def test_bf16_row_kernel(gpu, s):
    torch, b = gpu
    y, x, w, name = run_conv(gpu, s, seed=33, dtype=b.GSPC_BF16)
    assert name.startswith("conv_row16"), name
    assert not np.isnan(y).any(), name
    _, xr = wl.round_to_bf16(x)
    _, wr = wl.round_to_bf16(w)
    ref_r = oracle.conv2d_grouped(xr, wr, s.stride, s.pad, s.groups, threads=8)
    assert rel_err(y, ref_r) < 1e-4, name
    ref = oracle.conv2d_grouped(x, w, s.stride, s.pad, s.groups, threads=8)
    assert rel_err(y, ref) < TOL_BF16, name


@pytest.mark.parametrize("env,expect", [
    ({"GSPC_ROWB_BANDS": "1"}, "conv_row16q<2,2>/1b"),
    ({"GSPC_ROWB_BANDS": "3"}, "conv_row16q<2,2>/3b"),
    ({"GSPC_ROWB_BANDS": "8"}, "conv_row16q<2,2>/7b"),       # 8 bands of 4 rows: the 26 rows need 7
    ({"GSPC_TILER": "0", "GSPC_ROWB_BANDS": "1"}, "conv_row16b<2,2,4,4>/1b"),   # the one-row-at-a-time form
    ({"GSPC_TILER": "0", "GSPC_ROWB_BANDS": "3"}, "conv_row16b<2,2,4,4>/3b"),
    ({"GSPC_TILER": "2"}, "conv_row16b<2,1,4,4>"),            # one filter quad per wave: two waves share the input
    ({"GSPC_TILER": "7"}, "conv_row16q<2,1>"),
    ({"GSPC_TILER": "5"}, "conv_row16b<2,2,8,2>"),            # seven rows in flight
])
def test_bf16_row_kernel_forms_and_bands(gpu, env, expect):
    """Both forms of the row-product kernel, and row bands (each re-reads one row of its
    neighbours above and below) that must tile the plane exactly, also when the band height
    does not divide the plane.  The choice is made per process, hence the child process."""
    import subprocess, sys, os, textwrap
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = textwrap.dedent(f"""
        import sys, numpy as np
        sys.path.insert(0, {root!r}); sys.path.insert(0, {os.path.join(root, "tests")!r})
        import torch, oracle
        from paper_2006_09791_amd import binding as b, workloads as wl
        from helpers import rel_err
        for s in (wl.ConvShape(3, 32, 26, 24, 32, 3, 3, 1, 1, 8), wl.ConvShape(5, 16, 9, 12, 16, 3, 3, 1, 1, 8)):
            x = wl.make_input((s.N, s.Cin, s.H, s.W), 5); w = wl.make_weight(s.Cout, s.Cin // s.groups, 3, 3, 6)
            pw = b.gspc_pack_weights(torch.from_numpy(w).cuda(), s.groups, b.GSPC_BF16)
            xd = b.gspc_pack_input_bf16(torch.from_numpy(x).cuda())
            y = torch.full((s.N, s.Cout, s.H, s.W), float("nan"), device="cuda")
            b.gspc_conv2d_grouped(xd, pw, s.N, s.Cin, s.H, s.W, s.Cout, 3, 3, 1, 1, s.groups, y)
            torch.cuda.synchronize()
            _, xr = wl.round_to_bf16(x); _, wr = wl.round_to_bf16(w)
            err = rel_err(y.cpu().numpy(), oracle.conv2d_grouped(xr, wr, 1, 1, s.groups, threads=8))
            print(b.gspc_last_kernel(), err < 1e-4)
    """)
    out = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, **env), check=True, capture_output=True,
                         text=True).stdout
    lines = [l for l in out.strip().splitlines() if l.startswith("conv_")]
    assert len(lines) == 2 and all(l.endswith("True") for l in lines), out
    assert lines[0].startswith(expect), out


def test_bf16_row_kernel_with_residual_and_relu(gpu):
    """Epilogue form of the row-product kernel in a chain: conv + residual + ReLU, whole tensors."""
    torch, b = gpu
    from helpers import gpu_chain, oracle_chain
    N, C, hw, g = 3, 64, 28, 16
    ch = wl.Chain("rowres", (N, C, hw, hw))
    ch.conv(0, 1, N, C, hw, hw, C, 3, 1, 1, g, relu=True)
    ch.conv(0, 2, N, C, hw, hw, C, 3, 1, 1, g, relu=True, residual=1)
    ch.conv(0, 3, N, C, hw, hw, C, 3, 1, 1, g, residual=2)
    x0 = wl.make_input(ch.input_shape, 43)
    _, x0r = wl.round_to_bf16(x0)
    weights = [wl.round_to_bf16(w)[1] for w in ch.make_weights(11)]
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), g, b.GSPC_BF16) for w in weights]
    xd = b.gspc_pack_input_bf16(torch.from_numpy(x0).to(dev))
    ref = oracle_chain(ch, x0r, weights, threads=8)
    # every layer reads the bf16 input (buffer 0) and writes fp32: run them one by one
    bufs = [xd] + [torch.full((N * C * hw * hw,), float("nan"), device=dev) for _ in range(3)]
    for li, l in enumerate(ch.layers):
        b.gspc_run_layer_chain(b.LayerChain([l._replace(wid=0)], [packed[li]], bufs))
        torch.cuda.synchronize()
        assert b.gspc_last_kernel().startswith("conv_row16"), b.gspc_last_kernel()
        got = bufs[l.dst].cpu().numpy().reshape(ref[l.dst].shape)
        assert rel_err(got, ref[l.dst]) < 1e-4, li


@pytest.mark.parametrize("s,expect", [
    (S(5, 32, 12, 12, 32, 3, 3, 1, 1, 16), "conv_mfma4r<4,"),    # 2 and 2 -> pairs of groups as 4 and 4
    (S(3, 16, 9, 8, 32, 3, 3, 2, 1, 8), "conv_mfma4r<4,"),       # 2 channels, 4 filters -> 4 and 8, stride 2
    (S(2, 8, 10, 10, 16, 3, 3, 1, 1, 8), "conv_mfma4r<4,"),      # 1 channel, 2 filters (channel multiplier) -> 4 and 8
    (S(2, 12, 7, 7, 12, 3, 3, 1, 1, 6), None),                   # six groups of 2: pairs merge, three merged groups
])
def test_small_groups_run_as_merged_groups(gpu, s, expect):
    """Groups of fewer than four channels or filters run as block-diagonal merged groups on the
    4x4x1 matrix-core kernel (fp32): same result as the definition, which never mixes groups."""
    name = check(gpu, s, seed=37)
    if expect:
        assert name.startswith(expect), name


def test_rerun_is_bit_identical(gpu):
    s = wl.wrn_grouped_shapes(2, 2)[2]
    y1, *_ = run_conv(gpu, s, seed=31)
    y2, *_ = run_conv(gpu, s, seed=31)
    assert np.array_equal(y1, y2)


def test_mismatch_and_errors_on_device(gpu):
    torch, b = gpu
    dev = torch.device("cuda:0")
    w = wl.make_weight(8, 4, 3, 3, 1)
    pw = b.gspc_pack_weights(torch.from_numpy(w).to(dev), 2)
    x = torch.zeros((1, 8, 6, 6), device=dev)
    y = torch.zeros((1, 8, 6, 6), device=dev)
    with pytest.raises(b.GspcError) as e:
        b.gspc_conv2d_grouped(x, pw, 1, 8, 6, 6, 8, 3, 3, 1, 1, 4, y)
    assert e.value.code == -5
    with pytest.raises(b.GspcError) as e:
        b.gspc_conv2d_grouped(x, pw, 1, 8, 1, 1, 8, 3, 3, 1, 0, 2, y)
    assert e.value.code == -2


def test_tile_table_overrides_the_planner(gpu, tmp_path):
    """A process started with GSPC_TUNE_FILE takes the table's kernel family and tile for
    the listed layer (and still matches the oracle); unlisted layers are untouched."""
    import subprocess, sys, os, textwrap
    table = tmp_path / "t.tune"
    table.write_text("# test table\n64 64 16 16 64 3 3 1 1 2 0 m 8\n3 64 16 16 64 3 3 1 1 2 0 x 2\n")
    code = textwrap.dedent(f"""
        import sys, numpy as np
        sys.path.insert(0, {os.path.dirname(os.path.dirname(os.path.abspath(__file__)))!r})
        sys.path.insert(0, {os.path.dirname(os.path.abspath(__file__))!r})
        import torch, oracle
        from paper_2006_09791_amd import binding as b, workloads as wl
        from helpers import rel_err
        S = wl.ConvShape
        b.gspc_set_winograd(0)   # the unlisted layer then shows the direct planner's own choice
        for s in (S(64, 64, 16, 16, 64, 3, 3, 1, 1, 2), S(64, 64, 16, 16, 64, 3, 3, 1, 1, 4), S(3, 64, 16, 16, 64, 3, 3, 1, 1, 2)):
            x = wl.make_input((s.N, s.Cin, s.H, s.W), 3); w = wl.make_weight(s.Cout, s.Cin // s.groups, 3, 3, 4)
            pw = b.gspc_pack_weights(torch.from_numpy(w).cuda(), s.groups)
            y = torch.empty((s.N, s.Cout, s.H, s.W), device="cuda")
            b.gspc_conv2d_grouped(torch.from_numpy(x).cuda(), pw, s.N, s.Cin, s.H, s.W, s.Cout, 3, 3, 1, 1, s.groups, y)
            torch.cuda.synchronize()
            err = rel_err(y.cpu().numpy(), oracle.conv2d_grouped(x, w, 1, 1, s.groups, threads=8))
            print(b.gspc_last_kernel(), err < 1e-4)
    """)
    env = dict(os.environ, GSPC_TUNE_FILE=str(table))
    out = subprocess.run([sys.executable, "-c", code], env=env, check=True, capture_output=True, text=True).stdout
    lines = [l for l in out.strip().splitlines() if l.startswith("conv_")]
    assert lines[0].startswith("conv_mfma16<1,1,1,4,3,3,1,f32,") and lines[0].endswith("True"), out
    assert lines[1].startswith("conv_mfma16w<") and lines[1].endswith("True"), out
    # family 'x': Winograd F(2x2, 3x3) for a layer the automatic mode would leave to the direct kernels
    assert lines[2].startswith("conv_wino<1,1,2,2,") and lines[2].endswith("True"), out


def test_tile_table_is_keyed_by_the_callers_plane_size(gpu, tmp_path):
    """A 1x1 layer on 14x14 planes reaches the planners as a re-pitched plane; its table line,
    written with the caller's H and W, must still be found."""
    import subprocess, sys, os, textwrap
    table = tmp_path / "t.tune"
    table.write_text("64 64 14 14 128 1 1 1 0 1 0 m 8\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = textwrap.dedent(f"""
        import sys
        sys.path.insert(0, {root!r}); sys.path.insert(0, {os.path.join(root, "tests")!r})
        import torch, oracle
        from paper_2006_09791_amd import binding as b, workloads as wl
        from helpers import rel_err
        s = wl.ConvShape(64, 64, 14, 14, 128, 1, 1, 1, 0, 1)
        x = wl.make_input((s.N, s.Cin, s.H, s.W), 3); w = wl.make_weight(s.Cout, s.Cin, 1, 1, 4)
        pw = b.gspc_pack_weights(torch.from_numpy(w).cuda(), 1)
        y = torch.empty((s.N, s.Cout, s.H, s.W), device="cuda")
        b.gspc_conv2d_grouped(torch.from_numpy(x).cuda(), pw, s.N, s.Cin, s.H, s.W, s.Cout, 1, 1, 1, 0, 1, y)
        torch.cuda.synchronize()
        print(b.gspc_last_kernel(), rel_err(y.cpu().numpy(), oracle.conv2d_grouped(x, w, 1, 0, 1, threads=8)) < 1e-4)
    """)
    names = []
    for env in (dict(os.environ, GSPC_TUNE_FILE=str(table)), {k: v for k, v in os.environ.items() if k != "GSPC_TUNE_FILE"}):
        out = subprocess.run([sys.executable, "-c", code], env=env, check=True, capture_output=True, text=True).stdout
        line = [l for l in out.strip().splitlines() if l.startswith("conv_")][-1]
        assert line.endswith("True"), out
        names.append(line.split()[0])
    assert names[0].startswith("conv_mfma16<1,1,1,4,1,1,1,f32,"), names      # configuration 8 of family 'm'
    assert names[0] != names[1], names                                       # the heuristic choice is another one


# Filters per group that are not a multiple of 16 (the G(g) forms of a MobileNetV2-shaped
# network, Section IV-A: 96, 144, 192, 384, 576 and 960 channels over 2..16 groups): the plain
# 16x16x4 kernel zero-pads the last filter tile and drops its padding filters at the store.
PADDED_TILES = [
    S(2, 960, 7, 7, 960, 3, 3, 1, 1, 8),     # 120 filters: 8 tiles, the last half empty; scalar stores
    S(1, 144, 28, 28, 144, 3, 3, 1, 1, 2),   # 72: 5 tiles; 16-byte stores
    S(3, 144, 28, 28, 144, 3, 3, 2, 1, 2),   # stride 2
    S(2, 240, 14, 14, 240, 3, 3, 1, 1, 4),   # 60
    S(2, 144, 20, 20, 144, 3, 3, 1, 1, 4),   # 36
    S(1, 96, 56, 56, 96, 3, 3, 2, 1, 4),     # 24
    S(2, 144, 14, 14, 144, 3, 3, 1, 1, 8),   # 18 filters and 18 channels: both edges padded
    S(2, 192, 28, 28, 192, 3, 3, 2, 1, 16),  # 12
    S(3, 144, 12, 12, 144, 3, 3, 1, 1, 16),  # 9
    S(2, 96, 16, 16, 96, 3, 3, 2, 1, 16),    # 6
    S(2, 20, 9, 9, 20, 3, 3, 1, 1, 4),       # 5, odd plane
    S(2, 144, 28, 28, 24, 1, 1, 1, 0, 1),    # pointwise projection to 24 channels
    S(3, 96, 7, 7, 40, 1, 1, 1, 0, 1),       # pointwise, 49-element planes
    S(70, 144, 14, 14, 144, 3, 3, 1, 1, 2),  # 72 at a batch that fills the chip (larger block shapes)
]


@pytest.mark.parametrize("s", PADDED_TILES, ids=lambda s: "x".join(map(str, s)))
def test_filters_per_group_not_a_multiple_of_16(gpu, s):
    _, b = gpu
    b.gspc_set_winograd(0)   # the direct kernel is the one under test (large launches would take Winograd)
    try:
        name = check(gpu, s, seed=23)
    finally:
        b.gspc_set_winograd(None)
    assert name.startswith("conv_mfma16<"), name


# 1x1 layers on planes whose size is not a multiple of 4: the plane travels as one row of H*W elements
# and, where a block covers one image, four channels at a time are staged as one aligned row.
ODD_PLANES = [
    S(3, 64, 5, 5, 64, 1, 1, 1, 0, 1),
    S(2, 32, 9, 9, 48, 1, 1, 1, 0, 2),       # grouped, three filter tiles
    S(5, 128, 13, 13, 64, 1, 1, 1, 0, 1),    # 169-element planes
    S(2, 64, 15, 15, 32, 1, 1, 1, 0, 1),     # 225
    S(3, 24, 3, 3, 16, 1, 1, 1, 0, 1),       # 9: smaller than any tile
    S(70, 160, 7, 7, 960, 1, 1, 1, 0, 1),    # MobileNetV2 expansion at a batch that fills the chip
    S(1, 960, 7, 7, 160, 1, 1, 1, 0, 1),     # projection at batch 1: 240 k-steps
    S(2, 6, 7, 7, 16, 1, 1, 1, 0, 1),        # padded channels: single row, but no four-channel staging
    S(4, 40, 7, 9, 40, 1, 1, 1, 0, 2),       # non-square, 63 elements, 20 filters per group
]


@pytest.mark.parametrize("s", ODD_PLANES, ids=lambda s: "x".join(map(str, s)))
def test_pointwise_on_odd_planes(gpu, s):
    check(gpu, s, seed=29)


def test_pointwise_on_odd_planes_bf16(gpu):
    torch, b = gpu
    s = S(3, 64, 7, 7, 64, 1, 1, 1, 0, 1)
    y, x, w, name = run_conv(gpu, s, seed=30, dtype=b.GSPC_BF16)
    _, xr = wl.round_to_bf16(x)
    _, wr = wl.round_to_bf16(w)
    ref = oracle.conv2d_grouped(xr, wr, 1, 0, 1, threads=8)
    assert rel_err(y, ref) < 1e-4, name


# Dense pointwise layers with at least 128 filters at batches that give every compute unit two blocks run in
# eight-wave blocks of 128 filters x 128 pixels.
@pytest.mark.parametrize("s", [
    S(48, 64, 28, 28, 256, 1, 1, 1, 0, 1),     # 784-pixel planes: tiles straddle images
    S(113, 96, 30, 20, 128, 1, 1, 1, 0, 1),    # ragged last pixel tile, one filter block
    S(140, 160, 14, 14, 384, 1, 1, 1, 0, 1),   # 14x14 planes (re-pitched to rows of 4), three filter blocks
], ids=lambda s: "x".join(map(str, s)))
def test_pointwise_in_128_filter_blocks(gpu, s):
    name = check(gpu, s, seed=wl.make_seed(7, s.Cin, s.H))
    assert name.startswith("conv_mfma16<4,2,2,4,1,1,1,f32"), name
