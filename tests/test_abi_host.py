"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/gspc.h declares, and rejects bad arguments before any
GPU work (all these calls return before the first HIP call)."""
import ctypes
import os
import re

import pytest

from paper_2006_09791_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gspc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gspc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = b.load()
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), f"{n} declared in gspc.h but not exported"
    assert set(names) == set(b.EXPORTS)


def test_version_and_output_dims():
    assert b.gspc_version() == 1
    assert b.gspc_output_dims(32, 32, 3, 3, 1, 1) == (32, 32)
    assert b.gspc_output_dims(7, 7, 3, 3, 2, 1) == (4, 4)
    assert b.gspc_output_dims(224, 224, 7, 7, 2, 3) == (112, 112)
    with pytest.raises(b.GspcError) as e:
        b.gspc_output_dims(2, 2, 5, 5, 1, 0)
    assert e.value.code == -2
    with pytest.raises(b.GspcError) as e:
        b.gspc_output_dims(8, 8, 3, 3, 0, 1)
    assert e.value.code == -2


def test_layer_macs_is_eq2():
    assert b.gspc_layer_macs(1, 64, 64, 3, 3, 32, 32, 4) == 9437184
    assert b.gspc_layer_macs(2, 6, 4, 3, 3, 3, 2, 2) == 2 * 6 * 4 * 9 * 6 // 2
    assert b.gspc_layer_macs(1, 0, 4, 3, 3, 3, 2, 2) == 0


def test_packed_bytes_and_group_divisibility():
    lib = b.load()
    n = b.gspc_packed_weight_bytes(64, 64, 3, 3, 4)
    assert n >= 64 * 16 * 9 * 4 and n % 4 == 0
    # KPG = 16 carries a matrix-core section on top of the direct one
    assert n > b.gspc_packed_weight_bytes(64, 8, 3, 3, 4)
    assert lib.gspc_packed_weight_bytes(6, 4, 3, 3, 4, 0) == 0       # 6 % 4 != 0
    assert "divisible" in b.gspc_last_error()
    assert lib.gspc_packed_weight_bytes(8, 8, 3, 3, 2, 7) == 0       # unknown dtype
    assert lib.gspc_packed_weight_bytes(8, 8, 0, 3, 2, 0) == 0


def test_pack_and_conv_reject_bad_arguments_before_any_launch():
    lib = b.load()
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(256 * 1024)          # never dereferenced: validation fails first
    assert lib.gspc_pack_weights(None, 8, 8, 3, 3, 2, 0, fake, 1 << 20, ctypes.byref(h)) == -1
    assert lib.gspc_pack_weights(fake, 8, 8, 3, 3, 3, 0, fake, 1 << 20, ctypes.byref(h)) == -3
    assert lib.gspc_pack_weights(fake, 8, 8, 3, 3, 2, 5, fake, 1 << 20, ctypes.byref(h)) == -4
    assert lib.gspc_pack_weights(fake, 8, 8, 3, 3, 2, 0, fake, 16, ctypes.byref(h)) == -6
    assert lib.gspc_pack_weights(fake, 8, 8, 3, 3, 2, 0, ctypes.c_void_p(256 * 1024 + 4), 1 << 20,
                                 ctypes.byref(h)) == -8
    assert lib.gspc_conv2d_grouped(fake, None, 1, 8, 4, 4, 8, 3, 3, 1, 1, 2, fake) == -1
    odd = ctypes.c_void_p(256 * 1024 + 4)        # the alignment is checked before the handle is read
    assert lib.gspc_conv2d_grouped(odd, fake, 1, 8, 4, 4, 8, 3, 3, 1, 1, 2, fake) == -8
    assert lib.gspc_conv2d_grouped(fake, fake, 1, 8, 4, 4, 8, 3, 3, 1, 1, 2, odd) == -8
    assert lib.gspc_unpack_weights(None, 0, fake) == -1
    assert lib.gspc_packed_info(None, None, None, None, None, None, None, None) == -1
    assert lib.gspc_pack_input_bf16(None, 4, fake) == -1
    assert lib.gspc_force_path(9) == -8
    assert lib.gspc_force_path(-1) == 0
    lib.gspc_packed_free(None)


def test_chain_rejects_bad_arguments_before_any_launch():
    lib = b.load()
    layers = (b.GspcLayer * 1)()
    bufs = (ctypes.c_void_p * 2)(256 * 1024, 512 * 1024)
    sizes = (ctypes.c_size_t * 2)(1024, 1024)
    assert lib.gspc_run_layer_chain(None, 1, bufs, sizes, 2, None) == -1
    assert lib.gspc_run_layer_chain(layers, 0, bufs, sizes, 2, None) == -8
    odd_bufs = (ctypes.c_void_p * 2)(256 * 1024, 512 * 1024 + 8)
    assert lib.gspc_run_layer_chain(layers, 1, odd_bufs, sizes, 2, None) == -8  # misaligned buffer
    L = layers[0]
    L.op, L.src, L.dst, L.src2 = b.OP_RELU, 0, 5, -1
    L.N, L.Cin, L.H, L.W = 1, 4, 4, 4
    assert lib.gspc_run_layer_chain(layers, 1, bufs, sizes, 2, None) == -8     # dst out of range
    L.dst = 1
    L.Cin = 4096
    assert lib.gspc_run_layer_chain(layers, 1, bufs, sizes, 2, None) == -6     # buffer too small
    L.Cin, L.op = 4, 77
    assert lib.gspc_run_layer_chain(layers, 1, bufs, sizes, 2, None) == -8     # unknown op
    L.op, L.w = b.OP_CONV, None
    assert lib.gspc_run_layer_chain(layers, 1, bufs, sizes, 2, None) == -1     # conv without weights


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2006_09791_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle|liboracle|oracle_conv|#include.*oracle",
                                     text, flags=re.M), f"{f} reaches into the oracle"


def test_autotuner_table_lines_parse_back():
    """The autotuner's table format (one layer per line: ten shape integers, dtype, family
    letter, index) is what the library's reader expects: 13 whitespace-separated fields."""
    from paper_2006_09791_amd import autotune, workloads as wl
    s = wl.ConvShape(64, 32, 32, 32, 64, 3, 3, 2, 1, 4)
    line = autotune.table_line(s, "f32", "m", 7)
    f = line.split()
    assert len(f) == 13 and [int(v) for v in f[:11]] == [64, 32, 32, 32, 64, 3, 3, 2, 1, 4, 0]
    assert f[11] == "m" and f[12] == "7"
    assert autotune.table_line(s, "bf16", "b", 0).split()[10] == "1"
    shapes, dtype = autotune.workload_shapes("resnet34_bf16", 256)
    assert dtype == "bf16" and len(shapes) == 21


def test_mobilenetv2_shaped_chain_matches_the_published_model_size():
    """Section IV-A quotes 3.5 million parameters and 53 layers for MobileNetV2: the chain's
    52 convolutions carry 2.19 M weights, which with the 1280 -> 1000 classifier (1.281 M) and
    the 34 112 batch-norm scales and shifts (two per output channel of every convolution)
    give that figure; the depthwise form needs about 300 M multiply-accumulates (Eq. 2 summed)."""
    import numpy as np
    from paper_2006_09791_amd import workloads as wl
    ch = wl.mobilenetv2_chain(1)
    assert len(ch.layers) == 52 and all(l.op == "conv" for l in ch.layers)
    weights = sum(int(np.prod(s)) for s in ch.weight_shapes)
    bn = 2 * sum(s[0] for s in ch.weight_shapes)
    assert weights == 2189760 and bn == 34112
    assert abs(weights + bn + 1280 * 1000 + 1000 - 3.5e6) < 0.01 * 3.5e6
    assert abs(ch.macs() - 300e6) < 0.01 * 300e6
    assert ch.out_shape == (1, 1280, 7, 7)
    # G(g) variants keep every shape and scale the 3x3 work by channels / g
    for g in (2, 4, 8, 16):
        cg = wl.mobilenetv2_chain(1, g)
        assert [(l.Cin, l.Cout, l.H, l.KH, l.stride) for l in cg.layers] == [(l.Cin, l.Cout, l.H, l.KH, l.stride) for l in ch.layers]
        assert all(l.groups in (1, g) for l in cg.layers)
    # no step reads a buffer it writes
    for l in ch.layers:
        assert l.dst != l.src and l.dst != l.src2


def test_pointwise_form_doubles_the_3x3_layers():
    """Section IV-A: each 3x3 convolution becomes a grouped 3x3 a -> a plus a 1x1 a -> b."""
    from paper_2006_09791_amd import workloads as wl
    plain, pw = wl.wrn_chain(1, 4), wl.wrn_chain(1, 4, pointwise=True)
    n3 = sum(1 for l in plain.layers[1:] if l.KH == 3)
    assert len(pw.layers) == len(plain.layers) + n3
    for l in pw.layers[1:]:
        if l.KH == 3:
            assert l.Cin == l.Cout and l.groups == 4
    assert pw.out_shape == plain.out_shape


def test_minimal_filtering_identity_used_by_the_winograd_kernel():
    """F(2x2, 3x3): Y = A^T [(G g G^T) .* (B^T d B)] A equals the 2x2 valid correlation of a 4x4
    patch with a 3x3 filter, and the sum over channels may be taken in the transformed domain
    (what makes the grouped form of Section VI a set of 16 per-group GEMMs).  Checked in float64
    on random data against the plain definition."""
    import numpy as np
    BT = np.array([[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]], dtype=np.float64)
    G = np.array([[1, 0, 0], [0.5, 0.5, 0.5], [0.5, -0.5, 0.5], [0, 0, 1]], dtype=np.float64)
    AT = np.array([[1, 1, 1, 0], [0, 1, -1, -1]], dtype=np.float64)
    rng = np.random.default_rng(5)
    C = 6
    d = rng.standard_normal((C, 4, 4))
    g = rng.standard_normal((C, 3, 3))
    direct = np.zeros((2, 2))
    for i in range(2):
        for j in range(2):
            direct[i, j] = np.sum(d[:, i:i + 3, j:j + 3] * g)
    M = sum((G @ g[c] @ G.T) * (BT @ d[c] @ BT.T) for c in range(C))
    assert np.allclose(AT @ M @ AT.T, direct, rtol=1e-12, atol=1e-12)


def test_autotuner_rejects_a_candidate_whose_output_differs():
    """The offline tuner accepts a (family, tile) only if its sampled output agrees with the
    heuristic choice's: the rule itself, on made-up samples."""
    from paper_2006_09791_amd import autotune
    base = {"sample": [1.0, 2.0, -3.0], "rms": 2.0}
    assert autotune.agrees({"sample": [1.0, 2.0, -3.00001], "rms": 2.0}, base)
    assert not autotune.agrees({"sample": [1.0, 2.0, -3.001], "rms": 2.0}, base)
    assert autotune.agrees({"sample": [1.0, 2.0, -3.001], "rms": 2.0}, base, tol=1e-3)
    assert not autotune.agrees({"sample": [1.0, 2.0], "rms": 2.0}, base)
