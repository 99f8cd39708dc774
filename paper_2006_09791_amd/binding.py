"""ctypes binding of libgspc.so: argument marshalling only.

Function names and argument order mirror include/gspc.h.  Device buffers are
torch tensors (PyTorch is used for device memory and streams, nothing else);
every computation runs in the library's HIP kernels.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgspc.so")

GSPC_F32, GSPC_BF16 = 0, 1
PATH_AUTO, PATH_DIRECT, PATH_MFMA = -1, 0, 1
OP_CONV, OP_MAXPOOL, OP_ADD, OP_RELU = 0, 1, 2, 3
FLAG_RELU = 1

ERROR_NAMES = {0: "GSPC_OK", -1: "GSPC_ERR_NULL", -2: "GSPC_ERR_DIM", -3: "GSPC_ERR_GROUPS",
               -4: "GSPC_ERR_DTYPE", -5: "GSPC_ERR_MISMATCH", -6: "GSPC_ERR_SPACE",
               -7: "GSPC_ERR_HIP", -8: "GSPC_ERR_ARG"}

EXPORTS = [
    "gspc_version", "gspc_set_stream", "gspc_last_error", "gspc_output_dims", "gspc_layer_macs",
    "gspc_packed_weight_bytes", "gspc_pack_weights", "gspc_unpack_weights", "gspc_packed_free",
    "gspc_packed_info", "gspc_pack_input_bf16", "gspc_conv2d_grouped", "gspc_force_path",
    "gspc_last_path", "gspc_last_kernel", "gspc_set_graph_mode", "gspc_set_chain_fusion", "gspc_set_winograd", "gspc_run_layer_chain",
]


class GspcError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {message}")
        self.code = code


class GspcLayer(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int), ("src", ctypes.c_int), ("src2", ctypes.c_int),
                ("dst", ctypes.c_int), ("N", ctypes.c_int), ("Cin", ctypes.c_int),
                ("H", ctypes.c_int), ("W", ctypes.c_int), ("Cout", ctypes.c_int),
                ("KH", ctypes.c_int), ("KW", ctypes.c_int), ("stride", ctypes.c_int),
                ("pad", ctypes.c_int), ("groups", ctypes.c_int), ("flags", ctypes.c_int),
                ("w", ctypes.c_void_p)]


_lib = None


def load():
    """Loads libgspc.so (must have been built in-tree) and sets prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2006_09791_amd.build` "
            "(there is no fallback path)")
    # torch first: it brings the HIP runtime whose streams and allocations are
    # handed to the library, and libgspc.so must bind to that same runtime.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    ip = ctypes.POINTER(ctypes.c_int)
    lib.gspc_version.restype = i
    lib.gspc_set_stream.restype = i
    lib.gspc_set_stream.argtypes = [vp]
    lib.gspc_last_error.restype = ctypes.c_char_p
    lib.gspc_output_dims.restype = i
    lib.gspc_output_dims.argtypes = [i] * 6 + [ip, ip]
    lib.gspc_layer_macs.restype = ctypes.c_uint64
    lib.gspc_layer_macs.argtypes = [i] * 8
    lib.gspc_packed_weight_bytes.restype = sz
    lib.gspc_packed_weight_bytes.argtypes = [i] * 6
    lib.gspc_pack_weights.restype = i
    lib.gspc_pack_weights.argtypes = [vp] + [i] * 6 + [vp, sz, ctypes.POINTER(vp)]
    lib.gspc_unpack_weights.restype = i
    lib.gspc_unpack_weights.argtypes = [vp, i, vp]
    lib.gspc_packed_free.restype = None
    lib.gspc_packed_free.argtypes = [vp]
    lib.gspc_packed_info.restype = i
    lib.gspc_packed_info.argtypes = [vp] + [ip] * 7
    lib.gspc_pack_input_bf16.restype = i
    lib.gspc_pack_input_bf16.argtypes = [vp, sz, vp]
    lib.gspc_conv2d_grouped.restype = i
    lib.gspc_conv2d_grouped.argtypes = [vp, vp] + [i] * 10 + [vp]
    lib.gspc_force_path.restype = i
    lib.gspc_force_path.argtypes = [i]
    lib.gspc_last_path.restype = i
    lib.gspc_set_graph_mode.restype = i
    lib.gspc_set_graph_mode.argtypes = [i]
    lib.gspc_set_chain_fusion.restype = i
    lib.gspc_set_chain_fusion.argtypes = [i]
    lib.gspc_set_winograd.restype = i
    lib.gspc_set_winograd.argtypes = [i]
    lib.gspc_last_kernel.restype = ctypes.c_char_p
    lib.gspc_run_layer_chain.restype = i
    lib.gspc_run_layer_chain.argtypes = [ctypes.POINTER(GspcLayer), i, ctypes.POINTER(vp),
                                         ctypes.POINTER(sz), i, ctypes.POINTER(ctypes.c_float)]
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise GspcError(rc, load().gspc_last_error().decode())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def gspc_version():
    return load().gspc_version()


def gspc_last_error():
    return load().gspc_last_error().decode()


def gspc_set_stream(stream=None):
    """stream: torch.cuda.Stream, raw handle, or None for torch's current stream."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    handle = getattr(stream, "cuda_stream", stream)
    _check(load().gspc_set_stream(ctypes.c_void_p(handle)))


def gspc_output_dims(H, W, KH, KW, stride, pad):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    _check(load().gspc_output_dims(H, W, KH, KW, stride, pad, ctypes.byref(ho), ctypes.byref(wo)))
    return ho.value, wo.value


def gspc_layer_macs(N, Cin, Cout, KH, KW, Hout, Wout, groups):
    return int(load().gspc_layer_macs(N, Cin, Cout, KH, KW, Hout, Wout, groups))


def gspc_packed_weight_bytes(Cin, Cout, KH, KW, groups, dtype=GSPC_F32):
    n = load().gspc_packed_weight_bytes(Cin, Cout, KH, KW, groups, dtype)
    if n == 0:
        raise GspcError(-8, gspc_last_error())
    return int(n)


class PackedWeights:
    """Owns the device bytes (a torch uint8 tensor) and the host descriptor."""

    def __init__(self, handle, storage, Cin, Cout, KH, KW, groups, dtype):
        self.handle, self.storage = handle, storage
        self.Cin, self.Cout, self.KH, self.KW, self.groups, self.dtype = Cin, Cout, KH, KW, groups, dtype

    def info(self):
        vals = [ctypes.c_int() for _ in range(7)]
        _check(load().gspc_packed_info(self.handle, *[ctypes.byref(v) for v in vals]))
        keys = ["Cin", "Cout", "KH", "KW", "groups", "dtype", "has_mfma"]
        return dict(zip(keys, (v.value for v in vals)))

    def free(self):
        if self.handle:
            load().gspc_packed_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def gspc_pack_weights(weight, groups, dtype=GSPC_F32):
    """weight: fp32 CUDA tensor [Cout, Cin/g, KH, KW] -> PackedWeights."""
    import torch
    assert weight.is_cuda and weight.dtype == torch.float32 and weight.is_contiguous()
    Cout, CPG, KH, KW = weight.shape
    Cin = CPG * groups
    nbytes = gspc_packed_weight_bytes(Cin, Cout, KH, KW, groups, dtype)
    storage = torch.empty(nbytes + 256, dtype=torch.uint8, device=weight.device)
    off = (-storage.data_ptr()) % 256
    handle = ctypes.c_void_p()
    _check(load().gspc_pack_weights(_ptr(weight), Cin, Cout, KH, KW, groups, dtype,
                                    ctypes.c_void_p(storage.data_ptr() + off), nbytes,
                                    ctypes.byref(handle)))
    return PackedWeights(handle, storage, Cin, Cout, KH, KW, groups, dtype)


def gspc_unpack_weights(packed, which=PATH_DIRECT):
    import torch
    out = torch.empty((packed.Cout, packed.Cin // packed.groups, packed.KH, packed.KW),
                      dtype=torch.float32, device=packed.storage.device)
    _check(load().gspc_unpack_weights(packed.handle, which, _ptr(out)))
    return out


def gspc_pack_input_bf16(x):
    """fp32 CUDA tensor -> bf16 CUDA tensor of the same shape (library kernel)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(load().gspc_pack_input_bf16(_ptr(x), x.numel(), _ptr(out)))
    return out


def gspc_conv2d_grouped(input, packed_weight, N, Cin, H, W, Cout, KH, KW, stride, pad, groups,
                        output=None):
    """Returns the fp32 output tensor [N, Cout, Hout, Wout] (allocated if not given)."""
    import torch
    if output is None:
        ho, wo = gspc_output_dims(H, W, KH, KW, stride, pad)
        output = torch.empty((N, Cout, ho, wo), dtype=torch.float32, device=input.device)
    _check(load().gspc_conv2d_grouped(_ptr(input), packed_weight.handle, N, Cin, H, W, Cout, KH,
                                      KW, stride, pad, groups, _ptr(output)))
    return output


def gspc_force_path(path):
    _check(load().gspc_force_path(path))


def gspc_set_graph_mode(on):
    _check(load().gspc_set_graph_mode(1 if on else 0))


def gspc_set_chain_fusion(on):
    _check(load().gspc_set_chain_fusion(1 if on else 0))


def gspc_set_winograd(on):
    """on: True / 1 = every eligible layer, False / 0 = never, None / -1 = automatic (default)."""
    _check(load().gspc_set_winograd(-1 if on is None or (on is not True and on < 0) else (1 if on else 0)))


def gspc_last_path():
    return load().gspc_last_path()


def gspc_last_kernel():
    return load().gspc_last_kernel().decode()


class LayerChain:
    """Marshalled form of a list of workloads.Layer: C layer array, buffer table."""

    def __init__(self, layers, packed, buffers):
        """layers: list of workloads.Layer; packed: PackedWeights indexed by
        Layer.wid; buffers: CUDA tensors indexed by the layers' src/src2/dst."""
        ops = {"conv": OP_CONV, "maxpool": OP_MAXPOOL, "add": OP_ADD, "relu": OP_RELU}
        self.n_layers = len(layers)
        self.layers = (GspcLayer * self.n_layers)()
        for k, l in enumerate(layers):
            g = self.layers[k]
            g.op, g.src, g.src2, g.dst = ops[l.op], l.src, l.src2, l.dst
            g.N, g.Cin, g.H, g.W, g.Cout = l.N, l.Cin, l.H, l.W, l.Cout
            g.KH, g.KW, g.stride, g.pad, g.groups = l.KH, l.KW, l.stride, l.pad, l.groups
            g.flags = FLAG_RELU if l.relu else 0
            g.w = packed[l.wid].handle.value if l.op == "conv" else None
        self.keep = (packed, buffers)
        self.n_bufs = len(buffers)
        self.bufs = (ctypes.c_void_p * self.n_bufs)(*[b.data_ptr() for b in buffers])
        self.bytes = (ctypes.c_size_t * self.n_bufs)(*[b.numel() * b.element_size() for b in buffers])


def gspc_run_layer_chain(lc, per_layer_ms=False):
    ms = (ctypes.c_float * lc.n_layers)() if per_layer_ms else None
    _check(load().gspc_run_layer_chain(lc.layers, lc.n_layers, lc.bufs, lc.bytes, lc.n_bufs, ms))
    return list(ms) if per_layer_ms else None
