"""CPU oracle for grouped convolution: numpy-facing wrappers over liboracle.so.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg; never by the GPU library or its binding.  All
arrays are float64, C-contiguous; fp32 / bf16 data is widened by the caller.

Passages followed (arXiv 2006.09791): grouped convolution G(g) as defined in
Section II / Fig. 2; shapes and the four GSPC stages of Section III-B and
Algorithm 1; MAC count of Eq. 2 (Section IV-B).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None
_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.c_int


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if (not os.path.exists(path)
            or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
        path = _build.build()
    lib = ctypes.CDLL(path)
    lib.oracle_out_dim.restype = _I
    lib.oracle_out_dim.argtypes = [_I] * 4
    lib.oracle_macs.restype = ctypes.c_uint64
    lib.oracle_macs.argtypes = [_I] * 8
    lib.oracle_conv2d_grouped.restype = _I
    lib.oracle_conv2d_grouped.argtypes = (
        [_D, _D] + [_I] * 10 + [_D, _D, ctypes.POINTER(ctypes.c_uint64), _I])
    lib.oracle_conv2d_grouped_channels.restype = _I
    lib.oracle_conv2d_grouped_channels.argtypes = (
        [_D, _D] + [_I] * 10 + [ctypes.POINTER(_I), _I, _D, _I])
    lib.oracle_conv2d_standard.restype = _I
    lib.oracle_conv2d_standard.argtypes = [_D, _D] + [_I] * 9 + [_D]
    lib.oracle_alg1_pack_kernels.restype = _I
    lib.oracle_alg1_pack_kernels.argtypes = [_D] + [_I] * 7 + [_D]
    lib.oracle_alg1_pack_inputs.restype = _I
    lib.oracle_alg1_pack_inputs.argtypes = [_D] + [_I] * 7 + [_D]
    lib.oracle_alg1_conv.restype = _I
    lib.oracle_alg1_conv.argtypes = [_D, _D] + [_I] * 12 + [_D]
    lib.oracle_alg1_conv_vec.restype = _I
    lib.oracle_alg1_conv_vec.argtypes = [_D, _D] + [_I] * 12 + [_D, _I]
    lib.oracle_alg1_unpack_outputs.restype = _I
    lib.oracle_alg1_unpack_outputs.argtypes = [_D] + [_I] * 6 + [_D]
    lib.oracle_relu.restype = None
    lib.oracle_relu.argtypes = [_D, ctypes.c_size_t, _D]
    lib.oracle_add.restype = None
    lib.oracle_add.argtypes = [_D, _D, ctypes.c_size_t, _D]
    lib.oracle_maxpool2d.restype = _I
    lib.oracle_maxpool2d.argtypes = [_D] + [_I] * 7 + [_D]
    lib.oracle_max_threads.restype = _I
    lib.oracle_max_threads.argtypes = []
    _lib = lib
    return lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(_D)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle.{what}: invalid arguments (rc={rc})")


def out_dim(size, k, stride, pad):
    return int(_load().oracle_out_dim(size, k, stride, pad))


def macs(N, Cin, Cout, KH, KW, Hout, Wout, groups):
    """Eq. 2."""
    return int(_load().oracle_macs(N, Cin, Cout, KH, KW, Hout, Wout, groups))


def max_threads():
    return int(_load().oracle_max_threads())


def conv2d_grouped(x, w, stride=1, pad=0, groups=1, *, return_abs=False,
                   return_macs=False, threads=1):
    """Definition of G(g): x [N,Cin,H,W], w [Cout,Cin/g,KH,KW] -> y float64."""
    x, w = _f64(x), _f64(w)
    N, Cin, H, W = x.shape
    Cout, cpg, KH, KW = w.shape
    if groups <= 0 or Cin % groups or cpg != Cin // groups:
        raise ValueError("weight shape does not match Cin/groups")
    Ho, Wo = out_dim(H, KH, stride, pad), out_dim(W, KW, stride, pad)
    y = np.empty((N, Cout, max(Ho, 0), max(Wo, 0)), dtype=np.float64)
    a = np.empty_like(y) if return_abs else None
    cnt = ctypes.c_uint64(0)
    rc = _load().oracle_conv2d_grouped(
        _p(x), _p(w), N, Cin, H, W, Cout, KH, KW, stride, pad, groups, _p(y),
        _p(a) if a is not None else None, ctypes.byref(cnt), threads)
    _check(rc, "conv2d_grouped")
    out = (y,)
    if return_abs:
        out += (a,)
    if return_macs:
        out += (int(cnt.value),)
    return out[0] if len(out) == 1 else out


def conv2d_grouped_channels(x, w, oc_sel, stride=1, pad=0, groups=1, threads=1):
    """conv2d_grouped restricted to the output channels listed in oc_sel."""
    x, w = _f64(x), _f64(w)
    N, Cin, H, W = x.shape
    Cout, cpg, KH, KW = w.shape
    if groups <= 0 or Cin % groups or cpg != Cin // groups:
        raise ValueError("weight shape does not match Cin/groups")
    sel = np.ascontiguousarray(oc_sel, dtype=np.int32)
    Ho, Wo = out_dim(H, KH, stride, pad), out_dim(W, KW, stride, pad)
    y = np.empty((N, len(sel), Ho, Wo), dtype=np.float64)
    rc = _load().oracle_conv2d_grouped_channels(
        _p(x), _p(w), N, Cin, H, W, Cout, KH, KW, stride, pad, groups,
        sel.ctypes.data_as(ctypes.POINTER(_I)), len(sel), _p(y), threads)
    _check(rc, "conv2d_grouped_channels")
    return y


def conv2d_standard(x, w, stride=1, pad=0):
    """Standard convolution S, no group logic: w [Cout,Cin,KH,KW]."""
    x, w = _f64(x), _f64(w)
    N, Cin, H, W = x.shape
    Cout, cin2, KH, KW = w.shape
    if cin2 != Cin:
        raise ValueError("standard conv needs w.shape[1] == Cin")
    Ho, Wo = out_dim(H, KH, stride, pad), out_dim(W, KW, stride, pad)
    y = np.empty((N, Cout, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_conv2d_standard(_p(x), _p(w), N, Cin, H, W, Cout, KH,
                                        KW, stride, pad, _p(y))
    _check(rc, "conv2d_standard")
    return y


def alg1_pack_kernels(w, groups, T_I, T_O):
    """Algorithm 1 stage 1 -> W' [g, KPG/T_O, CPG/T_I, KH, KW, T_I, T_O]."""
    w = _f64(w)
    Cout, CPG, KH, KW = w.shape
    Cin = CPG * groups
    KPG = Cout // groups
    wp = np.empty((groups, KPG // max(T_O, 1), CPG // max(T_I, 1), KH, KW, T_I,
                   T_O), dtype=np.float64)
    rc = _load().oracle_alg1_pack_kernels(_p(w), Cin, Cout, KH, KW, groups,
                                          T_I, T_O, _p(wp))
    _check(rc, "alg1_pack_kernels")
    return wp


def alg1_pack_inputs(x, pad, groups, T_I):
    """Algorithm 1 stage 2 -> X' [g, N, CPG/T_I, H+2p, T_I, W+2p]."""
    x = _f64(x)
    N, Cin, H, W = x.shape
    CPG = Cin // groups
    xp = np.empty((groups, N, CPG // max(T_I, 1), H + 2 * pad, T_I,
                   W + 2 * pad), dtype=np.float64)
    rc = _load().oracle_alg1_pack_inputs(_p(x), N, Cin, H, W, pad, groups, T_I,
                                         _p(xp))
    _check(rc, "alg1_pack_inputs")
    return xp


def alg1_conv(xp, wp, N, Cin, H, W, Cout, KH, KW, stride, pad, groups, T_I,
              T_O, vectorised=False, threads=1):
    """Algorithm 1 stage 3 -> Y' [g, N, KPG/T_O, Hout, Wout, T_O].  vectorised:
    the CPU schedule of Sections III-B / III-C (T_O filters as one vector,
    (group, image) pairs over `threads` cores), a timed baseline with the same
    bits as the plain form."""
    xp, wp = _f64(xp), _f64(wp)
    KPG = Cout // groups
    Ho, Wo = out_dim(H, KH, stride, pad), out_dim(W, KW, stride, pad)
    yp = np.empty((groups, N, KPG // T_O, Ho, Wo, T_O), dtype=np.float64)
    if vectorised:
        rc = _load().oracle_alg1_conv_vec(_p(xp), _p(wp), N, Cin, H, W, Cout, KH, KW,
                                          stride, pad, groups, T_I, T_O, _p(yp), threads)
    else:
        rc = _load().oracle_alg1_conv(_p(xp), _p(wp), N, Cin, H, W, Cout, KH, KW,
                                      stride, pad, groups, T_I, T_O, _p(yp))
    _check(rc, "alg1_conv")
    return yp


def alg1_unpack_outputs(yp, Cout, groups, T_O):
    """Algorithm 1 stage 4 -> Y [N, Cout, Hout, Wout]."""
    yp = _f64(yp)
    _, N, _, Ho, Wo, _ = yp.shape
    y = np.empty((N, Cout, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_alg1_unpack_outputs(_p(yp), N, Cout, Ho, Wo, groups,
                                            T_O, _p(y))
    _check(rc, "alg1_unpack_outputs")
    return y


def gspc_alg1(x, w, stride, pad, groups, T_I, T_O, vectorised=False, threads=1, packed_w=None):
    """All four stages of Algorithm 1 in order (packed_w: a W' made ahead of time,
    as the paper does for inference)."""
    x, w = _f64(x), _f64(w)
    N, Cin, H, W = x.shape
    Cout, _, KH, KW = w.shape
    wp = packed_w if packed_w is not None else alg1_pack_kernels(w, groups, T_I, T_O)
    xp = alg1_pack_inputs(x, pad, groups, T_I)
    yp = alg1_conv(xp, wp, N, Cin, H, W, Cout, KH, KW, stride, pad, groups,
                   T_I, T_O, vectorised=vectorised, threads=threads)
    return alg1_unpack_outputs(yp, Cout, groups, T_O)


def relu(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_relu(_p(x), x.size, _p(y))
    return y


def add(a, b):
    a, b = _f64(a), _f64(b)
    if a.shape != b.shape:
        raise ValueError("add: shape mismatch")
    y = np.empty_like(a)
    _load().oracle_add(_p(a), _p(b), a.size, _p(y))
    return y


def maxpool2d(x, k=3, stride=2, pad=1):
    x = _f64(x)
    N, C, H, W = x.shape
    Ho, Wo = out_dim(H, k, stride, pad), out_dim(W, k, stride, pad)
    y = np.empty((N, C, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_maxpool2d(_p(x), N, C, H, W, k, stride, pad, _p(y))
    _check(rc, "maxpool2d")
    return y


def run_chain(layers, n_bufs, x0, weights, threads=1):
    """Executes a list of layer steps (objects with fields op, src, src2, dst,
    KH, stride, pad, groups, relu, wid) in float64.  A conv step adds buffer
    src2 (if >= 0) to its result and then applies the optional ReLU, like the
    residual blocks of the networks of Section IV-A.  Returns all buffers."""
    bufs = [None] * n_bufs
    bufs[0] = _f64(x0)
    for l in layers:
        if l.op == "conv":
            y = conv2d_grouped(bufs[l.src], weights[l.wid], l.stride, l.pad, l.groups,
                               threads=threads)
            if l.src2 >= 0:
                y = add(y, bufs[l.src2])
            if l.relu:
                y = relu(y)
        elif l.op == "maxpool":
            y = maxpool2d(bufs[l.src], l.KH, l.stride, l.pad)
        elif l.op == "add":
            y = add(bufs[l.src], bufs[l.src2])
            if l.relu:
                y = relu(y)
        elif l.op == "relu":
            y = relu(bufs[l.src])
        else:
            raise ValueError(f"unknown op {l.op}")
        bufs[l.dst] = y
    return bufs
