"""Shared test helpers: error metric, oracle-side chain executor, GPU plumbing."""
import numpy as np

import oracle
from paper_2006_09791_amd import workloads as wl

TOL_F32 = 1e-4      # fp32 path vs fp64 oracle (max relative error)
TOL_BF16 = 2e-2     # bf16 inputs / weights vs fp64 oracle on un-rounded data


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): element-wise relative error with
    the denominator floored at the tensor's RMS, so outputs that happen to be
    near zero do not blow the ratio up."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref))
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def err_metrics(got, ref, absum=None):
    """The error of a tensor three ways: 'floored' is rel_err (the metric the tolerances are stated in),
    'scaled' = max|g - r| / max|r|, and, when the oracle's sum |x*w| per output is given, 'bound' =
    max_i |g_i - r_i| / A_i, the quantity the textbook bound |fl(s) - s| <= gamma_K * A speaks about."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    out = {"floored": rel_err(got, ref), "scaled": 0.0}
    if ref.size:
        out["scaled"] = float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))
    if absum is not None and ref.size:
        out["bound"] = float(np.max(np.abs(got - ref) / np.maximum(np.asarray(absum, dtype=np.float64), 1e-30)))
    return out


def oracle_chain(chain, x0, weights, threads=8):
    """Runs a workloads.Chain with the CPU oracle, all in float64."""
    return oracle.run_chain(chain.layers, len(chain.buf_elems), x0, weights, threads=threads)


_side_stream = None


def side_stream():
    """A non-default torch stream (default priority): layer chains are only
    recorded into HIP graphs on a stream other than the null stream."""
    global _side_stream
    import torch
    if _side_stream is None:
        _side_stream = torch.cuda.Stream()
    return _side_stream


def gpu_chain(chain, x0, weights, dtype=None):
    """Packs weights, allocates buffers and returns (LayerChain, buffers).
    Setup runs on torch's current stream and is synchronised before return."""
    import torch
    from paper_2006_09791_amd import binding as b
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), g, dtype or b.GSPC_F32)
              for w, g in zip(weights, chain.weight_groups)]
    bufs = [torch.empty(max(n, 1), dtype=torch.float32, device=dev) for n in chain.buf_elems]
    bufs[0].copy_(torch.from_numpy(np.ascontiguousarray(x0, dtype=np.float32)).reshape(-1))
    torch.cuda.synchronize()
    return b.LayerChain(chain.layers, packed, bufs), bufs
