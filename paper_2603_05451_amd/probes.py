"""Thin Python binding of libattn_probes.so (include/attn_probes.h): measurement probes, a library
of their own next to the attention library.  Argument marshalling only; tests and profiles call it."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_probes.so")
_lib = None

ATTN_EXP2_RATE_BLOCKS = 2048
ATTN_MFMA_RATE_BLOCKS = 256
ATTN_LDS_RATE_BLOCKS = 512
ATTN_PROBE_WAVE_ISSUE_BLOCKS = 256


class ProbeError(RuntimeError):
    pass


def lib():
    """Load libattn_probes.so (built in-tree by build.py); fail loudly when it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2603_05451_amd.build`")
        import torch  # noqa: F401  (the HIP runtime that owns torch's streams must be loaded first)
        L = ctypes.CDLL(LIB_PATH)
        vp, i, ll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        for name in ("attn_exp2_rate", "attn_exp2_rate_partial", "attn_mfma_rate", "attn_lds_rate"):
            getattr(L, name).argtypes = [vp, i, i, vp]
            getattr(L, name).restype = ll
        L.attn_probe_wave_issue_configs.restype = i
        L.attn_probe_wave_issue.argtypes = [i, ctypes.POINTER(i), vp, vp, i, vp]
        L.attn_probe_wave_issue.restype = ll
        _lib = L
    return _lib


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _enqueue(name, out_elems, a, b, out, stream):
    import torch
    if out is None:
        out = torch.empty(out_elems, dtype=torch.float32, device="cuda")
    n = getattr(lib(), name)(ctypes.c_void_p(out.data_ptr()), int(a), int(b), _stream(stream))
    if n <= 0:
        raise ProbeError(f"{name} returned {n}")
    return int(n), out


def attn_exp2_rate(degree, iters, out=None, stream=None):
    """Enqueue the pure-ALU exp2 throughput kernel; returns (number of evaluations, out tensor)."""
    return _enqueue("attn_exp2_rate", ATTN_EXP2_RATE_BLOCKS * 256, degree, iters, out, stream)


def attn_exp2_rate_partial(emulated_of_8, iters, out=None, stream=None):
    """attn_exp2_rate with emulated_of_8 of every 8 evaluations on the degree-3 polynomial and the
    rest on the hardware instruction; returns (number of evaluations, out tensor)."""
    return _enqueue("attn_exp2_rate_partial", ATTN_EXP2_RATE_BLOCKS * 256, emulated_of_8, iters, out, stream)


def attn_mfma_rate(random_operands, iters, out=None, stream=None):
    """Enqueue the pure-MFMA ceiling kernel; returns (FLOPs enqueued, out tensor)."""
    return _enqueue("attn_mfma_rate", ATTN_MFMA_RATE_BLOCKS * 512, bool(random_operands), iters, out, stream)


def attn_lds_rate(pattern, iters, out=None, stream=None):
    """Enqueue the LDS read-rate kernel (pattern 0: ds_read_b128 A-operand fragments, 1: transposing
    reads); returns (bytes read from LDS, out tensor)."""
    return _enqueue("attn_lds_rate", ATTN_LDS_RATE_BLOCKS * 256, pattern, iters, out, stream)


def wave_issue_configs():
    """(nv, nb, ntr, dma, ring) of every built variant of the single-wave issue probe."""
    L = lib()
    res = []
    for c in range(L.attn_probe_wave_issue_configs()):
        d = (ctypes.c_int * 5)()
        L.attn_probe_wave_issue(c, d, None, None, 0, None)
        res.append(tuple(d))
    return res


def wave_issue(config, iters, stream=None):
    """Run variant `config` of the single-wave issue probe to completion; returns (shader cycles per
    step, shader clock in MHz, TFLOP/s of the whole chip by HIP events)."""
    import torch
    out = torch.zeros(ATTN_PROBE_WAVE_ISSUE_BLOCKS * 256, dtype=torch.float32, device="cuda")
    clk = torch.zeros(2, dtype=torch.int64, device="cuda")
    call = lambda n: lib().attn_probe_wave_issue(int(config), None, ctypes.c_void_p(out.data_ptr()),
                                                 ctypes.c_void_p(clk.data_ptr()), int(n), _stream(stream))
    if call(100) <= 0:
        raise ProbeError("attn_probe_wave_issue failed")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    steps = call(iters)
    e1.record()
    torch.cuda.synchronize()
    if steps <= 0:
        raise ProbeError("attn_probe_wave_issue failed")
    cyc, ticks = (int(t) for t in clk.cpu())
    flops = ATTN_PROBE_WAVE_ISSUE_BLOCKS * 4 * steps * 2.0 * 32 * 32 * 16
    return cyc / steps, cyc / (ticks / 100.0), flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
