"""CPU fp64 oracle for attention forward/backward -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

`attn_oracle.c` holds the arithmetic (plain definitions of paper Sec. 2.1 and the
tiled recurrences of Sec. 3.1.4).  This module only builds it with gcc, loads it
with ctypes and marshals numpy fp64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile attn_oracle.c into liboracle.so next to it (gcc, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        i, d = ctypes.c_int, ctypes.c_double
        _lib.oracle_attn_fwd.argtypes = [dp, dp, dp, dp, dp, i, i, i, i, i, i, i, d, i, ip]
        _lib.oracle_attn_fwd.restype = i
        _lib.oracle_attn_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, i, i, i, i, i, i, i, d, i, ip]
        _lib.oracle_attn_bwd.restype = i
        _lib.oracle_attn_fwd_online.argtypes = [dp, dp, dp, dp, dp, ip, i, i, i, i, i, i, i, d, i, i, d]
        _lib.oracle_attn_fwd_online.restype = i
        _lib.oracle_num_threads.restype = i
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(q, k, v):
    B, Nq, H, dqk = q.shape
    Bk, Nk, Hkv, dk_ = k.shape
    Bv, Nv, Hv, dv = v.shape
    if not (B == Bk == Bv and Nk == Nv and Hkv == Hv and dqk == dk_):
        raise ValueError(f"inconsistent shapes q{q.shape} k{k.shape} v{v.shape}")
    return B, H, Hkv, Nq, Nk, dqk, dv


def _qpos(q_pos, Nq):
    if q_pos is None:
        return None, None
    a = np.ascontiguousarray(q_pos, dtype=np.int32)
    if a.shape != (Nq,):
        raise ValueError("q_pos must have one entry per query row")
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def attn_fwd(q, k, v, scale, causal, q_pos=None):
    """O [B,Nq,H,dv] and LSE [B,H,Nq] in fp64 from q [B,Nq,H,dqk], k [B,Nk,Hkv,dqk], v [B,Nk,Hkv,dv]."""
    lib = _load()
    q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    B, H, Hkv, Nq, Nk, dqk, dv = _shapes(q, k, v)
    o = np.empty((B, Nq, H, dv), np.float64)
    lse = np.empty((B, H, Nq), np.float64)
    keep, pp = _qpos(q_pos, Nq)
    rc = lib.oracle_attn_fwd(qp, kp, vp, o.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                             lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                             B, H, Hkv, Nq, Nk, dqk, dv, float(scale), int(bool(causal)), pp)
    if rc != 0:
        raise RuntimeError(f"oracle_attn_fwd failed with code {rc}")
    return o, lse


def attn_bwd(q, k, v, d_o, scale, causal, q_pos=None):
    """dQ, dK, dV in fp64 (layouts of q, k, v).  Recomputes P itself; takes neither O nor LSE."""
    lib = _load()
    q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v); d_o, dop = _f64(d_o)
    B, H, Hkv, Nq, Nk, dqk, dv = _shapes(q, k, v)
    if d_o.shape != (B, Nq, H, dv):
        raise ValueError("d_o must be [B,Nq,H,dv]")
    dq = np.empty_like(q); dk = np.empty_like(k); dvv = np.empty_like(v)
    P = ctypes.POINTER(ctypes.c_double)
    keep, pp = _qpos(q_pos, Nq)
    rc = lib.oracle_attn_bwd(qp, kp, vp, dop, dq.ctypes.data_as(P), dk.ctypes.data_as(P),
                             dvv.ctypes.data_as(P), B, H, Hkv, Nq, Nk, dqk, dv,
                             float(scale), int(bool(causal)), pp)
    if rc != 0:
        raise RuntimeError(f"oracle_attn_bwd failed with code {rc}")
    return dq, dk, dvv


def attn_fwd_online(q, k, v, scale, causal, tile, tau):
    """Tiled online softmax with thresholded rescaling (paper Sec. 3.1.4) in fp64.

    Returns O, LSE and the per-row count of rescales after the first block."""
    lib = _load()
    q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    B, H, Hkv, Nq, Nk, dqk, dv = _shapes(q, k, v)
    o = np.empty((B, Nq, H, dv), np.float64)
    lse = np.empty((B, H, Nq), np.float64)
    nres = np.zeros((B, H, Nq), np.int32)
    P = ctypes.POINTER(ctypes.c_double)
    rc = lib.oracle_attn_fwd_online(qp, kp, vp, o.ctypes.data_as(P), lse.ctypes.data_as(P),
                                    nres.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                    B, H, Hkv, Nq, Nk, dqk, dv, float(scale),
                                    int(bool(causal)), int(tile), float(tau))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_fwd_online failed with code {rc}")
    return o, lse, nres
