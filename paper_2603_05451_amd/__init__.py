"""MI355X-native fused attention (forward + backward): thin Python binding of libattn.so.

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI
declared in include/attn.h.  PyTorch supplies device memory and streams.  There is no CPU
or eager fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn.so")
_lib = None

ATTN_OK, ATTN_EINVAL, ATTN_EUNSUPPORTED, ATTN_ELAUNCH = 0, -1, -2, -3


class AttnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libattn error {code}: {text}")
        self.code = code


def lib():
    """Load libattn.so (built in-tree by build.py); fail loudly when it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2603_05451_amd.build` "
                              "(hipcc --offload-arch=gfx950); there is no fallback path")
        # PyTorch ships its own HIP runtime (same SONAME as the system one).  Load torch first
        # so that libattn.so binds to the runtime that owns torch's streams and allocations;
        # two HIP runtimes in one process cannot launch on each other's streams.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.attn_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
        L.attn_fwd.restype = i
        L.attn_fwd_ex.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, vp]
        L.attn_fwd_ex.restype = i
        L.attn_bwd.argtypes = [vp] * 9 + [i, i, i, i, i, f, i, vp, sz, vp]
        L.attn_bwd.restype = i
        L.attn_bwd_ex.argtypes = [vp] * 9 + [i, i, i, i, i, i, f, i, vp, sz, vp]
        L.attn_bwd_ex.restype = i
        L.attn_bwd_phases.argtypes = [vp] * 9 + [i, i, i, i, i, i, f, i, vp, sz, vp, i]
        L.attn_bwd_phases.restype = i
        L.attn_bwd_noalloc.argtypes = [vp] * 9 + [i, i, i, i, i, i, f, i, vp]
        L.attn_bwd_noalloc.restype = i
        L.attn_bwd_workspace_bytes.argtypes = [i] * 6
        L.attn_bwd_workspace_bytes.restype = sz
        L.attn_fwd_dtype.argtypes = [i, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, vp]
        L.attn_fwd_dtype.restype = i
        L.attn_bwd_dtype.argtypes = [i] + [vp] * 9 + [i, i, i, i, i, i, f, i, vp, sz, vp]
        L.attn_bwd_dtype.restype = i
        L.attn_varlen_fwd_dtype.argtypes = [i] + [vp] * 7 + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_varlen_fwd_dtype.restype = i
        L.attn_varlen_bwd_dtype.argtypes = [i] + [vp] * 11 + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_varlen_bwd_dtype.restype = i
        L.attn_varlen_workspace_bytes.argtypes = [i] * 8
        L.attn_varlen_workspace_bytes.restype = sz
        sp = ctypes.POINTER(AttnStrides)
        L.attn_strided_workspace_bytes.argtypes = [i] * 8
        L.attn_strided_workspace_bytes.restype = sz
        L.attn_fwd_strided.argtypes = [i] + [vp, sp] * 4 + [vp] + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_fwd_strided.restype = i
        L.attn_bwd_strided.argtypes = [i] + [vp, sp] * 5 + [vp] + [vp, sp] * 3 + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_bwd_strided.restype = i
        L.attn_varlen_plan.argtypes = [vp, vp] + [i] * 7 + [vp, sz, vp]
        L.attn_varlen_plan.restype = i
        L.attn_varlen_fwd.argtypes = [vp] * 7 + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_varlen_fwd.restype = i
        L.attn_varlen_bwd.argtypes = [vp] * 11 + [i] * 7 + [f, i, vp, sz, vp]
        L.attn_varlen_bwd.restype = i
        L.attn_exp2_emulated.argtypes = [vp, vp, sz, i, vp]
        L.attn_exp2_emulated.restype = i
        L.attn_strerror.argtypes = [i]
        L.attn_strerror.restype = ctypes.c_char_p
        L.attn_version.restype = i
        _lib = L
    return _lib


def attn_strerror(code: int) -> str:
    return lib().attn_strerror(int(code)).decode()


def attn_version() -> int:
    return int(lib().attn_version())


def _check(rc: int):
    if rc != ATTN_OK:
        raise AttnError(rc, attn_strerror(rc))


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


ATTN_BF16, ATTN_F16 = 0, 1


def _dtype_code(t):
    """ATTN_BF16 / ATTN_F16 for a tensor's element type."""
    import torch
    if t.dtype == torch.bfloat16:
        return ATTN_BF16
    if t.dtype == torch.float16:
        return ATTN_F16
    raise ValueError(f"unsupported element type {t.dtype}: bf16 or fp16")


def _dev_bf16(t, name, shape=None, like=None):
    """Device pointer of a contiguous 16-bit CUDA tensor (bf16, or the element type of `like`)."""
    import torch
    want = torch.bfloat16 if like is None else like.dtype
    if not (t.is_cuda and t.dtype == want and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous {want} CUDA tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return ctypes.c_void_p(t.data_ptr())


def attn_bwd_workspace_bytes(B, H, Hkv, N, d_qk, d_v) -> int:
    return int(lib().attn_bwd_workspace_bytes(B, H, Hkv, N, d_qk, d_v))


def attn_fwd(q, k, v, scale, causal, o=None, lse=None, stream=None):
    """q [B,N,H,d_qk], k [B,N,Hkv,d_qk], v [B,N,Hkv,d_v] bf16 (or all fp16) on the GPU ->
    (o [B,N,H,d_v] of the same type, lse [B,H,N] fp32).  Outputs are allocated with torch unless
    passed in."""
    import torch
    B, N, H, dqk = q.shape
    Hkv, dv = k.shape[2], v.shape[3]
    code = _dtype_code(q)
    if o is None:
        o = torch.empty((B, N, H, dv), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and
            tuple(lse.shape) == (B, H, N)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [B,H,N]")
    args = (_dev_bf16(q, "q", like=q), _dev_bf16(k, "k", (B, N, Hkv, dqk), q),
            _dev_bf16(v, "v", (B, N, Hkv, dv), q), _dev_bf16(o, "o", (B, N, H, dv), q),
            ctypes.c_void_p(lse.data_ptr()), B, H, Hkv, N, dqk, dv,
            float(scale), int(bool(causal)), _stream(stream))
    rc = lib().attn_fwd_ex(*args) if code == ATTN_BF16 else lib().attn_fwd_dtype(code, *args)
    _check(rc)
    return o, lse


def attn_varlen_workspace_bytes(B, total_q, total_k, H, Hkv, d_qk, d_v, backward) -> int:
    return int(lib().attn_varlen_workspace_bytes(B, total_q, total_k, H, Hkv, d_qk, d_v, int(bool(backward))))


def attn_varlen_plan(cu_seqlens, total_q, total_k, H, Hkv, d_qk, d_v, workspace, cu_seqlens_k=None, stream=None):
    """Fills the tile tables of a backward-sized workspace once; later attn_varlen_fwd / attn_varlen_bwd
    calls on it may pass cu_seqlens=None and B=<number of sequences> to reuse them."""
    B = cu_seqlens.numel() - 1
    if cu_seqlens_k is None:
        cu_seqlens_k = cu_seqlens
    _check(lib().attn_varlen_plan(_dev_cu(cu_seqlens, B), _dev_cu(cu_seqlens_k, B, "cu_seqlens_k"), B, total_q, total_k,
                                  H, Hkv, d_qk, d_v, ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                  _stream(stream)))


def _dev_cu(cu, B, name="cu_seqlens"):
    import torch
    if cu is None:
        return None
    if not (cu.is_cuda and cu.dtype == torch.int32 and cu.is_contiguous() and tuple(cu.shape) == (B + 1,)):
        raise ValueError(f"{name} must be a contiguous int32 CUDA tensor [B+1]")
    return ctypes.c_void_p(cu.data_ptr())


def attn_varlen_fwd(q, k, v, cu_seqlens, scale, causal, o=None, lse=None, workspace=None, stream=None,
                    cu_seqlens_k=None, B=None):
    """Packed variable-length batch: q [Tq,H,d_qk], k [Tk,Hkv,d_qk], v [Tk,Hkv,d_v] bf16 (or all fp16),
    cu_seqlens [B+1] int32 (query rows; also the key rows unless cu_seqlens_k is given), all on the
    GPU -> (o [Tq,H,d_v], lse [H,Tq] fp32)."""
    import torch
    T, H, dqk = q.shape
    Tk, Hkv, dv = k.shape[0], k.shape[1], v.shape[2]
    if cu_seqlens is None:       # tables kept in `workspace` by attn_varlen_plan or an earlier call
        if B is None or workspace is None:
            raise ValueError("cu_seqlens=None needs B and the workspace that holds the tables")
    else:
        B = cu_seqlens.numel() - 1
        if cu_seqlens_k is None:
            cu_seqlens_k = cu_seqlens
    if o is None:
        o = torch.empty((T, H, dv), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((H, T), dtype=torch.float32, device=q.device)
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and tuple(lse.shape) == (H, T)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [H,Tq]")
    need = attn_varlen_workspace_bytes(B, T, Tk, H, Hkv, dqk, dv, False)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    code = _dtype_code(q)
    args = (_dev_bf16(q, "q", like=q), _dev_bf16(k, "k", (Tk, Hkv, dqk), q), _dev_bf16(v, "v", (Tk, Hkv, dv), q),
            _dev_bf16(o, "o", (T, H, dv), q), ctypes.c_void_p(lse.data_ptr()), _dev_cu(cu_seqlens, B),
            _dev_cu(cu_seqlens_k, B, "cu_seqlens_k"), B, T, Tk, H, Hkv, dqk, dv, float(scale), int(bool(causal)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream))
    rc = lib().attn_varlen_fwd(*args) if code == ATTN_BF16 else lib().attn_varlen_fwd_dtype(code, *args)
    _check(rc)
    return o, lse


def attn_varlen_bwd(q, k, v, o, d_o, lse, cu_seqlens, scale, causal, dq=None, dk=None, dv=None, workspace=None,
                    stream=None, cu_seqlens_k=None, B=None):
    """Backward of attn_varlen_fwd: returns (dq [Tq,H,d_qk], dk [Tk,Hkv,d_qk], dv [Tk,Hkv,d_v])."""
    import torch
    T, H, dqk = q.shape
    Tk, Hkv, dv_ = k.shape[0], k.shape[1], v.shape[2]
    if cu_seqlens is None:       # tables kept in `workspace` by attn_varlen_plan or an earlier backward call
        if B is None or workspace is None:
            raise ValueError("cu_seqlens=None needs B and the workspace that holds the tables")
    else:
        B = cu_seqlens.numel() - 1
        if cu_seqlens_k is None:
            cu_seqlens_k = cu_seqlens
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = attn_varlen_workspace_bytes(B, T, Tk, H, Hkv, dqk, dv_, True)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and tuple(lse.shape) == (H, T)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [H,Tq]")
    code = _dtype_code(q)
    args = (_dev_bf16(q, "q", like=q), _dev_bf16(k, "k", (Tk, Hkv, dqk), q), _dev_bf16(v, "v", (Tk, Hkv, dv_), q),
            _dev_bf16(o, "o", (T, H, dv_), q), _dev_bf16(d_o, "d_o", (T, H, dv_), q),
            ctypes.c_void_p(lse.data_ptr()), _dev_bf16(dq, "dq", (T, H, dqk), q),
            _dev_bf16(dk, "dk", (Tk, Hkv, dqk), q), _dev_bf16(dv, "dv", (Tk, Hkv, dv_), q),
            _dev_cu(cu_seqlens, B), _dev_cu(cu_seqlens_k, B, "cu_seqlens_k"), B, T, Tk, H, Hkv, dqk, dv_,
            float(scale), int(bool(causal)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream))
    rc = lib().attn_varlen_bwd(*args) if code == ATTN_BF16 else lib().attn_varlen_bwd_dtype(code, *args)
    _check(rc)
    return dq, dk, dv


class AttnStrides(ctypes.Structure):
    """attn_strides_t of include/attn.h: element strides of the batch, token and head axes."""
    _fields_ = [("batch", ctypes.c_longlong), ("row", ctypes.c_longlong), ("head", ctypes.c_longlong)]


def _view(t, name, shape, like):
    """(pointer, strides) of a [B, N, heads, d] view with a contiguous head dim."""
    if not (t.is_cuda and t.dtype == like.dtype and t.dim() == 4 and (t.stride(3) == 1 or t.shape[3] == 1)):
        raise ValueError(f"{name} must be a 4-d {like.dtype} CUDA tensor with a contiguous last axis")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return ctypes.c_void_p(t.data_ptr()), ctypes.byref(AttnStrides(t.stride(0), t.stride(1), t.stride(2)))


def attn_strided_workspace_bytes(B, H, Hkv, Nq, Nk, d_qk, d_v, backward) -> int:
    return int(lib().attn_strided_workspace_bytes(B, H, Hkv, Nq, Nk, d_qk, d_v, int(bool(backward))))


def attn_fwd_strided(q, k, v, scale, causal, o=None, lse=None, workspace=None, stream=None):
    """attn_fwd on views: q [B,Nq,H,d_qk], k [B,Nk,Hkv,d_qk], v [B,Nk,Hkv,d_v] of any strides (the
    last axis contiguous), e.g. x.permute(0, 2, 1, 3) of a [B,H,N,d] tensor; any Nq, Nk >= 1 (under a
    causal mask the last query sees the last key, Nk >= Nq).  o may be a view too (default: a new
    contiguous [B,Nq,H,d_v]); lse [B,H,Nq] fp32 contiguous."""
    import torch
    B, N, H, dqk = q.shape
    Nk, Hkv, dv = k.shape[1], k.shape[2], v.shape[3]
    if o is None:
        o = torch.empty((B, N, H, dv), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and tuple(lse.shape) == (B, H, N)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [B,H,Nq]")
    need = attn_strided_workspace_bytes(B, H, Hkv, N, Nk, dqk, dv, False)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    rc = lib().attn_fwd_strided(_dtype_code(q), *_view(q, "q", (B, N, H, dqk), q), *_view(k, "k", (B, Nk, Hkv, dqk), q),
                                *_view(v, "v", (B, Nk, Hkv, dv), q), *_view(o, "o", (B, N, H, dv), q),
                                ctypes.c_void_p(lse.data_ptr()), B, H, Hkv, N, Nk, dqk, dv, float(scale),
                                int(bool(causal)), ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                _stream(stream))
    _check(rc)
    return o, lse


def attn_bwd_strided(q, k, v, o, d_o, lse, scale, causal, dq=None, dk=None, dv=None, workspace=None, stream=None):
    """Backward of attn_fwd_strided; every tensor may be a view.  Gradients default to new
    contiguous tensors shaped like q, k and v."""
    import torch
    B, N, H, dqk = q.shape
    Nk, Hkv, dv_ = k.shape[1], k.shape[2], v.shape[3]
    dq = torch.empty((B, N, H, dqk), dtype=q.dtype, device=q.device) if dq is None else dq
    dk = torch.empty((B, Nk, Hkv, dqk), dtype=q.dtype, device=q.device) if dk is None else dk
    dv = torch.empty((B, Nk, Hkv, dv_), dtype=q.dtype, device=q.device) if dv is None else dv
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and tuple(lse.shape) == (B, H, N)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [B,H,Nq]")
    need = attn_strided_workspace_bytes(B, H, Hkv, N, Nk, dqk, dv_, True)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    rc = lib().attn_bwd_strided(_dtype_code(q), *_view(q, "q", (B, N, H, dqk), q), *_view(k, "k", (B, Nk, Hkv, dqk), q),
                                *_view(v, "v", (B, Nk, Hkv, dv_), q), *_view(o, "o", (B, N, H, dv_), q),
                                *_view(d_o, "d_o", (B, N, H, dv_), q), ctypes.c_void_p(lse.data_ptr()),
                                *_view(dq, "dq", (B, N, H, dqk), q), *_view(dk, "dk", (B, Nk, Hkv, dqk), q),
                                *_view(dv, "dv", (B, Nk, Hkv, dv_), q), B, H, Hkv, N, Nk, dqk, dv_, float(scale),
                                int(bool(causal)), ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                _stream(stream))
    _check(rc)
    return dq, dk, dv


def attn_exp2_emulated(x, degree, y=None, stream=None):
    """y = 2^x elementwise on the GPU: polynomial emulation of degree 3/4/5, or 0 = v_exp_f32."""
    import torch
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()):
        raise ValueError("x must be a contiguous fp32 CUDA tensor")
    y = torch.empty_like(x) if y is None else y
    _check(lib().attn_exp2_emulated(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(y.data_ptr()),
                                    x.numel(), int(degree), _stream(stream)))
    return y


ATTN_BWD_PREPARE, ATTN_BWD_DKDV, ATTN_BWD_DQ, ATTN_BWD_ALL = 1, 2, 4, 7


def attn_bwd(q, k, v, o, do, lse, scale, causal, dq=None, dk=None, dv=None, workspace=None,
             stream=None, phases=ATTN_BWD_ALL):
    """Gradients dq, dk, dv (bf16, layouts of q, k, v) from do, the forward's o and lse.
    phases != ATTN_BWD_ALL maps to attn_bwd_phases (per-kernel timing only)."""
    import torch
    B, N, H, dqk = q.shape
    Hkv, dvd = k.shape[2], v.shape[3]
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = attn_bwd_workspace_bytes(B, H, Hkv, N, dqk, dvd)
    if need == 0:
        _check(lib().attn_bwd_ex(*([None] * 9), B, H, Hkv, N, dqk, dvd, float(scale), 0, None, 0, None)
               or ATTN_EINVAL)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    code = _dtype_code(q)
    args = (_dev_bf16(q, "q", like=q), _dev_bf16(k, "k", (B, N, Hkv, dqk), q),
            _dev_bf16(v, "v", (B, N, Hkv, dvd), q), _dev_bf16(o, "o", (B, N, H, dvd), q),
            _dev_bf16(do, "do", (B, N, H, dvd), q), ctypes.c_void_p(lse.data_ptr()),
            _dev_bf16(dq, "dq", q.shape, q), _dev_bf16(dk, "dk", k.shape, q),
            _dev_bf16(dv, "dv", v.shape, q), B, H, Hkv, N, dqk, dvd, float(scale),
            int(bool(causal)), ctypes.c_void_p(workspace.data_ptr()),
            workspace.numel() * workspace.element_size(), _stream(stream))
    if code == ATTN_BF16:
        rc = lib().attn_bwd_phases(*args, int(phases))
    elif phases == ATTN_BWD_ALL:
        rc = lib().attn_bwd_dtype(code, *args)
    else:
        raise ValueError("per-kernel phases are exposed for bf16 only")
    _check(rc)
    return dq, dk, dv


ATTN_NOALLOC_MAX_ROWS = 1 << 20


def attn_bwd_noalloc(q, k, v, o, do, lse, scale, causal, dq, dk, dv, stream=None):
    """attn_bwd with the library's built-in workspace (bf16; B * H * N <= ATTN_NOALLOC_MAX_ROWS).
    The caller passes every output: nothing is allocated, here or in the library."""
    B, N, H, dqk = q.shape
    Hkv, dvd = k.shape[2], v.shape[3]
    if _dtype_code(q) != ATTN_BF16:
        raise ValueError("attn_bwd_noalloc takes bf16 tensors")
    _check(lib().attn_bwd_noalloc(_dev_bf16(q, "q", like=q), _dev_bf16(k, "k", (B, N, Hkv, dqk), q),
                                  _dev_bf16(v, "v", (B, N, Hkv, dvd), q), _dev_bf16(o, "o", (B, N, H, dvd), q),
                                  _dev_bf16(do, "do", (B, N, H, dvd), q), ctypes.c_void_p(lse.data_ptr()),
                                  _dev_bf16(dq, "dq", q.shape, q), _dev_bf16(dk, "dk", k.shape, q),
                                  _dev_bf16(dv, "dv", v.shape, q), B, H, Hkv, N, dqk, dvd, float(scale),
                                  int(bool(causal)), _stream(stream)))
    return dq, dk, dv
