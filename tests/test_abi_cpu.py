"""CPU-only checks of the C ABI: the library loads, exports every function include/attn.h
declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2603_05451_amd as A
    if not os.path.exists(A.LIB_PATH):
        from paper_2603_05451_amd import build
        build.build_library()
    return A.lib()


def declared_functions(header="attn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert {"attn_fwd", "attn_fwd_ex", "attn_bwd", "attn_bwd_ex", "attn_bwd_phases",
            "attn_bwd_workspace_bytes", "attn_strerror", "attn_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"libattn.so does not export {n}"


def test_every_declared_probe_is_exported_by_the_probe_library_only(L):
    """include/attn_probes.h belongs to libattn_probes.so; the attention library ships none of it."""
    from paper_2603_05451_amd import probes
    if not os.path.exists(probes.LIB_PATH):
        from paper_2603_05451_amd import build
        build.build_library()
    P = probes.lib()
    names = declared_functions("attn_probes.h")
    assert {"attn_exp2_rate", "attn_mfma_rate", "attn_lds_rate", "attn_probe_wave_issue"} <= set(names)
    for n in names:
        assert hasattr(P, n), f"libattn_probes.so does not export {n}"
        assert not hasattr(L, n), f"libattn.so exports the probe {n}"
    assert probes.wave_issue_configs()[0] == (0, 0, 0, 0, 4)      # host-side table, no GPU needed


def test_version_and_error_strings(L):
    import paper_2603_05451_amd as A
    assert A.attn_version() >= 100
    for code in (0, -1, -2, -3, -99):
        assert isinstance(A.attn_strerror(code), str) and A.attn_strerror(code)


def test_workspace_size(L):
    import paper_2603_05451_amd as A
    # D and base-2 LSE: two fp32 [B,H,N] arrays, each rounded up to 256 bytes
    assert A.attn_bwd_workspace_bytes(2, 16, 16, 8192, 128, 128) == 2 * 2 * 16 * 8192 * 4
    assert A.attn_bwd_workspace_bytes(1, 2, 2, 128, 64, 64) == 2 * 1024
    assert A.attn_bwd_workspace_bytes(1, 3, 2, 128, 64, 64) == 0      # H % Hkv != 0
    assert A.attn_bwd_workspace_bytes(1, 2, 2, 100, 64, 64) == 0      # N not a multiple of 128
    assert A.attn_bwd_workspace_bytes(1, 2, 2, 128, 80, 80) == 0      # unsupported head dim


def test_forward_argument_validation(L):
    import paper_2603_05451_amd as A
    p = ctypes.c_void_p(0x1000)            # aligned, never dereferenced: validation fails first
    fwd = lambda *a: L.attn_fwd_ex(*a)
    assert fwd(None, p, p, p, p, 1, 2, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, None, 1, 2, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, p, 0, 2, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, p, 1, 3, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, p, 1, 2, 2, 128, 64, 64, 0.0, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, p, 1, 2, 2, 128, 64, 64, float("nan"), 0, None) == A.ATTN_EINVAL
    assert fwd(ctypes.c_void_p(0x1008), p, p, p, p, 1, 2, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EINVAL
    assert fwd(p, p, p, p, p, 1, 2, 2, 192, 64, 64, 0.125, 0, None) == A.ATTN_EUNSUPPORTED
    assert fwd(p, p, p, p, p, 1, 2, 2, 128, 128, 64, 0.125, 0, None) == A.ATTN_EUNSUPPORTED
    assert L.attn_fwd(p, p, p, p, p, 1, 2, 2, 128, 512, 0.125, 0, None) == A.ATTN_EUNSUPPORTED


def test_backward_argument_validation(L):
    import paper_2603_05451_amd as A
    p = ctypes.c_void_p(0x1000)
    ok_ws = A.attn_bwd_workspace_bytes(1, 2, 2, 128, 64, 64)
    bwd = lambda *a: L.attn_bwd_ex(*a)
    nine = [p] * 9
    assert bwd(*nine, 1, 2, 2, 128, 64, 64, 0.125, 0, None, ok_ws, None) == A.ATTN_EINVAL      # no workspace
    assert bwd(*nine, 1, 2, 2, 128, 64, 64, 0.125, 0, p, ok_ws - 1, None) == A.ATTN_EINVAL     # too small
    assert bwd(*nine, 1, 2, 2, 128, 64, 64, 0.125, 0, ctypes.c_void_p(0x1010), ok_ws, None) == A.ATTN_EINVAL
    for i in range(9):
        args = list(nine)
        args[i] = None
        assert bwd(*args, 1, 2, 2, 128, 64, 64, 0.125, 0, p, ok_ws, None) == A.ATTN_EINVAL
    assert bwd(*nine, 1, 2, 2, 128, 192, 192, 0.125, 0, p, 1 << 20, None) == A.ATTN_EUNSUPPORTED
    assert L.attn_bwd_phases(*nine, 1, 2, 2, 128, 64, 64, 0.125, 0, p, ok_ws, None, 0) == A.ATTN_EINVAL
    assert L.attn_bwd_phases(*nine, 1, 2, 2, 128, 64, 64, 0.125, 0, p, ok_ws, None, 8) == A.ATTN_EINVAL


def test_input_recipe_is_reproducible():
    import torch
    from paper_2603_05451_amd import inputs as I
    a, b = I.make_inputs(I.CANARY), I.make_inputs(I.CANARY)
    for n in ("q", "k", "v", "do"):
        assert a[n].dtype == torch.bfloat16 and torch.equal(a[n], b[n])
    w = I.Workload("o", 1, 2, 1, 256, 192, 128, True, 5, outlier_frac=0.01)
    x = I.make_inputs(w)
    frac_big = (x["q"].float().abs() > 6).float().mean().item()
    assert 0.002 < frac_big < 0.02          # ~1 % of entries were multiplied by 8
    assert I.TARGET.fwd_flops() == 4 * 8192 ** 2 * 128 * 16 * 2
    assert I.GQA.fwd_flops() == 4 * 8192 ** 2 * 128 * 32 * 2 / 2


def test_varlen_workspace_and_validation(L):
    import paper_2603_05451_amd as A
    # tables: (T/128 + B) entries of 32 bytes per side, each rounded up to 256 (the forward call needs
    # the query-tile table only); backward adds -D and LSE2 [H, Tq]
    fwd = A.attn_varlen_workspace_bytes(3, 1000, 1000, 4, 2, 128, 128, False)
    bwd = A.attn_varlen_workspace_bytes(3, 1000, 1000, 4, 2, 128, 128, True)
    assert fwd == 512 and bwd == 512 + 512 + 2 * 16128  # 10 entries -> 320 -> 512; 4 * 1000 * 4 = 16000 -> 16128
    bwd_x = A.attn_varlen_workspace_bytes(3, 1000, 5000, 4, 2, 128, 128, True)
    assert bwd_x == 512 + 1536 + 2 * 16128              # 42 key-tile entries -> 1344 -> 1536; statistics sized by Tq
    assert A.attn_varlen_workspace_bytes(3, 1000, 1000, 3, 2, 128, 128, False) == 0      # H % Hkv != 0
    assert A.attn_varlen_workspace_bytes(3, 1000, 1000, 4, 2, 80, 80, False) == 0        # unsupported head dim
    assert A.attn_varlen_workspace_bytes(0, 1000, 1000, 4, 2, 64, 64, False) == 0
    assert A.attn_varlen_workspace_bytes(3, 1000, 0, 4, 2, 64, 64, False) == 0           # no keys at all
    p = ctypes.c_void_p(0x1000)
    w = ctypes.c_void_p(0x1000)
    call = lambda *a: L.attn_varlen_fwd(*a)
    ok_tail = (3, 1000, 1000, 4, 2, 128, 128, 0.1, 0, w, 1 << 20, None)
    assert call(None, p, p, p, p, p, p, *ok_tail) == A.ATTN_EINVAL
    assert call(p, p, p, p, p, None, p, *ok_tail) == A.ATTN_EINVAL                 # one of the two arrays missing
    assert call(p, p, p, p, p, p, None, *ok_tail) == A.ATTN_EINVAL                 # (both missing = cached tables)
    assert call(p, p, p, p, p, p, p, 3, 1000, 1000, 4, 2, 128, 128, 0.1, 0, w, 16, None) == A.ATTN_EINVAL   # workspace too small
    assert call(p, p, p, p, p, p, p, 3, 1000, 1000, 4, 2, 80, 80, 0.1, 0, w, 1 << 20, None) == A.ATTN_EUNSUPPORTED
    assert call(p, p, p, p, p, p, p, 3, 1000, 1000, 4, 2, 128, 128, -1.0, 0, w, 1 << 20, None) == A.ATTN_EINVAL
    assert L.attn_varlen_bwd(p, p, p, p, p, p, p, p, p, p, p, 3, 1000, 1000, 4, 2, 128, 128, 0.1, 0, w, 256,
                             None) == A.ATTN_EINVAL
    # plan tables alone: needs both arrays and a backward-sized workspace
    assert L.attn_varlen_plan(p, None, 3, 1000, 1000, 4, 2, 128, 128, w, 1 << 20, None) == A.ATTN_EINVAL
    assert L.attn_varlen_plan(p, p, 3, 1000, 1000, 4, 2, 128, 128, w, fwd, None) == A.ATTN_EINVAL
    assert L.attn_varlen_plan(p, p, 3, 1000, 1000, 4, 2, 80, 80, w, 1 << 20, None) == A.ATTN_EUNSUPPORTED


def test_strided_validation(L):
    import paper_2603_05451_amd as A
    # the two generated cu_seqlens arrays ((B + 1) ints -> 256 bytes each) precede the variable-length workspace
    assert A.attn_strided_workspace_bytes(2, 4, 2, 384, 384, 128, 128, False) == 512 + \
        A.attn_varlen_workspace_bytes(2, 768, 768, 4, 2, 128, 128, False)
    assert A.attn_strided_workspace_bytes(2, 4, 2, 100, 300, 64, 64, True) == 512 + \
        A.attn_varlen_workspace_bytes(2, 200, 600, 4, 2, 64, 64, True)
    assert A.attn_strided_workspace_bytes(2, 4, 2, 0, 100, 64, 64, True) == 0
    assert A.attn_strided_workspace_bytes(2, 4, 2, 100, 0, 64, 64, True) == 0
    assert A.attn_strided_workspace_bytes(2, 4, 2, 100, 100, 80, 80, True) == 0
    p = ctypes.c_void_p(0x1000)
    ok = ctypes.byref(A.AttnStrides(100 * 4 * 64, 4 * 64, 64))
    call = lambda sq, so, N=100, Nk=100, causal=0: L.attn_fwd_strided(
        A.ATTN_BF16, p, sq, p, ok, p, ok, p, so, p, 2, 4, 4, N, Nk, 64, 64, 0.125, causal, p, 1 << 20, None)
    assert call(None, ok) == A.ATTN_EINVAL                                              # strides missing
    assert call(ctypes.byref(A.AttnStrides(100 * 4 * 64, 4 * 64 + 4, 64)), ok) == A.ATTN_EINVAL   # not 16-byte steps
    assert call(ok, ctypes.byref(A.AttnStrides(0, 4 * 64, 64))) == A.ATTN_EINVAL        # batches on top of each other
    assert call(ok, ctypes.byref(A.AttnStrides(-8, 4 * 64, 64))) == A.ATTN_EINVAL
    assert call(ok, ok, N=0) == A.ATTN_EINVAL
    assert call(ok, ok, Nk=0) == A.ATTN_EINVAL
    assert call(ok, ok, N=100, Nk=99, causal=1) == A.ATTN_EINVAL                        # a query without a visible key
    assert L.attn_fwd_strided(7, p, ok, p, ok, p, ok, p, ok, p, 2, 4, 4, 100, 100, 64, 64, 0.125, 0, p, 1 << 20,
                              None) == A.ATTN_EUNSUPPORTED                              # unknown dtype
    assert L.attn_fwd_strided(A.ATTN_BF16, p, ok, p, ok, p, ok, p, ok, p, 2, 4, 4, 100, 100, 64, 64, 0.125, 0, p, 256,
                              None) == A.ATTN_EINVAL                                    # workspace too small
    bwd = lambda Nk, causal: L.attn_bwd_strided(
        A.ATTN_BF16, p, ok, p, ok, p, ok, p, ok, p, ok, p, p, ok, p, ok, p, ok, 2, 4, 4, 100, Nk, 64, 64,
        0.125, causal, p, 1 << 8, None)
    assert bwd(99, 1) == A.ATTN_EINVAL and bwd(0, 0) == A.ATTN_EINVAL
    assert bwd(100, 0) == A.ATTN_EINVAL                                                 # workspace too small


def test_varlen_workload_recipe_is_deterministic():
    from paper_2603_05451_amd import inputs as I
    w = I.VARLEN_MIX
    a, b = w.lengths(), w.lengths()
    assert a == b and len(a) == w.B and min(a) >= w.lo and max(a) <= w.hi
    x = I.make_varlen_inputs(w, with_do=False)
    T = sum(a)
    assert tuple(x["q"].shape) == (T, w.H, w.dqk) and tuple(x["k"].shape) == (T, w.Hkv, w.dqk)
    cu = x["cu_seqlens"].tolist()
    assert cu[0] == 0 and cu[-1] == T and [cu[i + 1] - cu[i] for i in range(w.B)] == a
    assert w.fwd_flops() == sum(2.0 * n * n * (w.dqk + w.dv) * w.H for n in a) / 2      # causal
