"""GPU parity of the fp16 entry points (attn_*_dtype with ATTN_F16) against the CPU fp64 oracle.

Inputs are the seeded N(0,1) tensors of the bf16 tests rounded to fp16 instead; the oracle sees
exactly those fp16 values.  fp16 has three more mantissa bits than bf16, so the bf16 tolerances
hold with room to spare; the test also checks that the error is in fact smaller."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import LSE_ABS, assert_close, errors

pytestmark = pytest.mark.gpu

CASES = [
    I.Workload("h_d64_c", 2, 4, 2, 384, 64, 64, True, 61),
    I.Workload("h_d96_c", 1, 4, 2, 384, 96, 96, True, 66),
    I.Workload("h_d128_nc", 1, 4, 4, 512, 128, 128, False, 62),
    I.Workload("h_d128_c_gqa", 2, 4, 1, 384, 128, 128, True, 63),
    I.Workload("h_d192_c", 1, 2, 2, 384, 192, 128, True, 64),
    I.Workload("h_d256_c", 1, 2, 1, 256, 256, 256, True, 67),
    # shapes that run the one-wave-per-SIMD kernels (64 queries per wave forward and dQ, one-wave dK/dV)
    I.Workload("h_d128_nc_2048_gqa", 1, 2, 1, 2048, 128, 128, False, 68),
    I.Workload("h_d128_c_4096", 1, 1, 1, 4096, 128, 128, True, 69),
    I.Workload("h_d64_nc_2048", 1, 2, 1, 2048, 64, 64, False, 71),
    I.Workload("h_d192_nc_2048_gqa", 1, 2, 1, 2048, 192, 128, False, 72),
]


def half_inputs(w):
    x = I.make_inputs(w)
    return {n: t.float().to(torch.float16) for n, t in x.items()}


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_fp16_fwd_bwd_parity(oracle, w):
    import paper_2603_05451_amd as A
    x = half_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    torch.cuda.synchronize()
    assert o.dtype == torch.float16 and dq.dtype == torch.float16
    f = [I.to_f64(x[n]) for n in ("q", "k", "v", "do")]
    ro, rlse = oracle.attn_fwd(f[0], f[1], f[2], w.scale, w.causal)
    rdq, rdk, rdv = oracle.attn_bwd(*f, w.scale, w.causal)
    n64 = lambda t: t.float().cpu().numpy()
    _, rf_o = assert_close(n64(o), ro, f"fp16 O {w.name}")
    assert np.abs(lse.cpu().numpy() - rlse).max() <= LSE_ABS
    assert_close(n64(dq), rdq, f"fp16 dQ {w.name}")
    assert_close(n64(dk), rdk, f"fp16 dK {w.name}")
    assert_close(n64(dv), rdv, f"fp16 dV {w.name}")
    assert rf_o <= 1e-3, rf_o          # bf16 sits at 2.3e-3 (its output rounding floor); fp16 is 8x finer


def test_fp16_fwd_d64_64_queries_per_wave(oracle):
    """d = 64, N = 8192 without a mask: the forward kernel with 64 queries per wave in its fp16 form."""
    import paper_2603_05451_amd as A
    w = I.Workload("h_d64_nc_8192", 1, 2, 1, 8192, 64, 64, False, 70)
    x = half_inputs(w)
    o, lse = A.attn_fwd(x["q"].cuda(), x["k"].cuda(), x["v"].cuda(), w.scale, w.causal)
    torch.cuda.synchronize()
    ro, rlse = oracle.attn_fwd(I.to_f64(x["q"]), I.to_f64(x["k"]), I.to_f64(x["v"]), w.scale, w.causal)
    _, rf_o = assert_close(o.float().cpu().numpy(), ro, f"fp16 O {w.name}")
    assert np.abs(lse.cpu().numpy() - rlse).max() <= LSE_ABS
    assert rf_o <= 1e-3, rf_o


def test_fp16_varlen_parity(oracle):
    import paper_2603_05451_amd as A
    lengths = [65, 128, 200, 1, 333]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T, H, Hkv, d = int(cu[-1]), 4, 2, 128
    x = {n: t[0].float().to(torch.float16) for n, t in I.make_inputs(I.Workload("hv", 1, H, Hkv, T, d, d, True, 65)).items()}
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    cud = torch.from_numpy(cu).cuda()
    o, lse = A.attn_varlen_fwd(q, k, v, cud, d ** -0.5, True)
    dq, dk, dv = A.attn_varlen_bwd(q, k, v, o, do, lse, cud, d ** -0.5, True)
    torch.cuda.synchronize()
    for b, n in enumerate(lengths):
        if n == 1:
            continue
        s = slice(int(cu[b]), int(cu[b + 1]))
        f = [I.to_f64(x[m][s][None]) for m in ("q", "k", "v", "do")]
        ro, _ = oracle.attn_fwd(f[0], f[1], f[2], d ** -0.5, True)
        rdq, rdk, rdv = oracle.attn_bwd(*f, d ** -0.5, True)
        for name, got, ref in (("O", o, ro), ("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
            assert_close(got[s].float().cpu().numpy()[None], ref, f"fp16 varlen {name} seq{b}")


def test_fp16_rejects_mixed_types_and_unknown_dtype():
    import ctypes
    import paper_2603_05451_amd as A
    w = CASES[0]
    x = half_inputs(w)
    with pytest.raises(ValueError):
        A.attn_fwd(x["q"].cuda(), x["k"].cuda().to(torch.bfloat16), x["v"].cuda(), w.scale, w.causal)
    p = ctypes.c_void_p(0x1000)
    assert A.lib().attn_fwd_dtype(7, p, p, p, p, p, 1, 2, 2, 128, 64, 64, 0.125, 0, None) == A.ATTN_EUNSUPPORTED
