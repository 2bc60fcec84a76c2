"""GPU parity of the variable-length entry points (paper Sec. 3.3) against the CPU fp64 oracle.

The oracle has no notion of packing: every sequence of the packed batch is cut out and handed to
it as a batch of one, which is the definition of "attention inside each sequence only"."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import LSE_ABS, assert_close

pytestmark = pytest.mark.gpu

# lengths chosen to hit: a single row, one short of / exactly / one past the 64-key and 128-row
# tiles, odd numbers of key tiles, an empty sequence, and a longer ragged one
LENGTHS_A = [1, 63, 64, 65, 127, 128, 129, 0, 200, 333, 1000]
LENGTHS_B = [517, 128, 3, 256, 77]


def packed_inputs(lengths, H, Hkv, dqk, dv, seed, with_do=False):
    """Seeded N(0,1) packed tensors: the recipe of inputs.make_inputs with B = 1, N = total tokens."""
    T = int(sum(lengths))
    w = I.Workload("varlen", 1, H, Hkv, T, dqk, dv, False, seed)
    x = I.make_inputs(w, with_do=with_do)
    out = {n: t[0] for n, t in x.items()}                 # drop the batch axis: [T, heads, d]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    return out, cu, w.scale


CASES = [
    ("d64_nc", LENGTHS_A, 4, 2, 64, 64, False, 31),
    ("d64_c", LENGTHS_A, 2, 2, 64, 64, True, 32),
    ("d128_nc", LENGTHS_A, 4, 1, 128, 128, False, 33),
    ("d128_c", LENGTHS_A, 4, 2, 128, 128, True, 34),
    ("d192_c", LENGTHS_B, 2, 1, 192, 128, True, 35),
    ("d192_nc", LENGTHS_B, 2, 2, 192, 128, False, 36),
]


@pytest.mark.parametrize("name,lengths,H,Hkv,dqk,dv,causal,seed", CASES, ids=[c[0] for c in CASES])
def test_varlen_fwd_parity(oracle, name, lengths, H, Hkv, dqk, dv, causal, seed):
    import paper_2603_05451_amd as A
    x, cu, scale = packed_inputs(lengths, H, Hkv, dqk, dv, seed)
    T = int(cu[-1])
    o = torch.full((T, H, dv), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((H, T), float("nan"), dtype=torch.float32, device="cuda")
    A.attn_varlen_fwd(x["q"].cuda(), x["k"].cuda(), x["v"].cuda(), torch.from_numpy(cu).cuda(), scale, causal,
                      o=o, lse=lse)
    torch.cuda.synchronize()
    o, lse = o.float().cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(o).all() and np.isfinite(lse).all()      # every row of every sequence was written
    for b, n in enumerate(lengths):
        if n == 0:
            continue
        s = slice(int(cu[b]), int(cu[b + 1]))
        ro, rlse = oracle.attn_fwd(I.to_f64(x["q"][s][None]), I.to_f64(x["k"][s][None]), I.to_f64(x["v"][s][None]),
                                   scale, causal)
        assert_close(o[s][None], ro, f"varlen O {name} seq{b} len{n}")
        err = np.abs(lse[:, s][None] - rlse).max()
        assert err <= LSE_ABS, f"varlen LSE {name} seq{b} len{n}: {err:.3e}"


def test_varlen_fwd_equals_fixed_length_bitwise():
    """Equal lengths that are multiples of 128: the packed call must reproduce attn_fwd bit for bit
    (same tiles, same order of operations)."""
    import paper_2603_05451_amd as A
    w = I.Workload("eq", 3, 4, 2, 384, 128, 128, True, 41)
    x = I.make_inputs(w, with_do=False)
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    cu = torch.arange(0, (w.B + 1) * w.N, w.N, dtype=torch.int32, device="cuda")
    T = w.B * w.N
    ov, lsev = A.attn_varlen_fwd(q.reshape(T, w.H, w.dqk), k.reshape(T, w.Hkv, w.dqk), v.reshape(T, w.Hkv, w.dv),
                                 cu, w.scale, w.causal)
    torch.cuda.synchronize()
    assert torch.equal(ov.reshape(o.shape), o)
    assert torch.equal(lsev.reshape(w.H, w.B, w.N).permute(1, 0, 2), lse)


@pytest.mark.parametrize("name,lengths,H,Hkv,dqk,dv,causal,seed", CASES, ids=[c[0] for c in CASES])
def test_varlen_bwd_parity(oracle, name, lengths, H, Hkv, dqk, dv, causal, seed):
    import paper_2603_05451_amd as A
    x, cu, scale = packed_inputs(lengths, H, Hkv, dqk, dv, seed, with_do=True)
    T = int(cu[-1])
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    cud = torch.from_numpy(cu).cuda()
    o, lse = A.attn_varlen_fwd(q, k, v, cud, scale, causal)
    nan = lambda t: torch.full_like(t, float("nan"))
    dq, dk, dvv = A.attn_varlen_bwd(q, k, v, o, do, lse, cud, scale, causal, dq=nan(q), dk=nan(k), dv=nan(v))
    torch.cuda.synchronize()
    dq, dk, dvv = (t.float().cpu().numpy() for t in (dq, dk, dvv))
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dvv).all()   # every row written
    for b, n in enumerate(lengths):
        if n == 0:
            continue
        s = slice(int(cu[b]), int(cu[b + 1]))
        rdq, rdk, rdv = oracle.attn_bwd(*(I.to_f64(x[m][s][None]) for m in ("q", "k", "v", "do")), scale, causal)
        if n == 1:     # a single key: dS = 0, so dQ and dK are exactly zero and a relative error has no meaning
            assert np.abs(rdq).max() == 0 and np.abs(dq[s]).max() <= 1e-5 and np.abs(dk[s] - rdk[0]).max() <= 1e-5
            assert_close(dvv[s][None], rdv, f"varlen dV {name} seq{b} len{n}")
            continue
        assert_close(dq[s][None], rdq, f"varlen dQ {name} seq{b} len{n}")
        assert_close(dk[s][None], rdk, f"varlen dK {name} seq{b} len{n}")
        assert_close(dvv[s][None], rdv, f"varlen dV {name} seq{b} len{n}")


def test_varlen_bwd_matches_fixed_length_and_is_reproducible():
    """Equal lengths that are multiples of 128: dQ is bit-identical to attn_bwd (same kernel
    structure); dK/dV use the unspecialised kernel at d = 128 and must agree to rounding.  Two
    packed calls give identical bits."""
    import paper_2603_05451_amd as A
    w = I.Workload("eq", 2, 4, 2, 384, 128, 128, True, 42)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    cu = torch.arange(0, (w.B + 1) * w.N, w.N, dtype=torch.int32, device="cuda")
    T = w.B * w.N
    p = lambda t: t.reshape(T, *t.shape[2:])
    ov, lsev = A.attn_varlen_fwd(p(q), p(k), p(v), cu, w.scale, w.causal)
    r1 = A.attn_varlen_bwd(p(q), p(k), p(v), ov, p(do), lsev, cu, w.scale, w.causal)
    r2 = A.attn_varlen_bwd(p(q), p(k), p(v), ov, p(do), lsev, cu, w.scale, w.causal)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(r1, r2))
    assert torch.equal(r1[0].reshape(dq.shape), dq)
    assert_close(r1[1].reshape(dk.shape).float().cpu().numpy(), dk.float().cpu().numpy(), "varlen dK vs fixed",
                 max_abs=2e-2, rel_fro=5e-3)
    assert_close(r1[2].reshape(dv.shape).float().cpu().numpy(), dv.float().cpu().numpy(), "varlen dV vs fixed",
                 max_abs=2e-2, rel_fro=5e-3)
