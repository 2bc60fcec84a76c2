"""GPU tests of the strided entry points: [B, H, N, d] tensors, slices of a fused QKV buffer and
padded buffers give what the contiguous [B, N, H, d] calls give (bit for bit where the tiles are
the same) and match the fp64 oracle where N is not a multiple of the tile."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import LSE_ABS, assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dqk,dv,H,Hkv,causal,seed", [(128, 128, 4, 2, True, 81), (64, 64, 2, 2, False, 82),
                                                       (192, 128, 2, 1, True, 83)])
def test_bhsd_views_match_contiguous_calls_bitwise(dqk, dv, H, Hkv, causal, seed):
    """Tensors stored [B, H, N, d], handed over as permuted views; gradients are written into
    [B, H, N, d] buffers through views as well.  N is a multiple of 128, so the strided call cuts
    the same tiles as attn_fwd / attn_bwd and must reproduce their bits."""
    import paper_2603_05451_amd as A
    w = I.Workload("bhsd", 2, H, Hkv, 384, dqk, dv, causal, seed)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o_ref, lse_ref = A.attn_fwd(q, k, v, w.scale, causal)
    g_ref = A.attn_bwd(q, k, v, o_ref, do, lse_ref, w.scale, causal)
    bhsd = lambda t: t.permute(0, 2, 1, 3).contiguous()              # storage [B, heads, N, d]
    view = lambda t: t.permute(0, 2, 1, 3)                           # logical [B, N, heads, d] again
    qs, ks, vs, dos = (bhsd(t) for t in (q, k, v, do))
    os_ = torch.full_like(bhsd(o_ref), float("nan"))
    o, lse = A.attn_fwd_strided(view(qs), view(ks), view(vs), w.scale, causal, o=view(os_))
    grads = [torch.full_like(t, float("nan")) for t in (qs, ks, vs)]
    A.attn_bwd_strided(view(qs), view(ks), view(vs), view(os_), view(dos), lse, w.scale, causal,
                       dq=view(grads[0]), dk=view(grads[1]), dv=view(grads[2]))
    torch.cuda.synchronize()
    assert torch.equal(view(os_), o_ref) and torch.equal(lse, lse_ref)
    for got, ref in zip(grads, g_ref):
        assert torch.equal(view(got), ref)


@pytest.mark.parametrize("d,N,causal,seed", [(64, 200, True, 84), (128, 333, False, 85), (128, 1, True, 86),
                                             (96, 130, True, 88), (256, 190, True, 89)])
def test_fused_qkv_buffer_any_length(oracle, d, N, causal, seed):
    """q, k, v are slices of one [B, N, H + 2 Hkv, d] buffer (the output of a fused projection), the
    gradients slices of another; N is not a multiple of any tile.  Checked against the oracle."""
    import paper_2603_05451_amd as A
    B, H, Hkv = 3, 4, 2
    w = I.Workload("fused", B, H, Hkv, N, d, d, causal, seed)
    x = I.make_inputs(w)
    qkv = torch.cat([x["q"], x["k"], x["v"]], dim=2).cuda()          # [B, N, H + 2 Hkv, d]
    q, k, v = qkv[:, :, :H], qkv[:, :, H:H + Hkv], qkv[:, :, H + Hkv:]
    assert not q.is_contiguous() and q.stride(1) == (H + 2 * Hkv) * d
    do = x["do"].cuda()
    o, lse = A.attn_fwd_strided(q, k, v, w.scale, causal)
    dqkv = torch.full_like(qkv, float("nan"))
    A.attn_bwd_strided(q, k, v, o, do, lse, w.scale, causal,
                       dq=dqkv[:, :, :H], dk=dqkv[:, :, H:H + Hkv], dv=dqkv[:, :, H + Hkv:])
    torch.cuda.synchronize()
    assert torch.isfinite(dqkv.float()).all()                         # every gradient element written
    f = lambda n: I.to_f64(x[n])
    ro, rlse = oracle.attn_fwd(f("q"), f("k"), f("v"), w.scale, causal)
    rdq, rdk, rdv = oracle.attn_bwd(f("q"), f("k"), f("v"), f("do"), w.scale, causal)
    g = dqkv.float().cpu().numpy()
    assert np.abs(lse.cpu().numpy() - rlse).max() <= LSE_ABS
    if N == 1:     # one key: P = 1, dS = 0, dQ = dK = 0 exactly, O = V, dV = sum over the group of dO
        assert np.abs(g[:, :, :H + Hkv]).max() <= 1e-5
        assert_close(o.float().cpu().numpy(), ro, "strided O N=1")
        assert_close(g[:, :, H + Hkv:], rdv, "strided dV N=1")
        return
    assert_close(o.float().cpu().numpy(), ro, f"strided O d{d} N{N}")
    assert_close(g[:, :, :H], rdq, f"strided dQ d{d} N{N}")
    assert_close(g[:, :, H:H + Hkv], rdk, f"strided dK d{d} N{N}")
    assert_close(g[:, :, H + Hkv:], rdv, f"strided dV d{d} N{N}")


def test_padded_rows_leave_the_padding_untouched():
    """Outputs that are views into wider buffers (row stride larger than heads x d): the elements
    between the rows keep their contents."""
    import paper_2603_05451_amd as A
    w = I.Workload("pad", 2, 2, 2, 256, 128, 128, True, 87)
    x = I.make_inputs(w, with_do=False)
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    o_ref, _ = A.attn_fwd(q, k, v, w.scale, True)
    wide = torch.full((2, 256, 2, 128 + 64), 7.0, dtype=torch.bfloat16, device="cuda")
    o, _ = A.attn_fwd_strided(q, k, v, w.scale, True, o=wide[..., :128])
    torch.cuda.synchronize()
    assert torch.equal(wide[..., :128], o_ref) and (wide[..., 128:] == 7.0).all()


CROSS = [("d128_c_append", 128, 128, 4, 2, 200, 457, True, 90), ("d64_nc_more_queries", 64, 64, 2, 2, 300, 77, False, 91),
         ("d128_c_decode", 128, 128, 4, 1, 1, 1000, True, 92), ("d192_c", 192, 128, 2, 1, 130, 384, True, 93),
         ("d96_nc", 96, 96, 4, 2, 64, 640, False, 94), ("d256_c", 256, 256, 2, 1, 129, 258, True, 95)]


@pytest.mark.parametrize("name,dqk,dv,H,Hkv,Nq,Nk,causal,seed", CROSS, ids=[c[0] for c in CROSS])
def test_separate_query_and_key_counts(oracle, name, dqk, dv, H, Hkv, Nq, Nk, causal, seed):
    """Equal-length batches with Nq queries against Nk keys per sequence (a chunk appended to a
    cached prefix, one decoded token, cross-attention), q/k/v stored [B, heads, N, d].  Under the
    causal mask the last query sees the last key, which the oracle expresses through the query
    positions Nk - Nq ... Nk - 1."""
    import paper_2603_05451_amd as A
    B = 3
    w = I.Workload("cross", B, H, Hkv, max(Nq, Nk), dqk, dv, causal, seed)
    x = I.make_inputs(w)
    cut = lambda n: x[n][:, :(Nq if n in ("q", "do") else Nk)]
    if name == "d128_c_append":      # one case in fp16 storage (the oracle sees the same fp16 values)
        x = {n: t.float().to(torch.float16) for n, t in x.items()}
    bhsd = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)   # storage [B, heads, N, d]
    q, k, v, do = (bhsd(cut(n)) for n in ("q", "k", "v", "do"))
    assert not q.is_contiguous() or Nq == 1
    o, lse = A.attn_fwd_strided(q, k, v, w.scale, causal)
    dq, dk, dvv = A.attn_bwd_strided(q, k, v, o, do, lse, w.scale, causal)
    torch.cuda.synchronize()
    assert tuple(o.shape) == (B, Nq, H, dv) and tuple(lse.shape) == (B, H, Nq) and tuple(dk.shape) == (B, Nk, Hkv, dqk)
    pos = np.arange(Nq) + (Nk - Nq)
    f = lambda n: I.to_f64(cut(n))
    ro, rlse = oracle.attn_fwd(f("q"), f("k"), f("v"), w.scale, causal, q_pos=pos)
    rdq, rdk, rdv = oracle.attn_bwd(f("q"), f("k"), f("v"), f("do"), w.scale, causal, q_pos=pos)
    got = [t.float().cpu().numpy() for t in (o, dq, dk, dvv)]
    assert all(np.isfinite(t).all() for t in got)
    assert np.abs(lse.cpu().numpy() - rlse).max() <= LSE_ABS
    assert_close(got[0], ro, f"{name} O")
    assert_close(got[1], rdq, f"{name} dQ")
    assert_close(got[2], rdk, f"{name} dK")
    assert_close(got[3], rdv, f"{name} dV")


def test_separate_counts_match_the_packed_calls_bitwise():
    """The strided call with Nq != Nk is the variable-length call on the boundaries {0, Nq, ...} and
    {0, Nk, ...}: same kernels, same tiles, same bits."""
    import paper_2603_05451_amd as A
    B, H, Hkv, Nq, Nk, d = 2, 4, 2, 200, 457, 128
    w = I.Workload("cross", B, H, Hkv, Nk, d, d, True, 96)
    x = I.make_inputs(w)
    q, do = (x[n][:, :Nq].contiguous().cuda() for n in ("q", "do"))
    k, v = x["k"].cuda(), x["v"].cuda()
    o, lse = A.attn_fwd_strided(q, k, v, w.scale, True)
    g = A.attn_bwd_strided(q, k, v, o, do, lse, w.scale, True)
    cuq = torch.arange(0, B + 1, dtype=torch.int32, device="cuda") * Nq
    cuk = torch.arange(0, B + 1, dtype=torch.int32, device="cuda") * Nk
    flat = lambda t: t.reshape(-1, t.shape[2], t.shape[3])
    o2, lse2 = A.attn_varlen_fwd(flat(q), flat(k), flat(v), cuq, w.scale, True, cu_seqlens_k=cuk)
    g2 = A.attn_varlen_bwd(flat(q), flat(k), flat(v), o2, flat(do), lse2, cuq, w.scale, True, cu_seqlens_k=cuk)
    torch.cuda.synchronize()
    assert torch.equal(flat(o), o2)
    assert torch.equal(lse.permute(1, 0, 2).reshape(H, B * Nq), lse2)
    for a, b in zip(g, g2):
        assert torch.equal(flat(a), b)
