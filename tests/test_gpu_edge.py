"""GPU edge cases through the C ABI: extreme head grouping, smallest N, guard regions around
every output, a non-default stream, caller-provided buffers and workspace reuse."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import LSE_ABS, assert_close

pytestmark = pytest.mark.gpu


def oracle_all(oracle, w, x):
    f = [I.to_f64(x[n]) for n in ("q", "k", "v", "do")]
    o, lse = oracle.attn_fwd(f[0], f[1], f[2], w.scale, w.causal)
    dq, dk, dv = oracle.attn_bwd(*f, w.scale, w.causal)
    return o, lse, dq, dk, dv


EDGE = [
    I.Workload("mqa8_d128_c", 1, 8, 1, 256, 128, 128, True, 41),        # MQA: 8 query heads, 1 KV head
    I.Workload("mqa8_d64_nc", 2, 8, 1, 128, 64, 64, False, 42),
    I.Workload("gqa4_d192_nc", 1, 8, 2, 256, 192, 128, False, 43),
    I.Workload("n128_d128_c", 3, 2, 2, 128, 128, 128, True, 44),        # smallest N, causal: one diagonal tile
    I.Workload("n128_d192_c", 1, 1, 1, 128, 192, 128, True, 45),
    I.Workload("b5_d64_c", 5, 2, 1, 384, 64, 64, True, 46),             # grid not a multiple of 8 (no XCD un-dealing)
    I.Workload("n896_d128_c", 1, 3, 3, 896, 128, 128, True, 47),        # 7 query tiles: odd tile counts everywhere
]


@pytest.mark.parametrize("w", EDGE, ids=lambda w: w.name)
def test_edge_shapes_full_parity(oracle, w):
    import paper_2603_05451_amd as A
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    torch.cuda.synchronize()
    ro, rlse, rdq, rdk, rdv = oracle_all(oracle, w, x)
    assert_close(o.float().cpu().numpy(), ro, f"O {w.name}")
    assert np.abs(lse.cpu().numpy() - rlse).max() <= LSE_ABS
    assert_close(dq.float().cpu().numpy(), rdq, f"dQ {w.name}")
    assert_close(dk.float().cpu().numpy(), rdk, f"dK {w.name}")
    assert_close(dv.float().cpu().numpy(), rdv, f"dV {w.name}")


def guarded(shape, dtype, guard=4096):
    """A tensor carved out of a larger NaN-filled allocation; returns (view, whole, lo, hi)."""
    n = int(np.prod(shape))
    whole = torch.full((n + 2 * guard,), float("nan"), dtype=dtype, device="cuda")
    return whole[guard:guard + n].view(shape), whole, guard, guard + n


def test_outputs_stay_inside_their_buffers_and_streams_are_honoured(oracle):
    """Every output and the workspace sit between NaN guard regions; the call runs on a side
    stream with caller-provided buffers, twice, reusing the workspace."""
    import paper_2603_05451_amd as A
    w = I.Workload("guard", 2, 4, 2, 384, 128, 128, True, 51)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, o_all, o_lo, o_hi = guarded((w.B, w.N, w.H, w.dv), torch.bfloat16)
    lse, lse_all, l_lo, l_hi = guarded((w.B, w.H, w.N), torch.float32)
    dq, dq_all, q_lo, q_hi = guarded(tuple(q.shape), torch.bfloat16)
    dk, dk_all, k_lo, k_hi = guarded(tuple(k.shape), torch.bfloat16)
    dv, dv_all, v_lo, v_hi = guarded(tuple(v.shape), torch.bfloat16)
    need = A.attn_bwd_workspace_bytes(w.B, w.H, w.Hkv, w.N, w.dqk, w.dv)
    ws_all = torch.full((need + 8192,), 0xAB, dtype=torch.uint8, device="cuda")
    ws = ws_all[4096:4096 + need]
    assert ws.data_ptr() % 256 == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for _ in range(2):
        A.attn_fwd(q, k, v, w.scale, w.causal, o, lse, stream=side)
        A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal, dq, dk, dv, ws, stream=side)
    side.synchronize()
    for whole, lo, hi in ((o_all, o_lo, o_hi), (lse_all, l_lo, l_hi), (dq_all, q_lo, q_hi),
                          (dk_all, k_lo, k_hi), (dv_all, v_lo, v_hi)):
        assert torch.isnan(whole[:lo].float()).all() and torch.isnan(whole[hi:].float()).all(), "guard overwritten"
        assert torch.isfinite(whole[lo:hi].float()).all()
    assert (ws_all[:4096] == 0xAB).all() and (ws_all[4096 + need:] == 0xAB).all(), "workspace overrun"
    ro, rlse, rdq, rdk, rdv = oracle_all(oracle, w, x)
    assert_close(o.float().cpu().numpy(), ro, "O guard")
    assert_close(dq.float().cpu().numpy(), rdq, "dQ guard")
    assert_close(dk.float().cpu().numpy(), rdk, "dK guard")
    assert_close(dv.float().cpu().numpy(), rdv, "dV guard")


def test_errors_raise_and_leave_outputs_untouched():
    import paper_2603_05451_amd as A
    q = torch.zeros((1, 192, 2, 64), dtype=torch.bfloat16, device="cuda")      # N not a multiple of 128
    o = torch.full((1, 192, 2, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(A.AttnError) as e:
        A.attn_fwd(q, q, q, 0.125, False, o=o)
    assert e.value.code == A.ATTN_EUNSUPPORTED
    torch.cuda.synchronize()
    assert (o == 7.0).all()
    q = torch.zeros((1, 128, 2, 80), dtype=torch.bfloat16, device="cuda")      # unsupported head dim
    with pytest.raises(A.AttnError):
        A.attn_fwd(q, q, q, 0.1, False)


@pytest.mark.parametrize("w", I.SWEEP_D64_NC[1:5] + I.SWEEP_D128_C[1:4], ids=lambda w: w.name)
def test_sweep_midpoints_sampled(oracle, w):
    """The sweep points between the smallest and largest N: sampled rows of O, LSE and dQ; dK and dV of
    every key of one head without a mask (the oracle runs all N query rows of that head), of the last
    128 keys under the causal mask (the complete-group check at N = 8192 covers the long loops)."""
    import paper_2603_05451_amd as A
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    torch.cuda.synchronize()
    rng = np.random.default_rng(w.seed + 100)
    rows = np.unique(np.concatenate([[0, 127, 128, w.N - 1], rng.integers(0, w.N, 12)]))
    b, h = w.B - 1, w.H // 2
    f = lambda name, r: I.to_f64(x[name][b:b + 1, :, h:h + 1][:, r])
    kk, vv = I.to_f64(x["k"][b:b + 1, :, h:h + 1]), I.to_f64(x["v"][b:b + 1, :, h:h + 1])
    ro, rlse = oracle.attn_fwd(f("q", rows), kk, vv, w.scale, w.causal, q_pos=rows)
    rdq, _, _ = oracle.attn_bwd(f("q", rows), kk, vv, f("do", rows), w.scale, w.causal, q_pos=rows)
    assert_close(o[b, :, h].float().cpu().numpy()[rows], ro[0, :, 0], f"O rows {w.name}")
    assert np.abs(lse[b, h].cpu().numpy()[rows] - rlse[0, 0]).max() <= LSE_ABS
    assert_close(dq[b, :, h].float().cpu().numpy()[rows], rdq[0, :, 0], f"dQ rows {w.name}")
    if w.causal:
        tail = np.arange(w.N - 128, w.N)
        _, rdk, rdv = oracle.attn_bwd(f("q", tail), kk, vv, f("do", tail), w.scale, True, q_pos=tail)
        assert_close(dk[b, :, h].float().cpu().numpy()[tail], rdk[0, tail, 0], f"dK tail {w.name}")
        assert_close(dv[b, :, h].float().cpu().numpy()[tail], rdv[0, tail, 0], f"dV tail {w.name}")
    else:
        allrows = np.arange(w.N)
        _, rdk, rdv = oracle.attn_bwd(f("q", allrows), kk, vv, f("do", allrows), w.scale, False)
        assert_close(dk[b, :, h].float().cpu().numpy(), rdk[0, :, 0], f"dK all keys {w.name}")
        assert_close(dv[b, :, h].float().cpu().numpy(), rdv[0, :, 0], f"dV all keys {w.name}")


def test_literal_north_star_entry_points_on_live_tensors():
    """attn_fwd and attn_bwd, the two signatures with a single head dim d, called directly through
    ctypes on live tensors: the bits of the attn_fwd_ex / attn_bwd_phases route the binding takes."""
    import ctypes
    import paper_2603_05451_amd as A
    w = I.Workload("literal", 2, 4, 2, 384, 128, 128, True, 71)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o_ref, lse_ref = A.attn_fwd(q, k, v, w.scale, True)
    g_ref = A.attn_bwd(q, k, v, o_ref, do, lse_ref, w.scale, True)
    L = A.lib()
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    o = torch.full_like(o_ref, float("nan")); lse = torch.full_like(lse_ref, float("nan"))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.attn_fwd(p(q), p(k), p(v), p(o), p(lse), w.B, w.H, w.Hkv, w.N, 128, ctypes.c_float(w.scale), 1, stream) == 0
    nbytes = L.attn_bwd_workspace_bytes(w.B, w.H, w.Hkv, w.N, 128, 128)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    got = [torch.full_like(t, float("nan")) for t in (q, k, v)]
    assert L.attn_bwd(p(q), p(k), p(v), p(o), p(do), p(lse), p(got[0]), p(got[1]), p(got[2]),
                      w.B, w.H, w.Hkv, w.N, 128, ctypes.c_float(w.scale), 1, p(ws), nbytes, stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    for a, b in zip(got, g_ref):
        assert torch.equal(a, b)


@pytest.mark.parametrize("causal,d,N", [(True, 128, 4096), (False, 128, 4096), (True, 64, 8192), (False, 64, 2048)])
def test_dq_of_every_row_of_the_first_and_last_query_tiles(oracle, causal, d, N):
    """The dQ kernel with 64 queries per wave at its shortest sequences (d = 128: N = 4096; d = 64: N = 8192
    with the causal mask, 2048 without).  Every row of the first two and of the
    last two 256-query tiles of one (batch, head) against the oracle: under the causal mask the first
    tiles have the shortest rows and the largest P, so one wrong (query, key) pair of the last key block
    of a tile shows there and nowhere else (sampled rows of long sequences do not see it)."""
    import paper_2603_05451_amd as A
    w = I.Workload("dq_tiles", 1, 4, 2, N, d, d, causal, 73)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, causal)
    dq, _, _ = A.attn_bwd(q, k, v, o, do, lse, w.scale, causal)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(0, 512), np.arange(w.N - 512, w.N)])
    f = lambda name, r=slice(None), h=3: I.to_f64(x[name][0, r, h])[None, :, None, :]
    rdq, _, _ = oracle.attn_bwd(f("q", rows), f("k", h=1), f("v", h=1), f("do", rows), w.scale, causal, q_pos=rows)
    got = dq[0, torch.from_numpy(rows).cuda(), 3].float().cpu().numpy()[None, :, None, :]
    assert_close(got, rdq, f"dQ all rows of four tiles, causal={causal} d={d}")
    # row by row as well: an error confined to a few rows must not hide in the norm of a thousand
    err = np.abs(got - rdq)[0, :, 0].max(axis=1)
    assert (err <= 2e-3 + 2.0 ** -8 * np.abs(rdq)[0, :, 0].max(axis=1)).all(), (rows[err.argmax()], err.max())
