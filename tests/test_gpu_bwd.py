"""GPU parity of the backward pass against the CPU fp64 oracle, through the C ABI.

The GPU backward consumes the bf16 O and fp32 LSE written by the GPU forward (as the ABI
requires); the oracle recomputes everything from q, k, v, dO in fp64."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import assert_close, assert_close_terms, rounded_reference, term_magnitudes

pytestmark = pytest.mark.gpu


def gpu_fwd_bwd(w, x):
    import paper_2603_05451_amd as A
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    torch.cuda.synchronize()
    return tuple(t.float().cpu().numpy() for t in (dq, dk, dv))


SMALL = [
    I.CANARY,
    I.Workload("s_d64_c", 2, 4, 2, 384, 64, 64, True, 21),
    I.Workload("s_d64_nc", 1, 3, 1, 256, 64, 64, False, 22),
    I.Workload("s_d96_c", 2, 4, 2, 384, 96, 96, True, 28),
    I.Workload("s_d96_nc", 1, 3, 3, 640, 96, 96, False, 29),
    I.Workload("s_d128_nc", 2, 4, 4, 384, 128, 128, False, 23),
    I.Workload("s_d128_c", 2, 4, 2, 640, 128, 128, True, 24),
    I.Workload("s_d256_c", 1, 4, 2, 384, 256, 256, True, 20),
    I.Workload("s_d256_nc", 2, 2, 2, 256, 256, 256, False, 19),
    I.Workload("s_d192_c", 1, 4, 2, 384, 192, 128, True, 25),
    I.Workload("s_d192_nc", 1, 2, 2, 256, 192, 128, False, 26),
    I.Workload("s_d192_c_outl", 1, 2, 1, 512, 192, 128, True, 27, outlier_frac=0.01),
    # d = 64 without a mask from N = 2048: the one-wave-per-SIMD kernels (64 queries per wave for dQ, 64 keys
    # per wave for dK / dV), GQA with three heads per group, 8 and 9 blocks of 256 rows
    I.Workload("s_d64_nc_2048_gqa", 1, 3, 1, 2048, 64, 64, False, 18),
    I.Workload("s_d64_nc_2304", 2, 2, 2, 2304, 64, 64, False, 17),
    # d = 64 under the causal mask: the one-wave-per-SIMD kernels start at N = 8192 (two query heads per KV head)
    I.Workload("s_d64_c_8192_gqa", 1, 2, 1, 8192, 64, 64, True, 14),
    # (192, 128) from N = 1024 with the causal mask and N = 512 without: the one-wave dQ kernel with 32 queries per wave
    I.Workload("s_d192_c_1024_gqa", 1, 3, 1, 1024, 192, 128, True, 16),
    I.Workload("s_d192_nc_640", 2, 2, 2, 640, 192, 128, False, 15),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_bwd_small_full_parity(oracle, w):
    x = I.make_inputs(w)
    dq, dk, dv = gpu_fwd_bwd(w, x)
    rdq, rdk, rdv = oracle.attn_bwd(*(I.to_f64(x[n]) for n in ("q", "k", "v", "do")), w.scale, w.causal)
    if not w.outlier_frac:
        assert_close(dq, rdq, f"dQ {w.name}")
        assert_close(dk, rdk, f"dK {w.name}")
        assert_close(dv, rdv, f"dV {w.name}")
        return
    G = w.H // w.Hkv
    for b in range(w.B):
        for kvh in range(w.Hkv):
            hs = slice(kvh * G, (kvh + 1) * G)
            args = (I.to_f64(x["q"][b, :, hs]), I.to_f64(x["k"][b, :, kvh]), I.to_f64(x["v"][b, :, kvh]),
                    I.to_f64(x["do"][b, :, hs]), w.scale, w.causal)
            _, a_dq, a_dk, a_dv = term_magnitudes(*args)
            _, r_dq, r_dk, r_dv = rounded_reference(*args)
            assert_close_terms(dq[b, :, hs], rdq[b, :, hs], a_dq, f"dQ {w.name} b{b} kvh{kvh}", r_dq)
            assert_close_terms(dk[b, :, kvh], rdk[b, :, kvh], a_dk, f"dK {w.name} b{b} kvh{kvh}", r_dk)
            assert_close_terms(dv[b, :, kvh], rdv[b, :, kvh], a_dv, f"dV {w.name} b{b} kvh{kvh}", r_dv)


def test_bwd_is_bit_reproducible():
    """No atomics anywhere in the backward pass: two runs give identical bits."""
    w = I.Workload("rep", 1, 4, 2, 1024, 128, 128, True, 31)
    x = I.make_inputs(w)
    a = gpu_fwd_bwd(w, x)
    b = gpu_fwd_bwd(w, x)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


@pytest.mark.parametrize("dqk,dv,N,causal,seed", [(128, 128, 4096, False, 32), (128, 128, 384, True, 33),
                                                  (64, 64, 256, False, 34), (96, 96, 384, True, 35),
                                                  (192, 128, 256, True, 36), (256, 256, 256, False, 37)])
def test_bwd_phases_compose(dqk, dv, N, causal, seed):
    """The backward pass split at its kernel boundaries gives the bits of the whole call, in both
    orders the workspace allows: the prepare kernel, then dK/dV, then dQ (the standalone prepare
    kernel and the dQ kernel's own prologue must write the same -D and base-2 LSE), and dQ first,
    then dK/dV on what it left."""
    import paper_2603_05451_amd as A
    w = I.Workload("phases", 2, 4, 2, N, dqk, dv, causal, seed)
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, causal)
    ref = A.attn_bwd(q, k, v, o, do, lse, w.scale, causal)
    nbytes = A.attn_bwd_workspace_bytes(w.B, w.H, w.Hkv, N, dqk, dv)
    for order in ((A.ATTN_BWD_PREPARE, A.ATTN_BWD_DKDV, A.ATTN_BWD_DQ), (A.ATTN_BWD_DQ, A.ATTN_BWD_DKDV),
                  (A.ATTN_BWD_PREPARE | A.ATTN_BWD_DKDV, A.ATTN_BWD_DQ)):
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")      # NaN bit patterns
        got = [torch.full_like(t, float("nan")) for t in (q, k, v)]
        for ph in order:
            A.attn_bwd(q, k, v, o, do, lse, w.scale, causal, got[0], got[1], got[2], ws, phases=ph)
        torch.cuda.synchronize()
        for a, b in zip(got, ref):
            assert torch.equal(a, b), f"phases {order}"


FULL = [I.TARGET, I.SWEEP_D64_NC[0], I.SWEEP_D64_NC[5], I.SWEEP_D128_C[0], I.SWEEP_D128_C[4], I.GQA]


@pytest.mark.parametrize("w", FULL, ids=lambda w: w.name)
def test_bwd_full_size_one_complete_group(oracle, w):
    """Benchmark sizes.  The oracle runs one complete (batch, KV head) group: all N query rows of all
    G query heads of the group against all N keys, so dK and dV of EVERY key of the group are compared
    element by element, from the first key tile (the longest query loop: G N / 64 rounds, head
    switches included) to the last; dQ on sampled rows of the same group."""
    x = I.make_inputs(w)
    dq, dk, dv = gpu_fwd_bwd(w, x)
    for t in (dq, dk, dv):
        assert np.isfinite(t).all()
    G = w.H // w.Hkv
    b, kvh = w.B - 1, w.Hkv - 1
    hs = slice(kvh * G, (kvh + 1) * G)
    f = lambda name, heads: I.to_f64(x[name][b:b + 1, :, heads])
    rdq, rdk, rdv = oracle.attn_bwd(f("q", hs), f("k", slice(kvh, kvh + 1)), f("v", slice(kvh, kvh + 1)), f("do", hs),
                                    w.scale, w.causal)
    assert_close(dk[b:b + 1, :, kvh:kvh + 1], rdk, f"dK all keys {w.name}")
    assert_close(dv[b:b + 1, :, kvh:kvh + 1], rdv, f"dV all keys {w.name}")
    # the first key tile separately: its error must not hide in the norm of the whole group
    assert_close(dk[b:b + 1, :128, kvh:kvh + 1], rdk[:, :128], f"dK keys 0-127 {w.name}")
    assert_close(dv[b:b + 1, :128, kvh:kvh + 1], rdv[:, :128], f"dV keys 0-127 {w.name}")
    rng = np.random.default_rng(w.seed)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, 255, 256, w.N - 65, w.N - 64, w.N - 1],
                                     rng.integers(0, w.N, 24)]))
    assert_close(dq[b:b + 1, rows][:, :, hs], rdq[:, rows], f"dQ rows {w.name}")


def test_bwd_heavy_tailed_full_size(oracle):
    """The (192, 128) workload at N = 32768 with 1 % of the q, k entries multiplied by 8: one head with
    all 32768 query rows through the oracle (about a minute of CPU), dK and dV compared on the first
    256 keys and on 256 keys drawn at random, dQ on every row of the head; under the term-scaled gate,
    audited against the bf16-rounded definition (parity.py)."""
    w = I.MLA_OUTLIER
    x = I.make_inputs(w)
    dq, dk, dv = gpu_fwd_bwd(w, x)
    for t in (dq, dk, dv):
        assert np.isfinite(t).all()
    b, h = 0, w.H - 1
    kvh = h // (w.H // w.Hkv)
    f = lambda name, hh: I.to_f64(x[name][b:b + 1, :, hh:hh + 1])
    q, k, v, do = f("q", h), f("k", kvh), f("v", kvh), f("do", h)
    rdq, rdk, rdv = oracle.attn_bwd(q, k, v, do, w.scale, True)
    rng = np.random.default_rng(55)
    keys = np.unique(np.concatenate([np.arange(256), rng.integers(256, w.N, 256)]))
    # magnitudes of the summed terms and the bf16-rounded definition: dQ is separable by query row;
    # dK / dV of a key collect every later query row, accumulated over blocks of rows
    a_dk = np.zeros((w.N, w.dqk)); a_dv = np.zeros((w.N, w.dv)); a_dq = np.zeros((w.N, 1, w.dqk))
    r_dk = np.zeros((w.N, w.dqk)); r_dv = np.zeros((w.N, w.dv)); r_dq = np.zeros((w.N, 1, w.dqk))
    from parity import to_bf16
    for lo in range(0, w.N, 2048):
        r = np.arange(lo, lo + 2048)
        args = (q[0, r], k[0, :, 0], v[0, :, 0], do[0, r], w.scale, True)
        _, a_dq[r], ak, av = term_magnitudes(*args, q_pos=r)
        a_dk += ak; a_dv += av
        _, r_dq[r], rk, rv = rounded_reference(*args, q_pos=r, round_kv=False)
        r_dk += rk; r_dv += rv
    r_dk, r_dv = to_bf16(r_dk), to_bf16(r_dv)
    assert_close_terms(dk[b, keys, kvh], rdk[0, keys, 0], a_dk[keys], "dK first 256 + random 256 keys, heavy tails", r_dk[keys])
    assert_close_terms(dv[b, keys, kvh], rdv[0, keys, 0], a_dv[keys], "dV first 256 + random 256 keys, heavy tails", r_dv[keys])
    # every row: a relative Frobenius error over a few dozen rows of this workload is set by the two or three
    # rows whose softmax sits on one key (dS_ij = P_ij (dP_ij - D_i) cancels there and carries the whole
    # rounding error of D_i), so it is taken over the head
    assert_close_terms(dq[b, :, h:h + 1], rdq[0], a_dq, "dQ every row of one head, heavy tails", r_dq)
    # a ceiling on the plain maximum error next to the scaled gate: twice what the roundings the method
    # prescribes cost the definition itself on the same rows
    worst, worst_rounded = np.abs(dq[b, :, h:h + 1] - rdq[0]).max(), np.abs(r_dq - rdq[0]).max()
    assert worst <= 2.0 * worst_rounded, f"dQ max error {worst:.3e}, of the bf16-rounded definition {worst_rounded:.3e}"
