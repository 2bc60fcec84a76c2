"""GPU parity of the forward pass against the CPU fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2603_05451_amd import inputs as I
from parity import LSE_ABS, assert_close, assert_close_terms, rounded_reference, term_magnitudes

pytestmark = pytest.mark.gpu


def gpu_fwd(w, x):
    import paper_2603_05451_amd as A
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    torch.cuda.synchronize()
    return o.float().cpu().numpy(), lse.cpu().numpy()


SMALL = [
    I.CANARY,
    I.Workload("s_d64_c", 2, 4, 2, 384, 64, 64, True, 11),
    I.Workload("s_d64_nc", 1, 3, 1, 256, 64, 64, False, 12),
    I.Workload("s_d96_c", 2, 4, 2, 384, 96, 96, True, 18),
    I.Workload("s_d96_nc", 1, 3, 3, 640, 96, 96, False, 19),
    I.Workload("s_d128_nc", 2, 4, 4, 384, 128, 128, False, 13),
    I.Workload("s_d128_c", 2, 4, 2, 640, 128, 128, True, 14),
    I.Workload("s_d256_c", 1, 4, 2, 384, 256, 256, True, 10),
    I.Workload("s_d256_nc", 2, 2, 2, 256, 256, 256, False, 9),
    I.Workload("s_d192_c", 1, 4, 2, 384, 192, 128, True, 15),
    I.Workload("s_d192_nc", 1, 2, 2, 256, 192, 128, False, 16),
    I.Workload("s_d192_c_outl", 1, 2, 1, 512, 192, 128, True, 17, outlier_frac=0.01),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_fwd_small_full_parity(oracle, w):
    x = I.make_inputs(w, with_do=False)
    o, lse = gpu_fwd(w, x)
    ro, rlse = oracle.attn_fwd(I.to_f64(x["q"]), I.to_f64(x["k"]), I.to_f64(x["v"]), w.scale, w.causal)
    if w.outlier_frac:
        G = w.H // w.Hkv
        for b in range(w.B):
            for kvh in range(w.Hkv):
                hs = slice(kvh * G, (kvh + 1) * G)
                args = (I.to_f64(x["q"][b, :, hs]), I.to_f64(x["k"][b, :, kvh]), I.to_f64(x["v"][b, :, kvh]),
                        np.zeros((w.N, G, w.dv)), w.scale, w.causal)
                assert_close_terms(o[b, :, hs], ro[b, :, hs], term_magnitudes(*args)[0], f"O {w.name} b{b} kvh{kvh}",
                                   rounded_reference(*args)[0])
    else:
        assert_close(o, ro, f"O {w.name}")
    assert np.abs(lse - rlse).max() <= LSE_ABS, f"LSE {w.name}: {np.abs(lse - rlse).max():.3e}"


FULL = [I.TARGET, I.SWEEP_D64_NC[0], I.SWEEP_D64_NC[5], I.SWEEP_D128_C[0], I.SWEEP_D128_C[4], I.GQA,
        I.MLA_OUTLIER]


@pytest.mark.parametrize("w", FULL, ids=lambda w: w.name)
def test_fwd_full_size_sampled_rows(oracle, w):
    """At the benchmark sizes the oracle computes sampled query rows one by one (all keys)."""
    x = I.make_inputs(w, with_do=False)
    o, lse = gpu_fwd(w, x)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    rng = np.random.default_rng(w.seed)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, 255, 256, w.N - 257, w.N - 256, w.N - 129, w.N - 128, w.N - 1],
                                     rng.integers(0, w.N, 48)]))
    G = w.H // w.Hkv
    for b, kvh in {(0, 0), (w.B - 1, w.Hkv - 1)}:
        hs = slice(kvh * G, (kvh + 1) * G)
        q = I.to_f64(x["q"][b:b + 1, :, hs][:, rows])
        k = I.to_f64(x["k"][b:b + 1, :, kvh:kvh + 1])
        v = I.to_f64(x["v"][b:b + 1, :, kvh:kvh + 1])
        ro, rlse = oracle.attn_fwd(q, k, v, w.scale, w.causal, q_pos=rows)
        if w.outlier_frac:
            args = (q[0], k[0, :, 0], v[0, :, 0], np.zeros((len(rows), G, w.dv)), w.scale, w.causal)
            assert_close_terms(o[b, :, hs][rows], ro[0], term_magnitudes(*args, q_pos=rows)[0],
                               f"O rows {w.name} b{b} kvh{kvh}", rounded_reference(*args, q_pos=rows)[0])
        else:
            assert_close(o[b:b + 1, :, hs][:, rows], ro, f"O rows {w.name} b{b} kvh{kvh}")
        err = np.abs(lse[b:b + 1, hs][:, :, rows] - rlse).max()
        assert err <= LSE_ABS, f"LSE {w.name}: {err:.3e}"


Q64 = [I.Workload("q64_nc_2048", 1, 3, 1, 2048, 128, 128, False, 31),
       I.Workload("q64_nc_2304", 2, 2, 2, 2304, 128, 128, False, 32),
       I.Workload("q64_d64_nc_8192", 1, 2, 1, 8192, 64, 64, False, 33),
       I.Workload("q64_d64_c_16384", 1, 1, 1, 16384, 64, 64, True, 34),
       I.Workload("q64_d192_nc_2304", 1, 3, 1, 2304, 192, 128, False, 35),
       I.Workload("q64_d192_c_8192", 1, 2, 2, 8192, 192, 128, True, 36)]


@pytest.mark.parametrize("w", Q64, ids=lambda w: w.name)
def test_fwd_64_queries_per_wave_full_parity(oracle, w):
    """Shapes that run the kernel with 64 queries per wave (N % 256 = 0; d = 128 and (192, 128) from
    N = 2048 without a mask and N = 8192 with it, d = 64 from N = 8192 without and N = 16384 with the mask),
    small enough for the oracle to compute every row: 8 to 64 query blocks of 256, GQA and MHA, key loops
    of 32 to 256 tiles."""
    x = I.make_inputs(w, with_do=False)
    o, lse = gpu_fwd(w, x)
    ro, rlse = oracle.attn_fwd(I.to_f64(x["q"]), I.to_f64(x["k"]), I.to_f64(x["v"]), w.scale, w.causal)
    assert_close(o, ro, f"O {w.name}")
    assert np.abs(lse - rlse).max() <= LSE_ABS, f"LSE {w.name}: {np.abs(lse - rlse).max():.3e}"


@pytest.mark.parametrize("causal,N,d,dv", [(False, 2048, 128, 128), (True, 8192, 128, 128), (False, 8192, 64, 64), (True, 16384, 64, 64),
                                           (False, 2048, 192, 128), (True, 8192, 192, 128)])
def test_fwd_growing_scores_restart_with_exact_maxima(oracle, causal, N, d, dv):
    """Scores that grow along the key axis by hundreds of binary orders: relative to the first
    tile's maximum the exponentials overflow, so the pipelined loop of the 64-queries-per-wave
    kernel cannot produce these results; they come from its restart with a row maximum per tile
    and the thresholded rescale (paper Sec. 3.1.4).  Compared on sampled rows."""
    import paper_2603_05451_amd as A
    g = torch.Generator("cpu").manual_seed(77)
    H = 2
    q = torch.randn(1, N, H, d, generator=g).abs().to(torch.bfloat16)
    k = (torch.randn(1, N, 1, d, generator=g).abs() * torch.linspace(0.2, 30.0, N).view(1, N, 1, 1)).to(torch.bfloat16)
    v = torch.randn(1, N, 1, dv, generator=g).to(torch.bfloat16)
    scale = d ** -0.5
    o, lse = A.attn_fwd(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    torch.cuda.synchronize()
    o, lse = o.float().cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 255, 256, N - 257, N - 1], rng.integers(0, N, 40)]))
    ro, rlse = oracle.attn_fwd(I.to_f64(q[:, rows]), I.to_f64(k), I.to_f64(v), scale, causal, q_pos=rows)
    assert_close(o[:, rows], ro, f"O growing scores causal={causal}")
    err = np.abs(lse[:, :, rows] - rlse).max()
    assert err <= LSE_ABS, f"LSE growing scores: {err:.3e} (values up to {np.abs(rlse).max():.0f})"


@pytest.mark.parametrize("causal,N,d,dv", [(False, 4096, 128, 128), (True, 8192, 192, 128), (False, 8192, 64, 64)])
def test_fwd_reference_steps_inside_the_pipelined_loop(oracle, causal, N, d, dv):
    """Scores that climb along the key axis by about 300 binary orders in small steps: relative to the first
    tile's maximum the tile sums pass 2^90 several times without ever becoming infinite, so the kernel
    with 64 queries per wave must raise its reference inside the pipelined loop (the rescale of paper
    Sec. 3.1.4 with a power-of-two step); no second pass is involved.  Every 37th row against the oracle."""
    import paper_2603_05451_amd as A
    g = torch.Generator("cpu").manual_seed(78)
    H = 2
    climb = torch.linspace(0.0, 300.0 / (1.4427 * d ** 0.5), N).view(1, N, 1, 1)         # score = sqrt(d) * climb
    q = (1.0 + 0.1 * torch.randn(1, N, H, d, generator=g)).to(torch.bfloat16)
    k = (climb + 0.1 * torch.randn(1, N, 1, d, generator=g)).to(torch.bfloat16)
    v = torch.randn(1, N, 1, dv, generator=g).to(torch.bfloat16)
    scale = d ** -0.5
    o, lse = A.attn_fwd(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    torch.cuda.synchronize()
    o, lse = o.float().cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    rows = np.unique(np.concatenate([[0, 1, 255, 256, N - 257, N - 1], np.arange(5, N, 37)]))
    ro, rlse = oracle.attn_fwd(I.to_f64(q[:, rows]), I.to_f64(k), I.to_f64(v), scale, causal, q_pos=rows)
    assert_close(o[:, rows], ro, f"O climbing scores causal={causal} d={d}")
    err = np.abs(lse[:, :, rows] - rlse).max()
    assert err <= LSE_ABS * max(1.0, np.abs(rlse).max() / 64), f"LSE climbing scores: {err:.3e} (values up to {np.abs(rlse).max():.0f})"
