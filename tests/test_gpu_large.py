"""Tensors of more than 2^31 elements (4.4 GB each): element and byte offsets beyond 32 bits in
every kernel.  Inputs are drawn on the GPU (seeded); the oracle checks sampled query rows and the
last keys of the first and of the last (batch, head), whose data sit at the two ends of the
tensors."""
import numpy as np
import pytest
import torch

from parity import LSE_ABS, assert_close

pytestmark = pytest.mark.gpu


def test_offsets_beyond_32_bits(oracle):
    import paper_2603_05451_amd as A
    B, N, H, d = 33, 16384, 32, 128
    assert B * N * H * d > 2 ** 31
    if torch.cuda.mem_get_info()[0] < 80 * 2 ** 30:
        pytest.skip("needs about 60 GB of free device memory")
    g = torch.Generator(device="cuda").manual_seed(1234)
    draw = lambda: torch.randn((B, N, H, d), generator=g, device="cuda", dtype=torch.bfloat16)
    q, k, v, do = draw(), draw(), draw(), draw()
    scale, causal = 1.0 / np.sqrt(d), True
    o, lse = A.attn_fwd(q, k, v, scale, causal)
    dq, dk, dv = A.attn_bwd(q, k, v, o, do, lse, scale, causal)
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    for b, h in ((0, 0), (B - 1, H - 1), (B // 2, 5)):
        rows = np.unique(np.concatenate([[0, 127, 128, N - 1], rng.integers(0, N, 12), np.arange(N - 128, N)]))
        f = lambda t, r=slice(None): t[b, r, h].double().cpu().numpy()[None, :, None, :]
        ridx = torch.from_numpy(rows).cuda()
        fq, fdo = f(q, ridx), f(do, ridx)
        fk, fv = f(k), f(v)
        ro, rlse = oracle.attn_fwd(fq, fk, fv, scale, causal, q_pos=rows)
        rdq, rdk, rdv = oracle.attn_bwd(fq, fk, fv, fdo, scale, causal, q_pos=rows)
        tag = f"b{b} h{h}"
        assert_close(f(o, ridx), ro, "large O " + tag)
        assert np.abs(lse[b, h, ridx].cpu().numpy()[None, None] - rlse).max() <= LSE_ABS
        assert_close(f(dq, ridx), rdq, "large dQ " + tag)
        # under the causal mask only the last 128 queries reach the last 128 keys: complete sums
        last = slice(N - 128, N)
        assert_close(f(dk, last), rdk[:, N - 128:], "large dK " + tag)
        assert_close(f(dv, last), rdv[:, N - 128:], "large dV " + tag)

    # the same data as a packed batch of 33 equal sequences: the variable-length kernels, with their
    # own offset arithmetic.  Forward: the packed call runs 128-query blocks, attn_fwd at this length
    # the kernel with 64 queries per wave (another summation order): one bf16 ulp.  Backward: the
    # same dK/dV kernel on the same tiles, from the same O and LSE: the same bits; dQ see below.
    del rdq, rdk, rdv, ro
    T = B * N
    cu = torch.arange(0, T + 1, N, dtype=torch.int32, device="cuda")
    p = lambda t: t.reshape(T, H, d)
    ov, lsev = A.attn_varlen_fwd(p(q), p(k), p(v), cu, scale, causal)
    torch.cuda.synchronize()
    for lo in range(0, T, T // 33):
        a, b_ = ov[lo:lo + T // 33].float(), p(o)[lo:lo + T // 33].float()
        assert ((a - b_).abs() <= 2.0 ** -7 * b_.abs() + 1e-6).all()
    assert (lsev.reshape(H, B, N).permute(1, 0, 2) - lse).abs().max().item() <= 2e-5
    del ov, lsev
    lse_packed = lse.permute(1, 0, 2).reshape(H, T).contiguous()
    gq, gk, gv = A.attn_varlen_bwd(p(q), p(k), p(v), p(o), p(do), lse_packed, cu, scale, causal)
    torch.cuda.synchronize()
    assert torch.equal(gk, p(dk)) and torch.equal(gv, p(dv))
    # dQ: attn_bwd runs the kernel with 64 queries per wave at this length, whose dP accumulators start from
    # -D (fp32 rounding of dP - D, i.e. now and then one ulp of a dS element): compared in slices to bound
    # the memory of the float copies
    for lo in range(0, T, T // 33):
        a, b_ = gq[lo:lo + T // 33].float(), p(dq)[lo:lo + T // 33].float()
        assert ((a - b_).abs() <= 2.0 ** -7 * torch.maximum(a.abs(), b_.abs()) + 2e-3).all()
