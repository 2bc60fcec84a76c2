"""attn_bwd_noalloc (the backward pass with the workspace inside the library's device image, for
callers that cannot allocate) against attn_bwd_ex: the same bits, on two calls in a row, the second
with a smaller input, both through the C ABI."""
import pytest
import torch

from paper_2603_05451_amd import inputs as I

pytestmark = pytest.mark.gpu


def _both(w):
    import paper_2603_05451_amd as A
    x = I.make_inputs(w)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    ref = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
    got = [torch.full_like(t, float("nan")) for t in (q, k, v)]
    A.attn_bwd_noalloc(q, k, v, o, do, lse, w.scale, w.causal, *got)
    torch.cuda.synchronize()
    return ref, got


def test_noalloc_backward_equals_attn_bwd_on_two_calls_in_a_row():
    first = I.Workload("noalloc_a", 2, 8, 2, 1024, 128, 128, True, 61)        # 16 384 rows of workspace
    second = I.Workload("noalloc_b", 1, 2, 2, 384, 64, 64, False, 62)         # 768 rows: a smaller call after it
    for w in (first, second):
        ref, got = _both(w)
        for name, a, b in zip(("dq", "dk", "dv"), got, ref):
            assert torch.isfinite(a.float()).all(), f"{w.name} {name}"
            assert torch.equal(a, b), f"{w.name} {name}: differs from attn_bwd"


def test_noalloc_backward_rejects_sizes_beyond_its_workspace():
    import paper_2603_05451_amd as A
    B, H, N, d = 1, 16, 131072, 64                      # 2^21 rows > ATTN_NOALLOC_MAX_ROWS
    assert B * H * N > A.ATTN_NOALLOC_MAX_ROWS
    t = torch.zeros(1, 128, 1, d, dtype=torch.bfloat16, device="cuda")   # never read: the call must refuse first
    q = t.as_strided((B, N, H, d), (0, 0, 0, 1))
    lse = torch.zeros(1, device="cuda").as_strided((B, H, N), (0, 0, 0))
    rc = A.lib().attn_bwd_noalloc(*(t.data_ptr(),) * 5, lse.data_ptr(), *(t.data_ptr(),) * 3,
                                  B, H, H, N, d, d, 0.125, 0, None)
    assert rc == -4 and b"ATTN_NOALLOC_MAX_ROWS" in A.lib().attn_strerror(rc)
