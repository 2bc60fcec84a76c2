"""Pins for the CPU fp64 oracle: closed forms, invariants, finite differences, library cross-check.

None of these retype the oracle's own formula: each one states a fact that the
definition of attention (paper Sec. 2.1) implies and that a dropped term, a wrong
sign, index or transposed operand in the oracle would break.
"""
import numpy as np
import pytest
import torch

RNG = np.random.default_rng(1234)


def rnd(*shape):
    return RNG.standard_normal(shape)


# --------------------------------------------------------------------------- forward closed forms

@pytest.mark.parametrize("causal", [False, True])
def test_identical_keys_give_mean_of_v(oracle, causal):
    # All keys equal => every visible key has the same score => uniform P =>
    # O_i is the (prefix) mean of V and LSE_i = scale q_i.kbar + ln(n_i).
    B, N, H, Hkv, dqk, dv = 2, 13, 4, 2, 6, 5
    q, v = rnd(B, N, H, dqk), rnd(B, N, Hkv, dv)
    kbar = rnd(B, 1, Hkv, dqk)
    k = np.broadcast_to(kbar, (B, N, Hkv, dqk)).copy()
    scale = 0.37
    o, lse = oracle.attn_fwd(q, k, v, scale, causal)
    G = H // Hkv
    for b in range(B):
        for h in range(H):
            for i in range(N):
                n = i + 1 if causal else N
                np.testing.assert_allclose(o[b, i, h], v[b, :n, h // G].mean(0), rtol=0, atol=1e-13)
                want = scale * q[b, i, h] @ kbar[b, 0, h // G] + np.log(n)
                assert abs(lse[b, h, i] - want) < 1e-12
    # and the softmax Jacobian annihilates constants: sum_j dS_ij = 0 => dQ = 0 exactly-ish
    dq, dk, dvv = oracle.attn_bwd(q, k, v, rnd(B, N, H, dv), scale, causal)
    assert np.abs(dq).max() < 1e-13


def test_dominant_logit_selects_its_v_row(oracle):
    # One key aligned with q and very long: its score exceeds all others by a gap g,
    # so ||O_i - V_j*|| <= 2 (n-1) e^{-g} max|V| and S_ij* <= LSE_i <= S_ij* + (n-1) e^{-g}.
    N, d, dv = 9, 4, 3
    q = np.zeros((1, N, 1, d)); k = np.zeros((1, N, 1, d)); v = rnd(1, N, 1, dv)
    for i in range(N):
        q[0, i, 0, i % d] = 1.0
    k[0] = 0.1 * rnd(N, 1, d)
    jstar = [(3 * i + 1) % N for i in range(N)]
    # query i has its unit entry at i % d; give key jstar(i) a large entry there.  Queries
    # that share a coordinate would collide, so handle one query row per call.
    for i in range(N):
        kk = k.copy()
        kk[0, jstar[i], 0, i % d] = 60.0
        o, lse = oracle.attn_fwd(q, kk, v, 1.0, False)
        s = kk[0, :, 0, :] @ q[0, i, 0]
        g = s[jstar[i]] - np.delete(s, jstar[i]).max()
        assert g > 50
        bound = 2 * (N - 1) * np.exp(-g) * np.abs(v).max()
        assert np.abs(o[0, i, 0] - v[0, jstar[i], 0]).max() <= bound + 1e-15
        assert s[jstar[i]] - 1e-12 <= lse[0, 0, i] <= s[jstar[i]] + (N - 1) * np.exp(-g) + 1e-12


def test_single_key_and_causal_first_row(oracle):
    # N = 1 (or causal row 0): P = [1] => O = V_0, LSE = S_00; backward: dV_0 gets dO_0,
    # dS = 0 => that row adds nothing to dQ or dK.
    q, k, v, do = rnd(1, 1, 2, 3), rnd(1, 1, 1, 3), rnd(1, 1, 1, 4), rnd(1, 1, 2, 4)
    o, lse = oracle.attn_fwd(q, k, v, 0.7, False)
    np.testing.assert_allclose(o[0, 0, 0], v[0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(lse[0, :, 0], 0.7 * q[0, 0] @ k[0, 0, 0], atol=1e-14)
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, 0.7, False)
    assert np.abs(dq).max() == 0 and np.abs(dk).max() == 0
    np.testing.assert_allclose(dvv[0, 0, 0], do[0, 0].sum(0), atol=1e-15)
    # causal row 0 of a longer sequence
    N = 5
    q, k, v = rnd(1, N, 1, 3), rnd(1, N, 1, 3), rnd(1, N, 1, 2)
    o, lse = oracle.attn_fwd(q, k, v, 1.3, True)
    np.testing.assert_allclose(o[0, 0, 0], v[0, 0, 0], atol=1e-15)
    assert abs(lse[0, 0, 0] - 1.3 * q[0, 0, 0] @ k[0, 0, 0]) < 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_p_rows_sum_to_one_via_ones_column(oracle, causal):
    # Append a column of ones to V: that output column is sum_j P_ij, which must be 1.
    # With V = one-hot rows, O reproduces P itself, so P >= 0 and the causal zero pattern show.
    N, d = 11, 5
    q, k = rnd(2, N, 2, d), rnd(2, N, 2, d)
    v = np.concatenate([rnd(2, N, 2, 3), np.ones((2, N, 2, 1))], -1)
    o, _ = oracle.attn_fwd(q, k, v, 0.4, causal)
    np.testing.assert_allclose(o[..., -1], 1.0, atol=1e-14)
    eye = np.broadcast_to(np.eye(N)[None, :, None, :], (2, N, 2, N)).copy()
    P, lse = oracle.attn_fwd(q, k, eye, 0.4, causal)     # P[b,i,h,j]
    assert (P >= 0).all()
    if causal:
        iu = np.triu_indices(N, 1)
        assert np.abs(P[:, iu[0], :, iu[1]]).max() == 0.0
    # LSE consistency: P_ij = exp(S_ij - LSE_i) for a visible entry
    b, h, i, j = 1, 0, N - 1, 2
    s = 0.4 * q[b, i, h] @ k[b, j, h]
    assert abs(P[b, i, h, j] - np.exp(s - lse[b, h, i])) < 1e-14


# --------------------------------------------------------------------------- q = 0 closed forms

@pytest.mark.parametrize("causal", [False, True])
def test_zero_queries_closed_form(oracle, causal):
    # S = 0 => P uniform over n_i visible keys.  Then LSE = ln n_i, dK = 0 (it multiplies q),
    # dV_j = sum_{i sees j} dO_i / n_i, and dQ_i = (scale / n_i) sum_j (dP_ij - mean_j dP_ij) k_j.
    N, d, dv, scale = 7, 3, 4, 0.9
    q = np.zeros((1, N, 1, d)); k, v, do = rnd(1, N, 1, d), rnd(1, N, 1, dv), rnd(1, N, 1, dv)
    o, lse = oracle.attn_fwd(q, k, v, scale, causal)
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, scale, causal)
    assert np.abs(dk).max() == 0.0
    want_dv = np.zeros((N, dv)); want_dq = np.zeros((N, d))
    for i in range(N):
        n = i + 1 if causal else N
        assert abs(lse[0, 0, i] - np.log(n)) < 1e-14
        want_dv[:n] += do[0, i, 0] / n
        dp = v[0, :n, 0] @ do[0, i, 0]
        want_dq[i] = scale / n * ((dp - dp.mean()) @ k[0, :n, 0])
    np.testing.assert_allclose(dvv[0, :, 0], want_dv, atol=1e-13)
    np.testing.assert_allclose(dq[0, :, 0], want_dq, atol=1e-13)


# --------------------------------------------------------------------------- invariances

def test_key_shift_value_scale_and_permutation(oracle):
    N, d, dv, scale = 10, 4, 3, 0.6
    q, k, v, do = rnd(1, N, 2, d), rnd(1, N, 2, d), rnd(1, N, 2, dv), rnd(1, N, 2, dv)
    o, lse = oracle.attn_fwd(q, k, v, scale, False)
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, scale, False)
    # adding the same vector c to every key shifts each row of S by scale q_i.c: P, O unchanged
    c = rnd(1, 1, 2, d)
    o2, lse2 = oracle.attn_fwd(q, k + c, v, scale, False)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(lse2 - lse, scale * np.einsum("bihc,bhc->bhi", q, c[:, 0]), atol=1e-12)
    # joint permutation of key/value rows: O unchanged, dK and dV permuted the same way
    perm = RNG.permutation(N)
    o3, _ = oracle.attn_fwd(q, k[:, perm], v[:, perm], scale, False)
    dq3, dk3, dv3 = oracle.attn_bwd(q, k[:, perm], v[:, perm], do, scale, False)
    np.testing.assert_allclose(o3, o, atol=1e-13)
    np.testing.assert_allclose(dq3, dq, atol=1e-13)
    np.testing.assert_allclose(dk3, dk[:, perm], atol=1e-13)
    np.testing.assert_allclose(dv3, dvv[:, perm], atol=1e-13)
    # V -> a V scales O, dQ, dK by a and leaves dV alone
    dq4, dk4, dv4 = oracle.attn_bwd(q, k, 3.0 * v, do, scale, False)
    np.testing.assert_allclose(dq4, 3.0 * dq, atol=1e-12)
    np.testing.assert_allclose(dk4, 3.0 * dk, atol=1e-12)
    np.testing.assert_allclose(dv4, dvv, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_softmax_jacobian_identities(oracle, causal):
    # (a) D identity: with K = 0 column trick we cannot read dS directly, so use linearity:
    # dQ is linear in K's role as the right factor of dS K.  Setting K' = K for scores but reading
    # sum_j dS_ij needs K rows = ones; instead check sum_j dS_ij = 0 through a shifted copy:
    # dQ(K + c) - dQ(K) = scale (sum_j dS_ij) c = 0 because P (hence dS) is shift invariant.
    N, d, dv, scale = 9, 4, 5, 0.8
    q, k, v, do = rnd(1, N, 1, d), rnd(1, N, 1, d), rnd(1, N, 1, dv), rnd(1, N, 1, dv)
    c = rnd(1, 1, 1, d)
    dq, _, _ = oracle.attn_bwd(q, k, v, do, scale, causal)
    dq2, _, _ = oracle.attn_bwd(q, k + c, v, do, scale, causal)
    np.testing.assert_allclose(dq2, dq, atol=1e-12)
    # (b) adding a constant vector u to every V row adds dO_i.u to every dP_ij of row i, which
    # the Jacobian removes: dQ and dK must not change.
    u = rnd(1, 1, 1, dv)
    dq3, dk3, _ = oracle.attn_bwd(q, k, v + u, do, scale, causal)
    _, dk, _ = oracle.attn_bwd(q, k, v, do, scale, causal)
    np.testing.assert_allclose(dq3, dq, atol=1e-12)
    np.testing.assert_allclose(dk3, dk, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv(oracle):
    B, N, H, Hkv, d, dv = 2, 8, 6, 2, 4, 3
    G = H // Hkv
    q, k, v, do = rnd(B, N, H, d), rnd(B, N, Hkv, d), rnd(B, N, Hkv, dv), rnd(B, N, H, dv)
    krep, vrep = np.repeat(k, G, axis=2), np.repeat(v, G, axis=2)
    for causal in (False, True):
        o, lse = oracle.attn_fwd(q, k, v, 0.5, causal)
        o2, lse2 = oracle.attn_fwd(q, krep, vrep, 0.5, causal)
        np.testing.assert_array_equal(o, o2)
        np.testing.assert_array_equal(lse, lse2)
        dq, dk, dvv = oracle.attn_bwd(q, k, v, do, 0.5, causal)
        dq2, dk2, dv2 = oracle.attn_bwd(q, krep, vrep, do, 0.5, causal)
        np.testing.assert_array_equal(dq, dq2)
        np.testing.assert_allclose(dk, dk2.reshape(B, N, Hkv, G, d).sum(3), atol=1e-13)
        np.testing.assert_allclose(dvv, dv2.reshape(B, N, Hkv, G, dv).sum(3), atol=1e-13)


def test_q_pos_subset_matches_full_rows(oracle):
    # Passing a subset of query rows with their true positions must reproduce those rows.
    N, d, dv = 12, 3, 4
    q, k, v, do = rnd(1, N, 2, d), rnd(1, N, 1, d), rnd(1, N, 1, dv), rnd(1, N, 2, dv)
    rows = np.array([0, 3, 7, 11])
    for causal in (False, True):
        o, lse = oracle.attn_fwd(q, k, v, 0.5, causal)
        o_s, lse_s = oracle.attn_fwd(q[:, rows], k, v, 0.5, causal, q_pos=rows)
        np.testing.assert_array_equal(o_s, o[:, rows])
        np.testing.assert_array_equal(lse_s, lse[:, :, rows])
        dq, dk, dvv = oracle.attn_bwd(q, k, v, do, 0.5, causal)
        dq_s, _, _ = oracle.attn_bwd(q[:, rows], k, v, do[:, rows], 0.5, causal, q_pos=rows)
        np.testing.assert_array_equal(dq_s, dq[:, rows])
    # causal: the last n keys only receive gradient from the last n rows
    n = 4
    tail = np.arange(N - n, N)
    _, dk_t, dv_t = oracle.attn_bwd(q[:, tail], k, v, do[:, tail], 0.5, True, q_pos=tail)
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, 0.5, True)
    np.testing.assert_allclose(dk_t[:, tail], dk[:, tail], atol=1e-14)
    np.testing.assert_allclose(dv_t[:, tail], dvv[:, tail], atol=1e-14)


# --------------------------------------------------------------------------- finite differences

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 1, 6, 4, 3), (2, 4, 2, 5, 3, 3)])
def test_backward_matches_central_differences(oracle, causal, shape):
    # L(q,k,v) = sum(O * dO); dL/dq, dL/dk, dL/dv by central differences in fp64.
    B, H, Hkv, N, d, dv = shape
    q, k, v, do = rnd(B, N, H, d), rnd(B, N, Hkv, d), rnd(B, N, Hkv, dv), rnd(B, N, H, dv)
    scale = 0.55
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, scale, causal)

    def loss(q_, k_, v_):
        o, _ = oracle.attn_fwd(q_, k_, v_, scale, causal)
        return float((o * do).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dvv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            num[idx] = (loss(args_p["q"], args_p["k"], args_p["v"]) -
                        loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
        err = np.abs(num - g).max() / max(np.abs(g).max(), 1e-30)
        assert err < 1e-7, (name, err)


# --------------------------------------------------------------------------- library cross-check

@pytest.mark.parametrize("causal", [False, True])
def test_against_torch_fp64_softmax_and_autograd(oracle, causal):
    # Special case that reduces to library routines: torch.softmax + autograd in fp64.
    B, H, Hkv, N, d, dv = 2, 4, 2, 33, 16, 8
    G = H // Hkv
    q, k, v, do = rnd(B, N, H, d), rnd(B, N, Hkv, d), rnd(B, N, Hkv, dv), rnd(B, N, H, dv)
    scale = 1 / np.sqrt(d)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    kk = tk.repeat_interleave(G, dim=2); vv = tv.repeat_interleave(G, dim=2)
    s = torch.einsum("bihc,bjhc->bhij", tq, kk) * scale
    if causal:
        s = s.masked_fill(torch.ones(N, N, dtype=torch.bool).triu(1), float("-inf"))
    p = torch.softmax(s, -1)
    to = torch.einsum("bhij,bjhc->bihc", p, vv)
    tlse = torch.logsumexp(s, -1)
    (to * torch.tensor(do)).sum().backward()
    o, lse = oracle.attn_fwd(q, k, v, scale, causal)
    dq, dk, dvv = oracle.attn_bwd(q, k, v, do, scale, causal)
    np.testing.assert_allclose(o, to.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(lse, tlse.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dvv, tv.grad.numpy(), atol=1e-13)


# --------------------------------------------------------------------------- tiled recurrences, Sec. 3.1.4

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("tau", [0.0, 8 * np.log(2.0), np.inf])
def test_thresholded_online_softmax_is_exact(oracle, causal, tau):
    # The tiled recurrences with a stale reference maximum must give the plain result for any
    # tau >= 0; LSE must be reference + ln(l) (using the true maximum there would fail here).
    B, H, Hkv, N, d, dv = 1, 2, 1, 70, 8, 5
    q, k, v = rnd(B, N, H, d), rnd(B, N, Hkv, d), rnd(B, N, Hkv, dv)
    # make logits grow along the sequence so later tiles exceed earlier maxima by > 8 ln 2
    k *= np.linspace(0.2, 6.0, N)[None, :, None, None]
    scale = 1.0
    o, lse = oracle.attn_fwd(q, k, v, scale, causal)
    for tile in (1, 7, 16, 64, 128):
        o2, lse2, nres = oracle.attn_fwd_online(q, k, v, scale, causal, tile, tau)
        np.testing.assert_allclose(o2, o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse2, lse, rtol=0, atol=1e-11)
        if tau == np.inf:
            assert nres.sum() == 0
    # both branches are exercised at the paper's threshold
    _, _, n8 = oracle.attn_fwd_online(q, k, v, scale, causal, 7, 8 * np.log(2.0))
    _, _, n0 = oracle.attn_fwd_online(q, k, v, scale, causal, 7, 0.0)
    assert 0 < n8.sum() < n0.sum()


def test_bad_arguments_are_rejected(oracle):
    q, k, v = rnd(1, 4, 3, 2), rnd(1, 4, 2, 2), rnd(1, 4, 2, 2)   # H % Hkv != 0
    with pytest.raises(RuntimeError):
        oracle.attn_fwd(q, k, v, 1.0, False)
    with pytest.raises(RuntimeError):   # a causal row that sees no key
        oracle.attn_fwd(rnd(1, 2, 1, 2), rnd(1, 4, 1, 2), rnd(1, 4, 1, 2), 1.0, True,
                        q_pos=np.array([-1, 0]))
