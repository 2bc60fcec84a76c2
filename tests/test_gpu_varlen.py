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
    ("d96_c", LENGTHS_A, 4, 2, 96, 96, True, 37),
    ("d96_nc", LENGTHS_B, 2, 2, 96, 96, False, 38),
    ("d128_nc", LENGTHS_A, 4, 1, 128, 128, False, 33),
    ("d128_c", LENGTHS_A, 4, 2, 128, 128, True, 34),
    ("d192_c", LENGTHS_B, 2, 1, 192, 128, True, 35),
    ("d256_c", LENGTHS_A, 2, 1, 256, 256, True, 39),
    ("d256_nc", LENGTHS_B, 2, 2, 256, 256, False, 40),
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


def _fixed_and_packed_fwd(B, N, causal):
    import paper_2603_05451_amd as A
    w = I.Workload("eq", B, 4, 2, N, 128, 128, causal, 41)
    x = I.make_inputs(w, with_do=False)
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
    cu = torch.arange(0, (w.B + 1) * w.N, w.N, dtype=torch.int32, device="cuda")
    T = w.B * w.N
    ov, lsev = A.attn_varlen_fwd(q.reshape(T, w.H, w.dqk), k.reshape(T, w.Hkv, w.dqk), v.reshape(T, w.Hkv, w.dv),
                                 cu, w.scale, w.causal)
    torch.cuda.synchronize()
    return o, lse, ov.reshape(o.shape), lsev.reshape(w.H, w.B, w.N).permute(1, 0, 2)


@pytest.mark.parametrize("B,N,causal", [(3, 384, True), (2, 1024, False), (1, 4096, True)])
def test_varlen_fwd_equals_fixed_length_bitwise(B, N, causal):
    """Equal lengths that are multiples of 128, at sizes where attn_fwd runs its 128-query blocks:
    the packed call must reproduce attn_fwd bit for bit (same tiles, same order of operations per
    wave)."""
    o, lse, ov, lsev = _fixed_and_packed_fwd(B, N, causal)
    assert torch.equal(ov, o)
    assert torch.equal(lsev, lse)


@pytest.mark.parametrize("B,N,causal", [(2, 2048, False), (1, 8192, True)])
def test_varlen_fwd_matches_fixed_length_on_long_sequences(B, N, causal):
    """From N = 2048 without a mask and N = 8192 with the causal mask attn_fwd runs the kernel with 64
    queries per wave, whose row sums are taken in another order and whose reference maximum is that
    of the first tile; the packed call keeps 128-query blocks.  Same mathematics, two roundings:
    O agrees within one bf16 ulp, LSE to fp32 rounding."""
    o, lse, ov, lsev = _fixed_and_packed_fwd(B, N, causal)
    o, ov = o.float(), ov.float()
    assert ((o - ov).abs() <= 2.0 ** -7 * o.abs() + 1e-6).all(), (o - ov).abs().max().item()
    assert (lse - lsev).abs().max().item() <= 2e-5


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
    """Equal lengths that are multiples of 128: the packed call runs the same kernels on the same
    tiles, so from the same O and LSE its dQ, dK and dV are bit-identical to attn_bwd; two packed
    calls give identical bits.  Last two cases: the fixed-length call runs the kernels with one wave per
    SIMD (d = 128; N >= 1024 without a mask, the dQ kernel also under the causal mask from N = 4096).
    Their dK and dV are the same bits; their dQ kernel starts the dP
    accumulators from -D instead of adding it afterwards, so its dQ may differ from the packed call's by
    the fp32 rounding of dP - D where that flips the 16-bit rounding of a dS element: a minority of
    the elements, each by about one ulp (relative Frobenius distance under 1e-3)."""
    import paper_2603_05451_amd as A
    for dqk, dv_, seed, N, causal in ((128, 128, 42, 384, True), (64, 64, 43, 384, True), (192, 128, 44, 384, True),
                                      (128, 128, 45, 4096, False), (128, 128, 46, 4096, True)):   # the last two: 64 queries per wave
        w = I.Workload("eq", 2 if N < 1024 else 1, 4, 2, N, dqk, dv_, causal, seed)
        x = I.make_inputs(w)
        q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
        o, lse = A.attn_fwd(q, k, v, w.scale, w.causal)
        ref = A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal)
        cu = torch.arange(0, (w.B + 1) * w.N, w.N, dtype=torch.int32, device="cuda")
        T = w.B * w.N
        p = lambda t: t.reshape(T, *t.shape[2:])
        # the same O and LSE for both (at N = 4096 the two forward calls run different kernels)
        ov, lsev = p(o), lse.permute(1, 0, 2).reshape(w.H, T).contiguous()
        r1 = A.attn_varlen_bwd(p(q), p(k), p(v), ov, p(do), lsev, cu, w.scale, w.causal)
        r2 = A.attn_varlen_bwd(p(q), p(k), p(v), ov, p(do), lsev, cu, w.scale, w.causal)
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(r1, r2))
        if N < 1024:
            assert all(torch.equal(a.reshape(b.shape), b) for a, b in zip(r1, ref)), (dqk, dv_)
        else:
            assert all(torch.equal(a.reshape(b.shape), b) for a, b in zip(r1[1:], ref[1:]))
            a, b = r1[0].reshape(ref[0].shape).float(), ref[0].float()
            # one ulp of the result, plus what one ulp of one dS element (|dS| up to about 0.5, |k| up to about 4,
            # scale 128 ** -0.5) moves the sum: 2 ** -8 * 0.5 * 4 * 0.088 = 7e-4
            assert ((a - b).abs() <= 2.0 ** -7 * torch.maximum(a.abs(), b.abs()) + 2e-3).all(), (a - b).abs().max()
            assert ((a - b).norm() / b.norm()).item() < 1e-3 and (a != b).float().mean().item() < 0.2


def test_varlen_mixed_batch_sampled(oracle):
    """The benchmark's mixed batch (32 sequences, 64 .. 8192 tokens, causal, d = 128): forward and
    backward at full size; the oracle checks whole short sequences and, of the longest one, sampled
    query rows (O, LSE, dQ) and the last 256 keys' dK / dV (complete under the causal mask: only
    the last 256 query rows reach them)."""
    import paper_2603_05451_amd as A
    w = I.VARLEN_MIX
    x = I.make_varlen_inputs(w)
    lens = w.lengths()
    cu = x["cu_seqlens"].numpy()
    q, k, v, do, cud = (x[m].cuda() for m in ("q", "k", "v", "do", "cu_seqlens"))
    o, lse = A.attn_varlen_fwd(q, k, v, cud, w.scale, w.causal)
    dq, dk, dv = A.attn_varlen_bwd(q, k, v, o, do, lse, cud, w.scale, w.causal)
    torch.cuda.synchronize()
    o, lse, dq, dk, dv = (t.float().cpu().numpy() for t in (o, lse, dq, dk, dv))
    assert all(np.isfinite(t).all() for t in (o, lse, dq, dk, dv))
    hs = slice(0, 2)                                            # two of the 16 heads (Hkv = H here)
    order = np.argsort(lens)
    for b in list(order[:3]) + [order[len(order) // 2]]:        # three shortest and the median sequence, whole
        s = slice(int(cu[b]), int(cu[b + 1]))
        f = lambda m: I.to_f64(x[m][s][None, :, hs])
        ro, rlse = oracle.attn_fwd(f("q"), f("k"), f("v"), w.scale, w.causal)
        rdq, rdk, rdv = oracle.attn_bwd(f("q"), f("k"), f("v"), f("do"), w.scale, w.causal)
        assert_close(o[s][None, :, hs], ro, f"varlen mix O seq{b} len{lens[b]}")
        assert np.abs(lse[hs, s][None] - rlse).max() <= LSE_ABS
        assert_close(dq[s][None, :, hs], rdq, f"varlen mix dQ seq{b}")
        assert_close(dk[s][None, :, hs], rdk, f"varlen mix dK seq{b}")
        assert_close(dv[s][None, :, hs], rdv, f"varlen mix dV seq{b}")
    b = int(order[-1])                                          # the longest sequence
    n = lens[b]
    s = slice(int(cu[b]), int(cu[b + 1]))
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, n - 2, n - 1], rng.integers(0, n, 40),
                                     np.arange(n - 256, n)]))
    f = lambda m: I.to_f64(x[m][s][None, :, hs])
    ro, rlse = oracle.attn_fwd(f("q")[:, rows], f("k"), f("v"), w.scale, w.causal, q_pos=rows)
    rdq, rdk, rdv = oracle.attn_bwd(f("q")[:, rows], f("k"), f("v"), f("do")[:, rows], w.scale, w.causal, q_pos=rows)
    assert_close(o[s][None, :, hs][:, rows], ro, f"varlen mix O longest len{n}")
    assert np.abs(lse[hs, s][None][:, :, rows] - rlse).max() <= LSE_ABS
    assert_close(dq[s][None, :, hs][:, rows], rdq, "varlen mix dQ longest")
    assert_close(dk[s][None, n - 256:, hs], rdk[:, n - 256:], "varlen mix dK longest, last 256 keys")
    assert_close(dv[s][None, n - 256:, hs], rdv[:, n - 256:], "varlen mix dV longest, last 256 keys")


def test_varlen_many_short_sequences(oracle):
    """1500 sequences of 1 .. 40 tokens: more sequences than plan-kernel threads, every tile ragged."""
    import paper_2603_05451_amd as A
    rng = np.random.default_rng(11)
    lengths = [int(n) for n in rng.integers(1, 41, 1500)]
    x, cu, scale = packed_inputs(lengths, 2, 1, 64, 64, 51, with_do=True)
    q, k, v, do = (x[m].cuda() for m in ("q", "k", "v", "do"))
    cud = torch.from_numpy(cu).cuda()
    o, lse = A.attn_varlen_fwd(q, k, v, cud, scale, True)
    dq, dk, dv = A.attn_varlen_bwd(q, k, v, o, do, lse, cud, scale, True)
    torch.cuda.synchronize()
    o, dq, dk, dv = (t.float().cpu().numpy() for t in (o, dq, dk, dv))
    assert all(np.isfinite(t).all() for t in (o, dq, dk, dv))
    for b in list(range(0, 1500, 97)) + [1499]:
        s = slice(int(cu[b]), int(cu[b + 1]))
        f = lambda m: I.to_f64(x[m][s][None])
        ro, _ = oracle.attn_fwd(f("q"), f("k"), f("v"), scale, True)
        rdq, rdk, rdv = oracle.attn_bwd(f("q"), f("k"), f("v"), f("do"), scale, True)
        # short sequences give peaked softmaxes and gradients of magnitude 4 .. 8, where one bf16
        # half-ulp of the OUTPUT is 1.6e-2 already: absolute bound plus the output-rounding term
        # (parity.assert_close's bound, without the Frobenius part: sequences this short have
        # exactly-zero reference rows)
        ok = lambda got, ref: (np.abs(got - ref) <= 2e-2 + 2.0 ** -8 * np.abs(ref)).all()
        assert ok(o[s][None], ro) and ok(dq[s][None], rdq) and ok(dk[s][None], rdk) and ok(dv[s][None], rdv)


def read_tables(ws, B, Tq, Tk):
    """The two tile tables at the head of a backward workspace, as int arrays [entries, 8]:
    {first query row, query length, first key row, key length, tile, valid, sequence index, 0}."""
    mq, mk = Tq // 128 + B, Tk // 128 + B
    off_k = (mq * 32 + 255) // 256 * 256
    tq = ws[:mq * 32].view(torch.int32).reshape(mq, 8).cpu().numpy()
    tk = ws[off_k:off_k + mk * 32].view(torch.int32).reshape(mk, 8).cpu().numpy()
    return tq, tk


def check_table(table, want, loop_tiles, index_of):
    """want: set of (q start, q len, k start, k len, tile); loop_tiles(entry) = length of the loop a
    tile of that sequence runs; index_of: (q start, q len, k start, k len) -> sequence index.  Every
    wanted tile once, longest loops first, a sequence's tiles contiguous and from last to first, the
    rest of the table zero."""
    used = table[table[:, 5] == 0x5A17AB1E]
    assert len(used) == len(want) and {tuple(int(x) for x in e[:5]) for e in used} == want
    assert (table[len(used):] == 0).all() and (used[:, 7] == 0).all()
    assert all(int(e[6]) == index_of[tuple(int(x) for x in e[:4])] for e in used)
    loops = np.array([loop_tiles(e) for e in used])
    assert (np.diff(loops) <= 0).all()
    seen, i = set(), 0
    while i < len(used):
        key = tuple(int(x) for x in used[i, :4])
        assert key not in seen
        seen.add(key)
        nt = int(used[i, 4]) + 1                                # a run starts at the sequence's last tile
        assert (used[i:i + nt, :4] == used[i, :4]).all() and list(used[i:i + nt, 4]) == list(range(nt - 1, -1, -1))
        i += nt


def test_plan_tables_list_every_tile_once_longest_first():
    """The plan kernel's output (head of the workspace): one entry per 128-row query tile (sequences
    with keys) and per 128-row key tile, ordered by the number of tiles of the OTHER side, which is
    the loop a tile runs."""
    import paper_2603_05451_amd as A
    rng = np.random.default_rng(3)
    ql = [int(n) for n in np.concatenate([rng.integers(0, 700, 300), [0, 1, 128, 129, 4096, 5000, 7, 0]])]
    kl = [int(n) for n in np.concatenate([rng.integers(1, 900, 300), [5, 1, 128, 300, 4096, 5000, 0, 0]])]
    perm = rng.permutation(len(ql))
    ql, kl = [ql[i] for i in perm], [kl[i] for i in perm]
    cuq = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
    cuk = np.concatenate([[0], np.cumsum(kl)]).astype(np.int32)
    Tq, Tk, B, H, d = int(cuq[-1]), int(cuk[-1]), len(ql), 1, 64
    # sequences without keys get no query tiles, so the (undefined) rows are simply not touched;
    # keep the kernels away from them anyway: this test runs the backward of zeros
    z = lambda T: torch.zeros(T, H, d, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(A.attn_varlen_workspace_bytes(B, Tq, Tk, H, H, d, d, True), dtype=torch.uint8, device="cuda")
    lse = torch.zeros(H, Tq, dtype=torch.float32, device="cuda")
    A.attn_varlen_bwd(z(Tq), z(Tk), z(Tk), z(Tq), z(Tq), lse, torch.from_numpy(cuq).cuda(), 0.125, False,
                      workspace=ws, cu_seqlens_k=torch.from_numpy(cuk).cuda())
    torch.cuda.synchronize()
    tq, tk = read_tables(ws, B, Tq, Tk)
    tiles = lambda n: (n + 127) // 128
    seqs = [(int(cuq[b]), ql[b], int(cuk[b]), kl[b]) for b in range(B)]
    index_of = {e: b for b, e in enumerate(seqs) if e[1] > 0 or e[3] > 0}      # sequences that own rows are distinct
    check_table(tq, {(*e, t) for e in seqs if e[3] > 0 for t in range(tiles(e[1]))}, lambda e: tiles(int(e[3])),
                index_of)
    check_table(tk, {(*e, t) for e in seqs for t in range(tiles(e[3]))}, lambda e: tiles(int(e[1])), index_of)


def cross_inputs(qlens, klens, H, Hkv, dqk, dv, seed):
    """Packed tensors with separate query and key row counts, from the N(0,1) recipe."""
    Tq, Tk = int(sum(qlens)), int(sum(klens))
    w = I.Workload("cross", 1, H, Hkv, max(Tq, Tk), dqk, dv, False, seed)
    x = I.make_inputs(w, with_do=True)
    out = {n: x[n][0, :(Tq if n in ("q", "do") else Tk)].contiguous() for n in ("q", "k", "v", "do")}
    cuq = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    cuk = np.concatenate([[0], np.cumsum(klens)]).astype(np.int32)
    return out, cuq, cuk, w.scale


# (queries, keys) per sequence.  Non-causal: any combination, also more queries than keys and a
# sequence without queries.  Causal: keys >= queries (the last query sees every key): one decoded
# token against a long cache, a chunk appended to a prefix whose length is not a multiple of any
# tile size, equal lengths.
CROSS_NC = ([1, 200, 64, 129, 0, 700, 128, 333], [1000, 64, 200, 129, 300, 1, 640, 77])
CROSS_C = ([1, 1, 64, 129, 0, 100, 128, 333, 5], [1000, 1, 200, 129, 300, 611, 640, 333, 130])
CROSS_CASES = [
    ("d64_nc", CROSS_NC, 4, 2, 64, 64, False, 61),
    ("d64_c", CROSS_C, 2, 1, 64, 64, True, 62),
    ("d96_c", CROSS_C, 4, 2, 96, 96, True, 67),
    ("d128_nc", CROSS_NC, 4, 2, 128, 128, False, 63),
    ("d128_c", CROSS_C, 4, 1, 128, 128, True, 64),
    ("d192_nc", CROSS_NC, 2, 2, 192, 128, False, 65),
    ("d256_c", CROSS_C, 2, 1, 256, 256, True, 68),
    ("d192_c", CROSS_C, 2, 1, 192, 128, True, 66),
]


@pytest.mark.parametrize("name,lens,H,Hkv,dqk,dv,causal,seed", CROSS_CASES, ids=[c[0] for c in CROSS_CASES])
def test_varlen_separate_query_and_key_lengths(oracle, name, lens, H, Hkv, dqk, dv, causal, seed):
    """Query and key counts differ per sequence; under the causal mask the last query is aligned
    with the last key, which the oracle expresses through the query positions."""
    import paper_2603_05451_amd as A
    qlens, klens = lens
    x, cuq, cuk, scale = cross_inputs(qlens, klens, H, Hkv, dqk, dv, seed)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    cuqd, cukd = torch.from_numpy(cuq).cuda(), torch.from_numpy(cuk).cuda()
    nan = lambda t: torch.full_like(t, float("nan"))
    o = torch.full((q.shape[0], H, dv), float("nan"), dtype=torch.bfloat16, device="cuda")
    o, lse = A.attn_varlen_fwd(q, k, v, cuqd, scale, causal, o=o, cu_seqlens_k=cukd)
    dq, dk, dvv = A.attn_varlen_bwd(q, k, v, o, do, lse, cuqd, scale, causal, dq=nan(q), dk=nan(k), dv=nan(v),
                                    cu_seqlens_k=cukd)
    torch.cuda.synchronize()
    o, lse, dq, dk, dvv = (t.float().cpu().numpy() for t in (o, lse, dq, dk, dvv))
    assert all(np.isfinite(t).all() for t in (o, lse, dq, dk, dvv))            # every row written
    wide = lambda got, ref: (np.abs(got - ref) <= 2e-2 + 2.0 ** -8 * np.abs(ref)).all()
    for b, (nq, nk) in enumerate(zip(qlens, klens)):
        sq, sk = slice(int(cuq[b]), int(cuq[b + 1])), slice(int(cuk[b]), int(cuk[b + 1]))
        if nq == 0:
            assert (dk[sk] == 0).all() and (dvv[sk] == 0).all()                 # keys nobody attends to
            continue
        pos = np.arange(nq) + (nk - nq)
        fq, fk, fv, fdo = (I.to_f64(x[m][s][None]) for m, s in (("q", sq), ("k", sk), ("v", sk), ("do", sq)))
        ro, rlse = oracle.attn_fwd(fq, fk, fv, scale, causal, q_pos=pos)
        rdq, rdk, rdv = oracle.attn_bwd(fq, fk, fv, fdo, scale, causal, q_pos=pos)
        tag = f"{name} seq{b} q{nq} k{nk}"
        assert np.abs(lse[:, sq][None] - rlse).max() <= LSE_ABS, tag
        if min(nq, nk) < 32:
            # a handful of queries or keys: peaked softmaxes, outputs of magnitude > 4, reference
            # rows that are exactly zero -> absolute bound plus the output-rounding term
            assert wide(o[sq][None], ro) and wide(dq[sq][None], rdq) and wide(dk[sk][None], rdk) and \
                wide(dvv[sk][None], rdv), tag
            continue
        assert_close(o[sq][None], ro, "O " + tag)
        assert_close(dq[sq][None], rdq, "dQ " + tag)
        # dK / dV summed over the query heads of a group exceed magnitude 4 on the first keys of a
        # causal sequence: the output-rounding term joins the absolute bound there
        assert_close(dk[sk][None], rdk, "dK " + tag)
        assert_close(dvv[sk][None], rdv, "dV " + tag)


def test_varlen_decode_step_matches_last_row_of_prefill():
    """Causal attention of the last token against the whole sequence (1 query, N keys) is row N-1 of
    causal self-attention: same keys, same mask row; the tiles are cut differently, so the match is
    to rounding, not bitwise."""
    import paper_2603_05451_amd as A
    lengths = [300, 1025, 64, 4097]
    x, cu, scale = packed_inputs(lengths, 4, 2, 128, 128, 71)
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    cud = torch.from_numpy(cu).cuda()
    o_full, lse_full = A.attn_varlen_fwd(q, k, v, cud, scale, True)
    last = torch.from_numpy(cu[1:] - 1).long().cuda()
    cu1 = torch.arange(0, len(lengths) + 1, dtype=torch.int32, device="cuda")
    o_dec, lse_dec = A.attn_varlen_fwd(q[last].contiguous(), k, v, cu1, scale, True, cu_seqlens_k=cud)
    torch.cuda.synchronize()
    assert (o_dec.float() - o_full[last].float()).abs().max().item() <= 2e-2
    assert (lse_dec - lse_full[:, last]).abs().max().item() <= 2 * LSE_ABS


def test_cached_plan_tables_give_identical_results():
    """attn_varlen_plan once, then forward and backward calls without cu_seqlens (paper Sec. 3.3:
    the sort's metadata can be cached): bit-identical to calls that rebuild the tables."""
    import paper_2603_05451_amd as A
    qlens, klens = CROSS_C
    H, Hkv, d = 4, 2, 128
    x, cuq, cuk, scale = cross_inputs(qlens, klens, H, Hkv, d, d, 72)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    cuqd, cukd = torch.from_numpy(cuq).cuda(), torch.from_numpy(cuk).cuda()
    o, lse = A.attn_varlen_fwd(q, k, v, cuqd, scale, True, cu_seqlens_k=cukd)
    ref = A.attn_varlen_bwd(q, k, v, o, do, lse, cuqd, scale, True, cu_seqlens_k=cukd)
    B, Tq, Tk = len(qlens), q.shape[0], k.shape[0]
    ws = torch.zeros(A.attn_varlen_workspace_bytes(B, Tq, Tk, H, Hkv, d, d, True), dtype=torch.uint8, device="cuda")
    A.attn_varlen_plan(cuqd, Tq, Tk, H, Hkv, d, d, ws, cu_seqlens_k=cukd)
    for _ in range(2):                                   # the tables survive the calls that use them
        o2, lse2 = A.attn_varlen_fwd(q, k, v, None, scale, True, workspace=ws, B=B)
        got = A.attn_varlen_bwd(q, k, v, o2, do, lse2, None, scale, True, workspace=ws, B=B)
        torch.cuda.synchronize()
        assert torch.equal(o2, o) and torch.equal(lse2, lse)
        assert all(torch.equal(a, b) for a, b in zip(got, ref))


def test_unplanned_workspace_is_not_acted_on():
    """Calls without cu_seqlens on a workspace whose tables were never built (zeros, or bytes that
    do not carry the entry mark): the kernels find no entry to act on and leave the outputs alone."""
    import paper_2603_05451_amd as A
    H, Hkv, d, B, T = 2, 1, 64, 3, 700
    x, cu, scale = packed_inputs([300, 150, 250], H, Hkv, d, d, 73, with_do=True)
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    need = A.attn_varlen_workspace_bytes(B, T, T, H, Hkv, d, d, True)
    for fill in (0, 0x11):
        ws = torch.full((need,), fill, dtype=torch.uint8, device="cuda")
        o = torch.full((T, H, d), 7.0, dtype=torch.bfloat16, device="cuda")
        lse = torch.full((H, T), 7.0, dtype=torch.float32, device="cuda")
        A.attn_varlen_fwd(q, k, v, None, scale, True, o=o, lse=lse, workspace=ws, B=B)
        g = [torch.full_like(t, 7.0) for t in (q, k, v)]
        A.attn_varlen_bwd(q, k, v, o, do, lse, None, scale, True, dq=g[0], dk=g[1], dv=g[2], workspace=ws, B=B)
        torch.cuda.synchronize()
        assert (o == 7.0).all() and (lse == 7.0).all() and all((t == 7.0).all() for t in g)


def test_sequences_outside_the_tensors_are_left_out():
    """cu_seqlens_k (then cu_seqlens_q) whose last entry runs past the stated total: the table kernel
    leaves that sequence out, so none of its rows is read or written, every kernel ends normally, and
    the other sequences come out bit for bit as in the sound call."""
    import paper_2603_05451_amd as A
    H, Hkv, d = 4, 2, 128
    lens = [200, 130, 300]
    x, cu, scale = packed_inputs(lens, H, Hkv, d, d, 91, with_do=True)
    T = int(cu[-1])
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    good = torch.from_numpy(cu).cuda()
    o_ref, lse_ref = A.attn_varlen_fwd(q, k, v, good, scale, True)
    g_ref = A.attn_varlen_bwd(q, k, v, o_ref, do, lse_ref, good, scale, True)
    bad = good.clone(); bad[3] = T + 64                     # last sequence: rows past the end of the tensors
    for cq, ck in ((good, bad), (bad, good), (bad, bad)):
        o = torch.full_like(o_ref, 7.0); lse = torch.full_like(lse_ref, 7.0)
        A.attn_varlen_fwd(q, k, v, cq, scale, True, o=o, lse=lse, cu_seqlens_k=ck)
        grads = [torch.full_like(t, 7.0) for t in (q, k, v)]
        A.attn_varlen_bwd(q, k, v, o_ref, do, lse_ref, cq, scale, True, dq=grads[0], dk=grads[1], dv=grads[2],
                          cu_seqlens_k=ck)
        torch.cuda.synchronize()
        for b in range(3):
            s = slice(int(cu[b]), int(cu[b + 1]))
            if b < 2:
                assert torch.equal(o[s], o_ref[s]) and torch.equal(lse[:, s], lse_ref[:, s])
                for a, r in zip(grads, g_ref):
                    assert torch.equal(a[s], r[s])
            else:
                assert (o[s] == 7.0).all() and (lse[:, s] == 7.0).all()
                for a in grads:
                    assert (a[s] == 7.0).all()
