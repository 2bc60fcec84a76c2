"""GPU software-exp2 (paper Sec. 3.1.3) against the numpy oracle and the paper's accuracy table; the
measurement probes of libattn_probes.so (rates of the exponential, the matrix cores, the LDS, and what
the instructions around an MFMA cost a wave that is alone on its SIMD)."""
import os

import numpy as np
import pytest
import torch

from oracle import exp2_emulation as E

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "exp2_accuracy_table.txt")


def table():
    return {ln.split()[0]: [float(v) for v in ln.split()[1:]] for ln in open(GOLDEN)
            if ln.strip() and not ln.startswith("#")}


@pytest.mark.parametrize("degree", [3, 4, 5])
def test_gpu_emulation_matches_oracle_and_table(degree):
    import paper_2603_05451_amd as A
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.random(1 << 22, dtype=np.float32),                       # the table's domain
                        rng.uniform(-126, 40, 1 << 16).astype(np.float32),           # range reduction
                        np.array([-1e4, -127.0, -126.5, -1.0, 0.0, 1.0, 17.0], np.float32)])
    y = A.attn_exp2_emulated(torch.from_numpy(x).cuda(), degree).cpu().numpy()
    ref = E.exp2_emulated(x, E.fit_coefficients(degree))
    # the oracle's coefficients come from a linear program, the kernel's from a Remez exchange:
    # the two fits agree to the last fp32 digit or two, so results agree within a few ulp
    rel = np.abs(y.astype(np.float64) - ref.astype(np.float64)) / np.maximum(np.abs(ref), 1e-37)
    assert rel.max() <= 1e-6, rel.max()
    assert y[-7] == 0.0 and y[-6] == 0.0 and y[-3] == 1.0 and y[-2] == 2.0 and y[-1] == 131072.0
    # and the GPU result reproduces the paper's error levels on [0, 1)
    want = table()[f"degree{degree}"]
    x01 = x[:1 << 22]
    true = np.exp2(x01.astype(np.float64))
    e32 = np.abs(y[:1 << 22].astype(np.float64) - true) / true
    e16 = np.abs(E.to_bf16(y[:1 << 22]).astype(np.float64) - true) / true
    assert abs(e32.mean() - want[1]) <= 0.05 * want[1]
    assert abs(e32.max() - want[0]) <= 0.10 * want[0]
    assert abs(e16.max() - want[2]) <= 0.02 * want[2] and abs(e16.mean() - want[3]) <= 0.02 * want[3]


def test_hardware_exp2_matches_table_row():
    import paper_2603_05451_amd as A
    x = np.random.default_rng(8).random(1 << 22, dtype=np.float32)
    y = A.attn_exp2_emulated(torch.from_numpy(x).cuda(), 0).cpu().numpy()
    true = np.exp2(x.astype(np.float64))
    e32 = np.abs(y.astype(np.float64) - true) / true
    # v_exp_f32 is a different unit from the paper's MUFU.EX2: same order of magnitude (1 ulp class)
    assert e32.max() < 3e-7 and e32.mean() < 6e-8


def test_emulation_is_slower_than_the_hardware_instruction(capsys):
    """The measurement behind keeping emulation off the path: evaluations per second of each
    variant, pure ALU, whole chip."""
    from paper_2603_05451_amd import probes as A
    rates = {}
    for degree in (0, 3, 4, 5):
        A.attn_exp2_rate(degree, 64)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n, out = A.attn_exp2_rate(degree, 2000)
        e1.record()
        e1.synchronize()
        assert torch.isfinite(out).all()
        rates[degree] = n / (e0.elapsed_time(e1) * 1e-3) / 1e12
    print("exp2 evaluations per second (T/s):", {k: round(v, 2) for k, v in rates.items()})
    path = os.path.join(os.path.dirname(os.path.dirname(__file__)), "gpurun_out", "exp2_rates.txt")
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("degree (0 = v_exp_f32) : T evaluations / s\n" + "\n".join(f"{k} : {v:.3f}" for k, v in rates.items()) + "\n")
    assert rates[3] < rates[0] and rates[4] < rates[0] and rates[5] < rates[0]


def test_partial_emulation_lowers_the_exponential_rate():
    """Paper Sec. 3.1.3 runs 10-25 % of a row's exponentials on the FMA pipes next to the hardware
    unit.  Here both issue from one vector port: every share of emulation lowers the total rate."""
    from paper_2603_05451_amd import probes as A
    rates = {}
    for emu in (0, 1, 2, 4, 8):
        A.attn_exp2_rate_partial(emu, 64)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n, out = A.attn_exp2_rate_partial(emu, 2000)
        e1.record()
        e1.synchronize()
        assert torch.isfinite(out).all()
        rates[emu] = n / (e0.elapsed_time(e1) * 1e-3) / 1e12
    path = os.path.join(os.path.dirname(os.path.dirname(__file__)), "gpurun_out", "exp2_partial_rates.txt")
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("emulated evaluations of 8 (degree 3) : T evaluations / s\n" +
                "\n".join(f"{k} : {v:.3f}" for k, v in rates.items()) + "\n")
    assert rates[1] < rates[0] and rates[2] < rates[1] and rates[8] < rates[4] < rates[2]


def test_matrix_core_ceiling_on_random_operands():
    """Pure-MFMA rate with constant and with N(0,1) operands: the second is the ceiling every bf16
    MFMA kernel on such data is bounded by (the power limit lowers the clock)."""
    from paper_2603_05451_amd import probes as A
    rates = {}
    for name, rnd in (("constant", 0), ("N(0,1)", 1)):
        A.attn_mfma_rate(rnd, 2000)
        best = 0.0
        for _ in range(2):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops, out = A.attn_mfma_rate(rnd, 40000)      # about 40-50 ms: long enough for the clock to settle
            e1.record()
            e1.synchronize()
            assert torch.isfinite(out).all()
            best = max(best, flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        rates[name] = best
    print("pure MFMA TFLOP/s:", {k: round(v) for k, v in rates.items()})
    path = os.path.join(os.path.dirname(os.path.dirname(__file__)), "gpurun_out", "mfma_rates.txt")
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("\n".join(f"{k} operands : {v:.0f} TFLOP/s" for k, v in rates.items()) + "\n")
    assert 1000 < rates["N(0,1)"] <= rates["constant"] * 1.02 < 2600


def test_lds_read_rate_in_the_kernels_access_patterns():
    """Bytes per clock and CU that the LDS delivers in the two read patterns of the attention
    kernels (swizzled tiles: no bank conflicts expected).  The forward kernel reads 32 KiB per
    wave and 64-key tile, i.e. about 55 bytes per clock and CU at its measured speed."""
    from paper_2603_05451_amd import probes as A
    rates = {}
    for name, pat in (("ds_read_b128, A-operand fragments", 0), ("ds_read_b64_tr_b16, transposed fragments", 1)):
        A.attn_lds_rate(pat, 200)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nbytes, out = A.attn_lds_rate(pat, 20000)
        e1.record()
        e1.synchronize()
        assert torch.isfinite(out).all()
        rates[name] = nbytes / (e0.elapsed_time(e1) * 1e-3) / 256 / 2.4e9      # bytes per clock and CU at 2.4 GHz
    print("LDS bytes / clock / CU:", {k: round(v) for k, v in rates.items()})
    path = os.path.join(os.path.dirname(os.path.dirname(__file__)), "gpurun_out", "lds_rates.txt")
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("\n".join(f"{k} : {v:.0f} B/clk/CU (at 2.4 GHz)" for k, v in rates.items()) + "\n")
    assert all(100 < v < 300 for v in rates.values())


def test_single_wave_issue_costs():
    """What accompanies an MFMA in a wave that is alone on its SIMD (the forward, dQ and dK/dV kernels
    of the target shape): shader cycles per step, the clock the power limit leaves, and the whole-chip
    rate, for every built variant.  Written to gpurun_out/wave_issue.txt; the assertions pin the
    facts the kernel designs rest on."""
    from paper_2603_05451_amd import probes as P
    rows = {}
    for c, cfg in enumerate(P.wave_issue_configs()):
        rows[cfg] = P.wave_issue(c, 4000)
    path = os.path.join(os.path.dirname(os.path.dirname(__file__)), "gpurun_out", "wave_issue.txt")
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("per step: 1 MFMA + ...                                   cycles/step  clock MHz  TFLOP/s\n")
        for (nv, nb, ntr, dma, ring), (cyc, mhz, tf) in rows.items():
            f.write(f"VALU {nv}  ds_read_b128 {nb}  tr pairs {ntr}  copy every {dma:2d}  ring {ring} : {cyc:8.1f} {mhz:10.0f} {tf:8.0f}\n")
    alone = rows[(0, 0, 0, 0, 4)]
    assert 31.5 < alone[0] < 36.0                                   # an MFMA of 8 passes every 32 cycles
    assert rows[(0, 1, 0, 0, 4)][0] < 40.0                          # one 16-byte LDS fragment per MFMA still (nearly) fits
    assert rows[(0, 2, 0, 0, 4)][0] > 45.0                          # two do not: LDS bandwidth
    assert rows[(0, 0, 0, 1, 4)][0] > 55.0                          # a copy instruction per MFMA: the copy path
    assert rows[(3, 0, 1, 0, 4)][2] < alone[2]                      # and everything costs clock or cycles
