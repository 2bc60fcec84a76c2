"""Seeded synthetic inputs shaped like the paper's benchmark tensors (Sec. 5: random
Q, K, V of a given batch, sequence length, head count and head dimension).

This module holds no attention arithmetic.  It is the only code shared by the tests
of the CPU oracle and of the HIP path: both sides receive the same bf16 bits.

Values are drawn on the CPU generator (reproducible without a GPU) as fp32 N(0,1),
optionally with a Bernoulli(outlier_frac) subset of Q and K entries multiplied by
outlier_scale, then rounded to bf16 (round-to-nearest-even).
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    Hkv: int
    N: int
    dqk: int
    dv: int
    causal: bool
    seed: int
    outlier_frac: float = 0.0
    outlier_scale: float = 8.0

    @property
    def scale(self) -> float:
        return 1.0 / float(self.dqk) ** 0.5

    def fwd_flops(self) -> float:
        """2 N^2 (dqk + dv) per head and batch, halved for causal (paper Sec. 5 convention)."""
        f = 2.0 * self.N * self.N * (self.dqk + self.dv) * self.H * self.B
        return f / 2 if self.causal else f

    def bwd_flops(self) -> float:
        """The paper's convention: backward = 2.5 x forward."""
        return 2.5 * self.fwd_flops()


def sweep(d: int, causal: bool, seed: int, tokens: int = 16384, H: int = 16):
    """The fixed-token-count sweep: N in {512..16k}, B = tokens / N."""
    tag = "c" if causal else "nc"
    return [Workload(f"sweep_d{d}_{tag}_N{N}", tokens // N, H, H, N, d, d, causal, seed)
            for N in (512, 1024, 2048, 4096, 8192, 16384)]


CANARY = Workload("canary_N128_d64", 1, 2, 2, 128, 64, 64, False, 0)
TARGET = Workload("target_N8192_d128_nc", 2, 16, 16, 8192, 128, 128, False, 6)
GQA = Workload("gqa_N8192_d128_c", 2, 32, 8, 8192, 128, 128, True, 4)
D96 = Workload("d96_N8192_c", 2, 16, 16, 8192, 96, 96, True, 10)      # a head dim between the paper's 64 and 128
D256 = Workload("d256_N8192_c", 2, 8, 8, 8192, 256, 256, True, 12)     # hidden = 2048 like the paper's settings
MLA_OUTLIER = Workload("d192x128_N32768_c_outliers", 1, 16, 16, 32768, 192, 128, True, 5,
                       outlier_frac=0.01)
SWEEP_D64_NC = sweep(64, False, 2)
SWEEP_D128_C = sweep(128, True, 3)


@dataclass(frozen=True)
class VarlenWorkload:
    """A packed batch of sequences of different lengths (paper Sec. 3.3: mixed prefill batches).
    Lengths are log-uniform integers in [lo, hi], drawn with the workload's seed and given in
    DRAWN order (not sorted: ordering is the library's job)."""
    name: str
    B: int
    H: int
    Hkv: int
    lo: int
    hi: int
    dqk: int
    dv: int
    causal: bool
    seed: int

    @property
    def scale(self) -> float:
        return 1.0 / float(self.dqk) ** 0.5

    def lengths(self):
        g = torch.Generator(device="cpu")
        g.manual_seed(self.seed + 1000)
        u = torch.rand(self.B, generator=g, dtype=torch.float64)
        import math
        return [int(round(math.exp(math.log(self.lo) + float(x) * (math.log(self.hi) - math.log(self.lo))))) for x in u]

    def fwd_flops(self) -> float:
        f = sum(2.0 * n * n * (self.dqk + self.dv) * self.H for n in self.lengths())
        return f / 2 if self.causal else f

    def bwd_flops(self) -> float:
        return 2.5 * self.fwd_flops()


VARLEN_MIX = VarlenWorkload("varlen_mix_B32_d128_c", 32, 16, 16, 64, 8192, 128, 128, True, 7)
VARLEN_MIX_GQA = VarlenWorkload("varlen_mix_B32_gqa_d128_c", 32, 32, 8, 64, 8192, 128, 128, True, 8)
VARLEN_MIX_D64 = VarlenWorkload("varlen_mix_B32_d64_nc", 32, 16, 16, 64, 8192, 64, 64, False, 9)


def make_varlen_inputs(w: VarlenWorkload, with_do: bool = True):
    """Packed bf16 CPU tensors q [T,H,dqk], k [T,Hkv,dqk], v [T,Hkv,dv], do [T,H,dv] (the recipe of
    make_inputs with B = 1 and N = T) and cu_seqlens [B+1] int32."""
    lens = w.lengths()
    T = sum(lens)
    x = make_inputs(Workload(w.name, 1, w.H, w.Hkv, T, w.dqk, w.dv, w.causal, w.seed), with_do=with_do)
    out = {n: t[0] for n, t in x.items()}
    out["cu_seqlens"] = torch.tensor([0] + list(torch.tensor(lens).cumsum(0).tolist()), dtype=torch.int32)
    return out


def make_inputs(w: Workload, with_do: bool = True):
    """Return bf16 CPU tensors q [B,N,H,dqk], k [B,N,Hkv,dqk], v [B,N,Hkv,dv], do [B,N,H,dv]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)

    def normal(*shape):
        return torch.randn(*shape, generator=g, dtype=torch.float32)

    def with_outliers(x):
        if w.outlier_frac > 0.0:
            hit = torch.rand(x.shape, generator=g) < w.outlier_frac
            x = torch.where(hit, x * w.outlier_scale, x)
        return x

    q = with_outliers(normal(w.B, w.N, w.H, w.dqk)).to(torch.bfloat16)
    k = with_outliers(normal(w.B, w.N, w.Hkv, w.dqk)).to(torch.bfloat16)
    v = normal(w.B, w.N, w.Hkv, w.dv).to(torch.bfloat16)
    out = {"q": q, "k": k, "v": v}
    if with_do:
        out["do"] = normal(w.B, w.N, w.H, w.dv).to(torch.bfloat16)
    return out


def to_f64(t: torch.Tensor):
    """Exact bf16 -> fp64 numpy conversion (every bf16 value is an fp64 value)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
