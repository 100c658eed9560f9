"""Seeded synthetic KV-cache workloads (inputs only; none of the method's arithmetic lives here).

The paper measures on Llama-2-7B KV data ("Experiments Setup"); neither the
weights nor the prompts are available, so these tensors stand in for them.  What
they imitate is the structure the paper reports in "Quantization of K-Cache" and
"Quantization of V-Cache": K is columnar (channels differ by orders of magnitude),
scores are wide-ranged, V has no column structure beyond per-channel scale.

Every tensor is drawn in fp32 from ``torch.Generator().manual_seed(1000 + cfg)``,
transformed, clipped to the finite fp16 range and rounded to fp16.  The same host
copy feeds the CPU oracle and the GPU library.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

FP16_MAX = 65504.0


@dataclass
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    Ncap: int
    k: torch.Tensor      # fp16 [B, Hkv, N, D]  (N = tokens generated, <= Ncap)
    v: torch.Tensor      # fp16 [B, Hkv, N, D]
    q: torch.Tensor      # fp16 [B, Hq, D]
    lens: torch.Tensor   # int32 [B] tokens of k/v that belong to each sequence
    append_last: bool    # the last token of each sequence is appended inside the timed step


_SHAPES = {
    1: dict(B=1, Hq=32, Hkv=32, N=1024),
    2: dict(B=8, Hq=32, Hkv=32, N=4096),
    3: dict(B=16, Hq=32, Hkv=32, N=8192),
    4: dict(B=8, Hq=32, Hkv=8, N=32768),
    5: dict(B=4, Hq=32, Hkv=8, N=131072),
}
_NAMES = {
    1: "cfg1 B1 H32/32 D128 N1024 N(0,1) + 4 outlier channels x20",
    2: "cfg2 Llama-2-7B layer B8 H32/32 D128 N4096 per-channel log-uniform scales",
    3: "cfg3 Llama-2-7B layer B16 H32/32 D128 N8192 scales + 1% token outliers x30 + append 1",
    4: "cfg4 Llama-3-8B GQA layer B8 H32/8 D128 N32768 scales + 4 outlier channels x20",
    5: "cfg5 long context B4 H32/8 D128 Ncap131072 len U[32K,128K] Student-t(3)",
}


def _to_fp16(x: torch.Tensor) -> torch.Tensor:
    return x.clamp_(-FP16_MAX, FP16_MAX).to(torch.float16)


def make(cfg: int, *, B: int | None = None, N: int | None = None, Hq: int | None = None, Hkv: int | None = None,
         seed: int | None = None) -> Workload:
    """Build config ``cfg`` (1..5); B / N / Hq / Hkv override the size for scaled-down parity cases."""
    shp = dict(_SHAPES[cfg])
    for key, val in (("B", B), ("N", N), ("Hq", Hq), ("Hkv", Hkv)):
        if val is not None:
            shp[key] = val
    B, Hq, Hkv, N, D = shp["B"], shp["Hq"], shp["Hkv"], shp["N"], 128
    gen = torch.Generator().manual_seed(1000 + cfg if seed is None else seed)
    randn = lambda *s: torch.randn(*s, generator=gen, dtype=torch.float32)
    rand = lambda *s: torch.rand(*s, generator=gen, dtype=torch.float32)

    q = _to_fp16(randn(B, Hq, D))
    lens = torch.full((B,), N, dtype=torch.int32)
    ks = torch.ones(Hkv, 1, D)
    vs = torch.ones(Hkv, 1, D)
    if cfg in (2, 3, 4):  # per-(head, channel) scales 10^U(-1,1), independent for K and V, shared over batch
        ks = torch.pow(10.0, rand(Hkv, 1, D) * 2 - 1)
        vs = torch.pow(10.0, rand(Hkv, 1, D) * 2 - 1)
    if cfg in (1, 4):  # 4 outlier channels x20 per head, independent for K and V
        for s in (ks, vs):
            for h in range(Hkv):
                idx = torch.randperm(D, generator=gen)[:4]
                s[h, 0, idx] *= 20.0
    if cfg == 5:
        lo = min(32768, max(1, N // 4))
        lens = torch.randint(lo, N + 1, (B,), generator=gen, dtype=torch.int64).to(torch.int32)

    k = torch.empty(B, Hkv, N, D, dtype=torch.float16)
    v = torch.empty(B, Hkv, N, D, dtype=torch.float16)
    for b in range(B):  # one sequence at a time keeps the fp32 temporaries small
        if cfg == 5:  # Student-t, nu = 3: normal / sqrt(chi2_3 / 3)
            kb = randn(Hkv, N, D) / torch.sqrt(randn(Hkv, N, D, 3).square_().sum(-1) / 3.0)
            vb = randn(Hkv, N, D) / torch.sqrt(randn(Hkv, N, D, 3).square_().sum(-1) / 3.0)
        else:
            kb = randn(Hkv, N, D) * ks
            vb = randn(Hkv, N, D) * vs
        if cfg == 3:  # 1 % of the (b, t) token rows of K and of V scaled x30
            kb[:, rand(N) < 0.01, :] *= 30.0
            vb[:, rand(N) < 0.01, :] *= 30.0
        k[b] = _to_fp16(kb)
        v[b] = _to_fp16(vb)
    return Workload(_NAMES[cfg], B, Hq, Hkv, D, ((N + 255) // 256) * 256, k, v, q, lens, append_last=(cfg == 3))


def edge_patterns(B: int, Hkv: int, N: int, D: int = 128, seed: int = 7) -> tuple[torch.Tensor, torch.Tensor]:
    """fp16 K, V made of raw random bit patterns restricted to finite values: zeros, subnormals,
    the largest finite numbers and both signs all occur (bit-exactness cases)."""
    gen = torch.Generator().manual_seed(seed)

    def one():
        bits = torch.randint(0, 65536, (B, Hkv, N, D), generator=gen, dtype=torch.int32)
        exp_all_ones = (bits & 0x7C00) == 0x7C00
        bits = torch.where(exp_all_ones, bits & ~0x0400, bits)  # Inf/NaN -> finite
        return bits.to(torch.uint16).view(torch.float16)
    return one(), one()


# ---------------------------------------------------------------------------------------------- weight GEMV
# The paper names the weights as the other operand its framework covers ("Precision Alignment in Uncertainty
# Calculation") and measures nothing on them; the shapes below are the projection matrices of its model
# (Llama-2-7B: hidden 4096, MLP 11008), the values are a stand-in: W ~ N(0, 1/K) times a per-row scale 10^U(-0.5, 0.5)
# (the rows of a trained projection differ in norm), x ~ N(0, 1) with `outliers` channels x20 (a few activation
# channels of a transformer carry values far above the rest).
WEIGHT_SHAPES = {"attn_proj": (4096, 4096), "mlp_up": (4096, 11008), "mlp_down": (11008, 4096)}


@dataclass
class WeightWorkload:
    name: str
    K: int
    N: int
    W: torch.Tensor   # fp16 [K, N]
    x: torch.Tensor   # fp16 [B, K]


def make_weights(shape: str | tuple[int, int] = "attn_proj", B: int = 1, *, outliers: int = 8, seed: int = 2001) -> WeightWorkload:
    K, N = WEIGHT_SHAPES[shape] if isinstance(shape, str) else shape
    gen = torch.Generator().manual_seed(seed)
    scale = torch.pow(10.0, torch.rand(K, 1, generator=gen) - 0.5) / (K ** 0.5)
    W = _to_fp16(torch.randn(K, N, generator=gen, dtype=torch.float32) * scale)
    x = torch.randn(B, K, generator=gen, dtype=torch.float32)
    for b in range(B):
        idx = torch.randperm(K, generator=gen)[:outliers]
        x[b, idx] *= 20.0
    return WeightWorkload(f"{shape} K{K} N{N} B{B} N(0,1/K) x row scales, x N(0,1) + {outliers} channels x20", K, N, W,
                          _to_fp16(x))
