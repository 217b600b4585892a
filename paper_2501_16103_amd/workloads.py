"""Seeded synthetic inputs for the MoE expert-GEMM workloads.

This module only draws random numbers and casts them to storage types with
library conversions; it holds none of the method's arithmetic (no task map, no
matrix product) and imports neither the HIP binding nor the CPU oracle.  Both
sides of a parity test receive the tensors produced here.

Recipes (all seeded from BASE_SEED, the workload name, T and a tensor tag):
  X  ~ N(0,1); W_e ~ N(0,1/K), one seed per expert so any expert can be drawn
  alone, on the CPU or on the GPU (the two devices give different streams; a
  test draws once and hands the same bytes to both sides).
  fp8: per-token scale max|x_t|/448 and per-expert scale max|W_e|/448, values
  divided by the scale and cast to OCP e4m3 by the tensor library.
  routing: "gauss_topk" top-k of Gaussian logits; "uniform_topk" top-k of
  uniform scores; "zipf" k draws without replacement from p ~ rank^-1.2 over a
  seeded expert permutation; "balanced" / "best" / "worst" are the paper's
  evaluation scenarios (Sec. 5).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, replace
from typing import Optional

import torch

BASE_SEED = 20250116
E4M3_MAX = 448.0


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    E: int
    k: int
    K: int
    N: int
    dtype: str = "bf16"          # "bf16" | "fp8"
    routing: str = "gauss_topk"
    tile_m: int = 128            # default tiling the benchmark uses for this point
    tile_n: int = 128
    tile_m_slack: int = 0        # rows the last m-tile of an expert may hold beyond tile_m

    @property
    def R(self) -> int:
        return self.T * self.k

    @property
    def flops(self) -> int:
        return 2 * self.T * self.k * self.K * self.N

    def with_T(self, T: int, **kw) -> "Workload":
        return replace(self, T=T, **kw)


def _seed(*parts) -> int:
    h = hashlib.sha256(("|".join(str(p) for p in (BASE_SEED,) + parts)).encode()).digest()
    return int.from_bytes(h[:7], "little")


def _gen(device, *parts) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_seed(*parts))
    return g


# The five benchmark workload families and the paper's own evaluation shape.
def tiny(T: int = 64) -> Workload:
    return Workload("tiny", T, 8, 2, 256, 512, "bf16", "gauss_topk", 32, 128)


def mixtral_up(T: int) -> Workload:
    tm = 256 if T >= 2048 else (128 if T >= 256 else 16)
    return Workload("mixtral_up", T, 8, 2, 4096, 28672, "bf16", "gauss_topk", tm, 256, 32 if tm == 256 else 0)


def mixtral_down_zipf(T: int) -> Workload:
    tm = 256 if T >= 2048 else 64
    return Workload("mixtral_down_zipf", T, 8, 2, 14336, 4096, "bf16", "zipf", tm, 256)


def fine_grained(T: int) -> Workload:
    tm = 256 if T >= 8192 else (128 if T >= 2048 else 16)
    return Workload("fine_grained", T, 256, 8, 7168, 4096, "bf16", "gauss_topk", tm, 256, 32 if tm == 256 else 0)


def decode_fp8(T: int) -> Workload:
    if T >= 1024:   # the same layer at prefill sizes
        return Workload("decode_fp8", T, 64, 6, 2048, 2816, "fp8", "uniform_topk", 256, 256)
    return Workload("decode_fp8", T, 64, 6, 2048, 2816, "fp8", "uniform_topk", 16, 256 if T == 8 else 128)


def paper_eval(scenario: str = "balanced", T: int = 4096) -> Workload:
    """Sec. 5: T=4096, 64 experts, top-8, expert weight [3584, 2560]."""
    return Workload("paper_eval_" + scenario, T, 64, 8, 3584, 2560, "bf16", scenario, 256, 256)


def make_routing(wl: Workload, device="cpu") -> torch.Tensor:
    """int32 [T, k] expert ids, distinct within a token."""
    T, E, k = wl.T, wl.E, wl.k
    g = _gen("cpu", wl.name, T, "routing")
    if T == 0:
        ids = torch.zeros((0, k), dtype=torch.int32)
    elif wl.routing == "gauss_topk":
        ids = torch.topk(torch.randn(T, E, generator=g), k, dim=1).indices
    elif wl.routing == "uniform_topk":
        ids = torch.topk(torch.rand(T, E, generator=g), k, dim=1).indices
    elif wl.routing == "zipf":
        p = torch.arange(1, E + 1, dtype=torch.float64) ** -1.2
        perm = torch.randperm(E, generator=g)
        draws = torch.multinomial((p / p.sum()).expand(T, E), k, replacement=False, generator=g)
        ids = perm[draws]
    elif wl.routing == "balanced":
        r = torch.arange(T * k).reshape(T, k)
        ids = r % E
    elif wl.routing == "best":
        ids = torch.arange(k).expand(T, k).clone()
    elif wl.routing == "worst":
        ids = torch.arange(k).expand(T, k).clone()
        n_single = min(E - k, T)
        ids[:n_single, k - 1] = k + torch.arange(n_single)
    else:
        raise ValueError(wl.routing)
    return ids.to(torch.int32).contiguous().to(device)


def make_x(wl: Workload, device="cpu"):
    """bf16: tensor [T,K] bf16.  fp8: (uint8 [T,K] e4m3 bytes, fp32 scale [T])."""
    g = _gen(device, wl.name, wl.T, "x")
    x = torch.randn(wl.T, wl.K, generator=g, device=device, dtype=torch.float32)
    if wl.dtype == "bf16":
        return x.to(torch.bfloat16)
    amax = x.abs().amax(dim=1).clamp_min(1e-12)
    scale = (amax / E4M3_MAX).to(torch.float32)
    q = (x / scale[:, None]).to(torch.float8_e4m3fn)
    return q.view(torch.uint8), scale


def make_w_expert(wl: Workload, e: int, device="cpu"):
    """One expert's weight [K,N] (N contiguous): bf16 tensor, or (uint8 bytes, fp32 scalar scale)."""
    g = _gen(device, wl.name, "w", e)
    w = torch.randn(wl.K, wl.N, generator=g, device=device, dtype=torch.float32) * (wl.K ** -0.5)
    if wl.dtype == "bf16":
        return w.to(torch.bfloat16)
    scale = (w.abs().amax().clamp_min(1e-12) / E4M3_MAX).to(torch.float32)
    q = (w / scale).to(torch.float8_e4m3fn)
    return q.view(torch.uint8), scale


def make_w(wl: Workload, device="cpu", out: Optional[torch.Tensor] = None):
    """All experts: bf16 [E,K,N], or (uint8 [E,K,N], fp32 scale [E])."""
    if wl.dtype == "bf16":
        W = out if out is not None else torch.empty(wl.E, wl.K, wl.N, dtype=torch.bfloat16, device=device)
        for e in range(wl.E):
            W[e].copy_(make_w_expert(wl, e, device))
        return W
    W = out if out is not None else torch.empty(wl.E, wl.K, wl.N, dtype=torch.uint8, device=device)
    scales = torch.empty(wl.E, dtype=torch.float32, device=device)
    for e in range(wl.E):
        q, s = make_w_expert(wl, e, device)
        W[e].copy_(q)
        scales[e] = s
    return W, scales


def bits(t: torch.Tensor):
    """Host numpy view of a tensor's storage bits (bf16 -> uint16, uint8 -> uint8, int32 -> int32)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
