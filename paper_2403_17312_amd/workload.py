"""Seeded synthetic decode workloads for Sparse Window Attention.

This module only produces INPUTS (random tensors with a stated distribution and
structure).  It holds none of the method's arithmetic and is the one piece of
code that both the HIP path and the CPU oracle's tests consume, so that both
sides see exactly the same bits.

Recipe (stands in, by shape only, for the paper's sampled-prompt throughput
workload, Section VI-A):
  * per (sequence, head) a direction  mu ~ N(0, I_d);
  * every query  q_t = (mu + eps_t) / sqrt(2), eps_t ~ N(0, I_d)  (marginally
    N(0,1) per coordinate, but with a component shared over time so that
    planted keys stay heavy hitters at every step);
  * keys and values of prompt and decode tokens ~ N(0, I_d);
  * heavy hitters: round(f * s) (at least 1) distinct prompt positions per
    sequence, uniform in [0, s - w), shared by the heads of the sequence; their
    keys get  + 3 * mu / |mu|  of the head's own mu;
  * everything is rounded once to the workload dtype; those bits are what every
    consumer reads;
  * prompt lengths are fixed, or i.i.d. uniform on [lo, hi] per sequence.
Tensors are generated with a torch.Generator on the requested device; CPU and
GPU generators give different streams, so a test generates once, on one
device, and hands the same tensors to both sides.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    b: int
    h: int
    d: int
    dtype: str            # "f32" | "f16" | "bf16"
    prompt_lo: int
    prompt_hi: int
    steps: int
    w: int
    sparsity_bp: int      # KV sparsity in basis points (8000 = 80 %)
    hh_frac: float        # fraction of prompt positions planted as heavy hitters
    prefill_R: int = 0    # >0: importance seeded from the last R prompt queries
    seed: int = 20240317

    @property
    def cap(self) -> int:
        """Slots per (sequence, head): room for the prompt plus every decode token, rounded up to
        a multiple of 64 so that every pair's rows of the fp32/int32 side arrays start on a
        256-byte boundary."""
        return (self.prompt_hi + self.steps + 1 + 63) // 64 * 64

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def torch_dtype(self) -> torch.dtype:
        return TORCH_DTYPE[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five workloads named by the benchmark definition of this repository.
CONFIGS: Dict[str, Workload] = {
    "c1_tiny": Workload("c1_tiny", 1, b=1, h=4, d=64, dtype="f32", prompt_lo=256, prompt_hi=256,
                        steps=16, w=8, sparsity_bp=8000, hh_frac=0.02),
    "c2_opt6p7b": Workload("c2_opt6p7b", 2, b=16, h=32, d=128, dtype="f16", prompt_lo=512,
                           prompt_hi=512, steps=32, w=16, sparsity_bp=8000, hh_frac=0.01),
    "c3_opt13b": Workload("c3_opt13b", 3, b=64, h=40, d=128, dtype="f16", prompt_lo=1024,
                          prompt_hi=1024, steps=64, w=32, sparsity_bp=8000, hh_frac=0.01),
    "c4_opt30b": Workload("c4_opt30b", 4, b=32, h=56, d=128, dtype="bf16", prompt_lo=4096,
                          prompt_hi=4096, steps=128, w=64, sparsity_bp=9000, hh_frac=0.01,
                          prefill_R=64),
    "c5_llama7b_sp50": Workload("c5_llama7b_sp50", 5, b=256, h=32, d=128, dtype="f16",
                                prompt_lo=512, prompt_hi=2048, steps=256, w=32, sparsity_bp=5000,
                                hh_frac=0.01),
    "c5_llama7b_sp80": Workload("c5_llama7b_sp80", 5, b=256, h=32, d=128, dtype="f16",
                                prompt_lo=512, prompt_hi=2048, steps=256, w=32, sparsity_bp=8000,
                                hh_frac=0.01),
    "c5_llama7b_sp90": Workload("c5_llama7b_sp90", 5, b=256, h=32, d=128, dtype="f16",
                                prompt_lo=512, prompt_hi=2048, steps=256, w=32, sparsity_bp=9000,
                                hh_frac=0.01),
}

# Not one of the five: a single long-context sequence (32 heads, an 8192-token prompt), the shape for which the
# rows of a pair are spread over several workgroups (few pairs, long caches).
EXTRA: Dict[str, Workload] = {
    "x_long_context_b1": Workload("x_long_context_b1", 6, b=1, h=32, d=128, dtype="f16", prompt_lo=8192,
                                  prompt_hi=8192, steps=32, w=64, sparsity_bp=8000, hh_frac=0.01),
}


def _gen(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    x = 0x9E3779B97F4A7C15
    for k in key:
        x = (x * 6364136223846793005 + 1442695040888963407 + int(k)) % (1 << 63)
    g.manual_seed(x)
    return g


def prompt_lengths(wl: Workload) -> torch.Tensor:
    """int32 [b] prompt length per sequence (host tensor)."""
    if wl.prompt_lo == wl.prompt_hi:
        return torch.full((wl.b,), wl.prompt_lo, dtype=torch.int32)
    g = _gen("cpu", wl.seed, wl.config_id, 101)
    return torch.randint(wl.prompt_lo, wl.prompt_hi + 1, (wl.b,), generator=g, dtype=torch.int32)


def heavy_hitter_positions(wl: Workload, seq: int, s: int) -> torch.Tensor:
    """int64 [count] distinct prompt positions of sequence `seq` (host tensor)."""
    # outside the local window where there is one (w < 0 is the even split of Algorithm 1: no fixed window),
    # and always inside the prompt
    hi = max(1, min(s, s - max(wl.w, 0)))
    count = min(hi, max(1, int(round(wl.hh_frac * s))))
    g = _gen("cpu", wl.seed, wl.config_id, 202, seq)
    return torch.randperm(hi, generator=g)[:count].sort().values


def make_mu(wl: Workload, device) -> torch.Tensor:
    """float32 [b,h,d] per-(sequence, head) query direction."""
    g = _gen(device, wl.seed, wl.config_id, 303)
    return torch.randn((wl.b, wl.h, wl.d), generator=g, device=device, dtype=torch.float32)


def make_prompt(wl: Workload, device, slack: str = "zero") -> dict:
    """Post-prompt cache state.

    Returns K, V [b,h,cap,d] (workload dtype), pos [b,h,cap] int32, cache_len
    [b] int32, mu [b,h,d] float32, lengths (host list).  Slots beyond the prompt
    hold zeros, or NaN when slack == "nan" (to expose reads of invalid slots).
    """
    dt = wl.torch_dtype
    lens = prompt_lengths(wl)
    mu = make_mu(wl, device)
    fill = float("nan") if slack == "nan" else 0.0
    K = torch.full((wl.b, wl.h, wl.cap, wl.d), fill, device=device, dtype=dt)
    V = torch.full((wl.b, wl.h, wl.cap, wl.d), fill, device=device, dtype=dt)
    pos = torch.full((wl.b, wl.h, wl.cap), -1, device=device, dtype=torch.int32)
    for s_i in range(wl.b):
        s = int(lens[s_i])
        g = _gen(device, wl.seed, wl.config_id, 404, s_i)
        k = torch.randn((wl.h, s, wl.d), generator=g, device=device, dtype=torch.float32)
        v = torch.randn((wl.h, s, wl.d), generator=g, device=device, dtype=torch.float32)
        hh = heavy_hitter_positions(wl, s_i, s).to(device)
        unit = mu[s_i] / mu[s_i].norm(dim=-1, keepdim=True)            # [h,d]
        k[:, hh, :] += 3.0 * unit[:, None, :]
        K[s_i, :, :s, :] = k.to(dt)
        V[s_i, :, :s, :] = v.to(dt)
        pos[s_i, :, :s] = torch.arange(s, device=device, dtype=torch.int32)[None, :]
    return {
        "K": K, "V": V, "pos": pos,
        "cache_len": lens.to(device),
        "mu": mu,
        "lengths": [int(x) for x in lens],
    }


def make_q_tail(wl: Workload, mu: torch.Tensor, R: int) -> torch.Tensor:
    """[b,h,R,d] (workload dtype): the last R prompt queries; row r is position s-R+r."""
    g = _gen(mu.device, wl.seed, wl.config_id, 505)
    eps = torch.randn((wl.b, wl.h, R, wl.d), generator=g, device=mu.device, dtype=torch.float32)
    return ((mu[:, :, None, :] + eps) / math.sqrt(2.0)).to(wl.torch_dtype)


def make_step(wl: Workload, t: int, mu: torch.Tensor):
    """(q, k_new, v_new), each [b,h,d] in the workload dtype, for decode step t."""
    g = _gen(mu.device, wl.seed, wl.config_id, 606, t)
    shape = (wl.b, wl.h, wl.d)
    eps = torch.randn(shape, generator=g, device=mu.device, dtype=torch.float32)
    q = ((mu + eps) / math.sqrt(2.0)).to(wl.torch_dtype)
    k_new = torch.randn(shape, generator=g, device=mu.device, dtype=torch.float32).to(wl.torch_dtype)
    v_new = torch.randn(shape, generator=g, device=mu.device, dtype=torch.float32).to(wl.torch_dtype)
    return q, k_new, v_new


def algorithmic_bytes_per_pair(d: int, elem_bytes: int, m: int, keep: int, kv_int8: bool = False,
                               window_rows: int = 0) -> int:
    """Bytes one (sequence, head) pair must move in one decode step.

    m key rows + keep value rows + importance read and write over m slots + the
    four per-step rows (q, k_new, v_new, out) + the kept-index list.  With fp16,
    one layer's K plus V of one token over all heads is 4 * hidden bytes, the
    per-token figure of the paper's caching-time model (Section V-A).  With the
    8-bit compressed cache of Section V-B a cache row is d bytes, the per-step
    rows stay fp16, and the pair's four fp32 parameter rows are read as well.
    With the strict local attention sum over a ring of window_rows attention rows,
    the other window_rows - 1 rows are read over the m slots and this step's row
    is written over the kept ones (in place of the running sum's read).
    """
    if window_rows > 0:
        row = d * elem_bytes
        return row * m + row * keep + 4 * (window_rows - 1) * m + 4 * m + 4 * keep + 4 * row + 4 * keep
    if kv_int8:
        return d * m + d * keep + 8 * m + 4 * (2 * d) + 4 * (4 * d) + 4 * keep
    row = d * elem_bytes
    return row * m + row * keep + 8 * m + 4 * row + 4 * keep
