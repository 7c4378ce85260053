"""Seeded synthetic Q/K/V for one attention layer.

This module only draws random inputs. It holds none of the method's arithmetic, so both the
CPU oracle's tests and the HIP path's tests may feed from it.

The paper evaluates on real activations of LLaMA-2-7B/13B, LLaMA-3-8B and Mistral-7B
(Experimental Settings, "Models"); those weights and datasets are not available here. What is
kept of them is the attention-layer shape (heads, head_dim, MHA vs GQA). Token redundancy, the
property the method measures, is produced by a prototype-plus-noise recipe:

* per tensor X in {Q, K, V} and per head h of that tensor, a table of P prototype vectors,
  iid N(0, 1), shape [P, d];
* per (batch row b, position t) one token identity z[b, t], shared by every head and by
  Q, K and V, so a repeated token is redundant in all heads at once;
* X[b, h, t, :] = prototype[h][z[b, t]] + sigma_h * N(0, I), generated in fp32 and rounded
  once to the workload dtype.

Identity processes:
* "zipf": z iid with Pr[z = i] proportional to (i + 1)^-1.2, i = 0..P-1;
* "runs": runs of one identity repeated L times, L = min(Geometric(mean 8), 64), the run's
  identity drawn from the same Zipf law (near-identical repeats, a stress case for ties).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Tuple

import torch

SEED_BASE = 20251207 * 10


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str              # "f32" or "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq: int
    head_dim: int
    prune_ratios: Tuple[float, ...]
    n_prototypes: int
    identity: str           # "zipf" or "runs"
    sigma_lo: float         # noise sigma of the first half of the heads
    sigma_hi: float         # noise sigma of the second half of the heads
    seed: int

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five workloads of the benchmark definition, in order; index 1 is the one the headline
# metric is quoted on.
WORKLOADS = (
    Workload("cfg1_f32_mha32_n512", "f32", 1, 32, 32, 512, 128, (0.5,), 64, "zipf", 0.3, 0.3,
             SEED_BASE + 1),
    Workload("cfg2_llama2_7b_bf16_b8_n4096", "bf16", 8, 32, 32, 4096, 128, (0.25, 0.5), 256,
             "zipf", 0.3, 0.3, SEED_BASE + 2),
    Workload("cfg3_llama2_13b_bf16_b4_n4096", "bf16", 4, 40, 40, 4096, 128, (0.5,), 256, "zipf",
             0.1, 1.0, SEED_BASE + 3),
    Workload("cfg4_llama3_8b_gqa_bf16_b2_n8192", "bf16", 2, 32, 8, 8192, 128, (0.5,), 512,
             "zipf", 0.3, 0.3, SEED_BASE + 4),
    Workload("cfg5_mistral_7b_gqa_bf16_b1_n32768", "bf16", 1, 32, 8, 32768, 128, (0.5,), 512,
             "runs", 0.05, 0.05, SEED_BASE + 5),
)


def workload(index_or_name) -> Workload:
    if isinstance(index_or_name, int):
        return WORKLOADS[index_or_name]
    for w in WORKLOADS:
        if w.name == index_or_name:
            return w
    raise KeyError(index_or_name)


def scaled(w: Workload, **changes) -> Workload:
    """A copy of `w` with some fields replaced (smaller batch or seq for CPU-sized cases)."""
    return dataclasses.replace(w, **changes)


def _zipf_cdf(p: int, exponent: float = 1.2) -> torch.Tensor:
    weights = torch.arange(1, p + 1, dtype=torch.float64).pow(-exponent)
    cdf = torch.cumsum(weights / weights.sum(), 0)
    cdf[-1] = 1.0
    return cdf


def _draw_zipf(shape, p: int, gen: torch.Generator) -> torch.Tensor:
    u = torch.rand(shape, generator=gen, dtype=torch.float64)
    return torch.searchsorted(_zipf_cdf(p), u).clamp_(max=p - 1)


def token_identities(w: Workload, gen: torch.Generator) -> torch.Tensor:
    """z[b, t] in [0, P): int64 tensor of shape [batch, seq]."""
    if w.identity == "zipf":
        return _draw_zipf((w.batch, w.seq), w.n_prototypes, gen)
    if w.identity != "runs":
        raise ValueError(w.identity)
    z = torch.empty((w.batch, w.seq), dtype=torch.int64)
    p_stop = 1.0 / 8.0                      # geometric with mean 8
    for b in range(w.batch):
        # enough runs to cover the row even if every run had length 1 is wasteful; draw in
        # slabs and stop when the row is full
        filled = 0
        while filled < w.seq:
            k = max(64, (w.seq - filled) // 4)
            u = torch.rand(k, generator=gen, dtype=torch.float64)
            lengths = torch.floor(torch.log1p(-u) / math.log1p(-p_stop)).to(torch.int64) + 1
            lengths.clamp_(min=1, max=64)
            ids = _draw_zipf((k,), w.n_prototypes, gen)
            run = torch.repeat_interleave(ids, lengths)
            take = min(run.numel(), w.seq - filled)
            z[b, filled:filled + take] = run[:take]
            filled += take
    return z


def _head_sigmas(n_heads: int, w: Workload) -> torch.Tensor:
    s = torch.full((n_heads,), w.sigma_lo, dtype=torch.float32)
    s[n_heads // 2:] = w.sigma_hi
    return s


def make_qkv(w: Workload, device: str = "cpu"):
    """Return (Q, K, V, z): Q [B, Hq, n, d], K and V [B, Hkv, n, d] in the workload dtype
    (contiguous, CPU unless `device` says otherwise; generation always happens on the CPU so
    both consumers see identical values), and the identities z [B, n]."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed)
    z = token_identities(w, gen)
    out = []
    for n_heads in (w.n_q_heads, w.n_kv_heads, w.n_kv_heads):
        protos = torch.randn((n_heads, w.n_prototypes, w.head_dim), generator=gen,
                             dtype=torch.float32)
        sig = _head_sigmas(n_heads, w).view(n_heads, 1, 1)
        x = torch.empty((w.batch, n_heads, w.seq, w.head_dim), dtype=w.torch_dtype)
        for b in range(w.batch):
            noise = torch.randn((n_heads, w.seq, w.head_dim), generator=gen,
                                dtype=torch.float32)
            row = protos[:, z[b], :] + sig * noise
            x[b] = row.to(w.torch_dtype)
        out.append(x if device == "cpu" else x.to(device))
    return out[0], out[1], out[2], z


def make_random_qkv(batch, n_q_heads, n_kv_heads, seq, head_dim, dtype="f32", seed=0,
                    n_prototypes=16, sigma=0.3, identity="zipf"):
    """Small ad-hoc case with the same recipe (for edge-case tests)."""
    w = Workload("adhoc", dtype, batch, n_q_heads, n_kv_heads, seq, head_dim, (0.5,),
                 n_prototypes, identity, sigma, sigma, seed)
    return make_qkv(w)
