"""Seeded synthetic inputs with the shapes of the routed-LoRA serving workloads.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic, and both the GPU tests and the CPU oracle tests feed from
it so that they see the same stored values.  The paper evaluates on prompts of
public benchmarks (Sec. 4.1); the cost of the hot path depends on shapes only,
so Gaussian hidden states with LLaMA-2 shapes (Sec. 3.1, Sec. 4.3) stand in
for them.

Layouts produced (all row-major, contiguous):
  base weight of site m : [d2, d1]        (Eq. 1's W transposed, d1 contiguous)
  A of (tenant, site)   : [d1, r_t]       (Eq. 1's W^A)
  B of (tenant, site)   : [r_t, d2]       (Eq. 1's W^B)
  router weight         : [T, 7, d]       (Eq. 3's W_r, one per tenant, column-major)
  prompt hidden states  : [M_tok, d] with per-request (seq_start, seq_len)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

NMOD = 7
SITES = ("q", "k", "v", "o", "gate", "up", "down")


def site_dims(site: int, d: int, F: int) -> Tuple[int, int]:
    """(d1, d2) of the linear at `site` (Sec. 3.1: Q,K,V,O are d x d; G,U are d x F; D is F x d)."""
    return (F if site == 6 else d, F if site in (4, 5) else d)


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str  # "bf16" or "f32": storage type of every tensor
    d: int
    F: int
    L: int
    T: int
    B: int
    ranks: Tuple[int, ...]  # rank choices; one value = the same rank for every tenant
    prompt_len: Tuple[int, int]  # inclusive range of valid prompt lengths
    pad_to: int = 0  # > 0: each prompt occupies pad_to rows of H (right-padded); 0: packed
    decode_steps: int = 0
    pool: str = "mean"
    act: str = "identity"
    rmsnorm: bool = False
    tenants: str = "identity"  # "identity": request b -> tenant b; "uniform": drawn with replacement
    route_skew: Optional[Tuple[float, ...]] = None  # per-site probabilities of a constructed table
    seed: int = 0
    sigma_w: float = 0.02
    sigma_lora: float = 0.02
    sigma_router: float = 0.02  # router matrices and self-attention queries

    @property
    def torch_dtype(self):
        return {"bf16": torch.bfloat16, "f32": torch.float32}[self.dtype]


# The five serving configurations this repository is measured on.
CONFIGS = {
    "toy_fp32": Workload("toy_fp32", "f32", 256, 688, 1, 4, 4, (8,), (16, 16), decode_steps=8,
                         pool="mean", act="tanh", seed=0),
    "llama7b_layer_b32": Workload("llama7b_layer_b32", "bf16", 4096, 11008, 1, 32, 32, (32,), (256, 256),
                                  decode_steps=64, pool="mean", act="gelu", seed=1, sigma_lora=0.08),
    "llama7b_stack_b64": Workload("llama7b_stack_b64", "bf16", 4096, 11008, 32, 64, 64, (32,), (128, 1024),
                                  decode_steps=128, pool="mean", act="gelu", rmsnorm=True, tenants="uniform", seed=2,
                                  sigma_lora=0.08),
    "llama7b_prefill_b16": Workload("llama7b_prefill_b16", "bf16", 4096, 11008, 1, 16, 16, (32,), (1024, 2048),
                                    pad_to=2048, pool="mean", act="gelu", seed=3, sigma_lora=0.08),
    "llama13b_stack_b128": Workload("llama13b_stack_b128", "bf16", 5120, 13824, 40, 128, 128, (8, 16, 64),
                                    (128, 1024), decode_steps=32, rmsnorm=True, tenants="permutation",
                                    route_skew=(0.08, 0.08, 0.08, 0.08, 0.08, 0.30, 0.30), seed=4, sigma_lora=0.12),
}

_KIND = {"base": 1, "A": 2, "B": 3, "router": 4, "prompt": 5, "decode": 6, "tenant": 7, "rank": 8, "len": 9,
         "route": 10, "w_sa": 11}


def _gen(wl: Workload, kind: str, layer: int = 0, extra: int = 0, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(((wl.seed * 1_000_003 + _KIND[kind]) * 10_007 + layer) * 1_009 + extra)
    return g


def _normal(shape, sigma, wl, gen, device):
    x = torch.empty(shape, dtype=torch.float32, device=device)
    x.normal_(0.0, sigma, generator=gen)
    return x.to(wl.torch_dtype)


def tenant_ranks(wl: Workload) -> List[int]:
    if len(wl.ranks) == 1:
        return [wl.ranks[0]] * wl.T
    idx = torch.randint(0, len(wl.ranks), (wl.T,), generator=_gen(wl, "rank"))
    return [wl.ranks[i] for i in idx.tolist()]


def tenant_ids(wl: Workload) -> torch.Tensor:
    if wl.tenants == "identity":
        return (torch.arange(wl.B) % wl.T).to(torch.int32)
    if wl.tenants == "permutation":
        return torch.randperm(wl.T, generator=_gen(wl, "tenant"))[: wl.B].to(torch.int32)
    return torch.randint(0, wl.T, (wl.B,), generator=_gen(wl, "tenant")).to(torch.int32)


def base_weights(wl: Workload, layer: int, device="cpu") -> List[torch.Tensor]:
    out = []
    for m in range(NMOD):
        d1, d2 = site_dims(m, wl.d, wl.F)
        out.append(_normal((d2, d1), wl.sigma_w, wl, _gen(wl, "base", layer, m, device), device))
    return out


@dataclass
class LayerAdapters:
    """LoRA stacks of one layer: A[t][m] is [d1, r_t], B[t][m] is [r_t, d2]; views of one buffer per site."""

    A: List[List[torch.Tensor]]
    B: List[List[torch.Tensor]]
    rank: List[int]
    buffers: List[torch.Tensor] = field(default_factory=list)


def adapters(wl: Workload, layer: int, device="cpu", zero_B: bool = False) -> LayerAdapters:
    ranks = tenant_ranks(wl)
    rsum = sum(ranks)
    A = [[None] * NMOD for _ in range(wl.T)]
    Bm = [[None] * NMOD for _ in range(wl.T)]
    bufs = []
    for m in range(NMOD):
        d1, d2 = site_dims(m, wl.d, wl.F)
        bufA = _normal((rsum * d1,), wl.sigma_lora, wl, _gen(wl, "A", layer, m, device), device)
        bufB = _normal((rsum * d2,), wl.sigma_lora, wl, _gen(wl, "B", layer, m, device), device)
        if zero_B:
            bufB.zero_()
        bufs += [bufA, bufB]
        off = 0
        for t, r in enumerate(ranks):
            A[t][m] = bufA[off * d1:(off + r) * d1].view(d1, r)
            Bm[t][m] = bufB[off * d2:(off + r) * d2].view(r, d2)
            off += r
    return LayerAdapters(A, Bm, ranks, bufs)


def router_weights(wl: Workload, layer: int, device="cpu") -> torch.Tensor:
    return _normal((wl.T, NMOD, wl.d), wl.sigma_router, wl, _gen(wl, "router", layer, 0, device), device)


def selfattn_query(wl: Workload, layer: int, device="cpu") -> torch.Tensor:
    return _normal((wl.T, wl.d), wl.sigma_router, wl, _gen(wl, "w_sa", layer, 0, device), device)


def prompt_lengths(wl: Workload) -> torch.Tensor:
    lo, hi = wl.prompt_len
    return torch.randint(lo, hi + 1, (wl.B,), generator=_gen(wl, "len")).to(torch.int32)


def prompts(wl: Workload, layer: int, device="cpu"):
    """Hidden states entering `layer` for the B prompts: (H [M_tok, d], seq_start [B], seq_len [B])."""
    lens = prompt_lengths(wl)
    if wl.pad_to:
        starts = (torch.arange(wl.B) * wl.pad_to).to(torch.int32)
        M_tok = wl.B * wl.pad_to
    else:
        starts = (torch.cumsum(lens, 0) - lens).to(torch.int32)
        M_tok = int(lens.sum())
    H = _normal((M_tok, wl.d), 1.0, wl, _gen(wl, "prompt", layer, 0, device), device)
    return H, starts, lens


def decode_input(wl: Workload, step: int, device="cpu") -> torch.Tensor:
    return _normal((wl.B, wl.d), 1.0, wl, _gen(wl, "decode", 0, step, device), device)


def constructed_routes(wl: Workload) -> torch.Tensor:
    """A route table [L, B] drawn from `route_skew` (the table is an input of decode)."""
    p = torch.tensor(wl.route_skew if wl.route_skew else [1.0 / NMOD] * NMOD, dtype=torch.float64)
    r = torch.multinomial(p, wl.L * wl.B, replacement=True, generator=_gen(wl, "route"))
    return r.view(wl.L, wl.B).to(torch.uint8)


def small_int_tensor(shape, lo, hi, dtype, seed, device="cpu") -> torch.Tensor:
    """Integers in [lo, hi] stored as `dtype`: products and short sums stay exact in every precision."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randint(lo, hi + 1, shape, generator=g).to(dtype).to(device)


def as_numpy(t: torch.Tensor) -> np.ndarray:
    """Host view of a tensor's stored values; bf16 becomes its uint16 bit pattern."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def adapters_as_numpy(ad: LayerAdapters):
    """(A, B, rank) with every matrix as a contiguous host array, in the oracle's storage convention."""
    A = [[np.ascontiguousarray(as_numpy(a)) for a in row] for row in ad.A]
    B = [[np.ascontiguousarray(as_numpy(b)) for b in row] for row in ad.B]
    return A, B, list(ad.rank)
