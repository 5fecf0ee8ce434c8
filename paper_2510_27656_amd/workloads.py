"""Seeded synthetic inputs for the MoE dispatch/combine shuffle.

This module only draws inputs (hidden states, router choices, router weights).
It holds none of the shuffle's arithmetic and is the one module that both the
CPU oracle's tests and the HIP path's tests/bench use, so both sides see the
same bytes.

The five named workloads stand in for the paper's kernel microbenchmark
(section "Kernel Microbenchmarks": DeepSeek-V3/R1 shape, hidden 7168, 128-token
decode batches and 4096-token prefill chunks, every token sent to 8 random
experts); no dataset or trained router is involved.

Router recipe (harness side, not part of the library): fp32 logits ~ N(0,1)
(+ an optional popularity bias), fp32 softmax over all experts, the K largest
probabilities in descending order with ties going to the lower expert id, and
weights = selected probabilities divided by their fp32 sum.
"""
from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_ranks: int
    n_experts: int
    tokens: int            # tokens per rank (max_tokens)
    hidden: int
    top_k: int
    seed: int
    dispatch_dtype: str = "bf16"      # "bf16" | "e4m3"
    expert: str = "scale"             # "identity" | "scale"  (stand-in expert stage)
    zipf_alpha: float = 0.0           # 0 = uniform routing
    zipf_beta: float = 0.0            # temperature on the popularity bias
    ragged: bool = False              # draw a different token count per rank

    @property
    def experts_per_rank(self):
        return self.n_experts // self.n_ranks


# Popularity temperatures were fixed once by bisection so that the hottest expert
# receives about ten times the mean load with these seeds (the realised ratio is
# reported by describe()).
WORKLOADS = {
    "tiny": Workload("tiny", 2, 8, 16, 256, 2, seed=0, expert="identity"),
    "dsv3_decode": Workload("dsv3_decode", 32, 256, 128, 7168, 8, seed=2),
    "dsv3_prefill": Workload("dsv3_prefill", 32, 256, 4096, 7168, 8, seed=3),
    "qwen3_skew": Workload("qwen3_skew", 16, 128, 256, 2048, 8, seed=4,
                           zipf_alpha=1.2, zipf_beta=0.444),
    "dsv3_fp8": Workload("dsv3_fp8", 32, 256, 128, 7168, 8, seed=5,
                         dispatch_dtype="e4m3", zipf_alpha=1.0, zipf_beta=0.325),
}


@dataclass
class Inputs:
    wl: Workload
    x: np.ndarray            # uint16 [N][T][H]  bf16 bit patterns
    indices: np.ndarray      # int32  [N][T][K]
    weights: np.ndarray      # float32 [N][T][K]
    num_tokens: np.ndarray   # int32  [N]
    expert_gain: np.ndarray  # float32 [E]  stand-in expert: y = bf16(float(x) * gain[e])
    popularity_rank: Optional[np.ndarray] = None


def _bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def route(logits: torch.Tensor, k: int):
    """Top-k of the fp32 softmax, ties to the lower expert id, weights renormalised."""
    probs = torch.softmax(logits.float(), dim=-1)
    order = torch.sort(probs, dim=-1, descending=True, stable=True)
    sel_p = order.values[:, :k].contiguous()
    sel_i = order.indices[:, :k].contiguous()
    w = sel_p / sel_p.sum(dim=-1, keepdim=True)
    return sel_i.to(torch.int32).numpy(), w.to(torch.float32).numpy()


def make_inputs(wl: Workload, with_x: bool = True) -> Inputs:
    N, E, T, H, K = wl.n_ranks, wl.n_experts, wl.tokens, wl.hidden, wl.top_k
    x = np.zeros((N, T, H), np.uint16) if with_x else np.zeros((N, T, 0), np.uint16)
    indices = np.zeros((N, T, K), np.int32)
    weights = np.zeros((N, T, K), np.float32)
    num_tokens = np.full((N,), T, np.int32)
    bias = None
    pop = None
    if wl.zipf_alpha > 0:
        gp = torch.Generator().manual_seed(wl.seed * 1000 + 999)
        pop = torch.randperm(E, generator=gp) + 1          # popularity rank 1..E per expert
        bias = (-wl.zipf_alpha * wl.zipf_beta) * torch.log(pop.float())
    if wl.ragged:
        gr = torch.Generator().manual_seed(wl.seed * 1000 + 998)
        num_tokens = torch.randint(0, T + 1, (N,), generator=gr).to(torch.int32).numpy()
        num_tokens[0] = T                                   # one full rank
        if N > 2:
            num_tokens[N - 2] = 0                           # one empty rank
    for r in range(N):
        g = torch.Generator().manual_seed(wl.seed * 1000 + r)
        if with_x:
            x[r] = _bf16_bits(torch.randn(T, H, generator=g))
        gl = torch.Generator().manual_seed(wl.seed * 1000 + 500 + r)   # router stream
        logits = torch.randn(T, E, generator=gl)
        if bias is not None:
            logits = logits + bias
        indices[r], weights[r] = route(logits, K)
    if wl.expert == "identity":
        gain = np.ones((E,), np.float32)
    else:
        gain = (1.0 + np.arange(E, dtype=np.float32) / 256.0).astype(np.float32)
    return Inputs(wl, x, indices, weights, num_tokens, gain,
                  None if pop is None else pop.numpy())


def describe(inp: Inputs) -> dict:
    """Realised routing statistics of a drawn workload (plain counting)."""
    wl = inp.wl
    N, E, K = wl.n_ranks, wl.n_experts, wl.top_k
    El = E // N
    load = np.zeros(E, np.int64)
    D = 0
    for s in range(N):
        idx = inp.indices[s, :inp.num_tokens[s]]
        load += np.bincount(idx.reshape(-1), minlength=E)
        owners = np.sort(idx // El, axis=1)
        D += int(idx.shape[0] + (np.diff(owners, axis=1) != 0).sum())
    ttot = int(inp.num_tokens.sum())
    rank_rows = load.reshape(N, El).sum(1)
    return {
        "tokens_total": ttot,
        "pairs": int(ttot * K),
        "dedup_rows": D,
        "dedup_per_token": D / max(ttot, 1),
        "hottest_expert_over_mean": float(load.max() / max(load.mean(), 1e-9)),
        "busiest_rank_over_mean": float(rank_rows.max() / max(rank_rows.mean(), 1e-9)),
        "max_rank_rows": int(rank_rows.max()),
    }


def custom(name, n_ranks, n_experts, tokens, hidden, top_k, seed, **kw) -> Workload:
    return Workload(name, n_ranks, n_experts, tokens, hidden, top_k, seed=seed, **kw)


def token_chunk(inp: Inputs, t0: int, chunk: int) -> Inputs:
    """Tokens [t0, t0 + chunk) of every rank as a workload of its own (same routing,
    same hidden states): what one pass of a chunked prefill hands to the shuffle.
    A last, shorter chunk is padded with absent tokens to the same shape."""
    from dataclasses import replace
    wl = replace(inp.wl, name=f"{inp.wl.name}[{t0}:{t0 + chunk}]", tokens=chunk)
    n = min(chunk, inp.wl.tokens - t0)
    nt = np.clip(inp.num_tokens - t0, 0, n).astype(np.int32)

    def cut(a):
        out = np.zeros((a.shape[0], chunk) + a.shape[2:], a.dtype)
        out[:, :n] = a[:, t0:t0 + n]
        return out
    idx = cut(inp.indices)
    idx[:, n:] = np.arange(inp.wl.top_k, dtype=np.int32)     # absent tokens still need valid-looking ids
    return Inputs(wl, cut(inp.x), idx, cut(inp.weights), nt, inp.expert_gain, inp.popularity_rank)
