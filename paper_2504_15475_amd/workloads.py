"""Seeded synthetic logits for the five benchmark workloads.

This module only draws inputs; it contains none of the method's arithmetic, so
that the GPU library and the CPU oracle can both be fed from it.  The tensors
stand in for next-token logits of a large target model and a small draft model
at LLM vocabulary sizes (the paper's experiments, Section 5, use text prompts
and trained weights that are not available here).

The data generator is independent of the race seed: torch.Generator seeded
with 1000 + workload index on the device the tensors are created on.  Values
are drawn in fp32 and rounded to the workload dtype (round-to-nearest-even), so
a host copy of the returned tensors has bit-identical contents.
"""
import math
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    variant: str          # "sequence" | "multi" | "tree" | "arrival_tree"
    B: int
    k: int                # drafted positions per sequence (tree: unused, 0)
    V: int
    dtype: torch.dtype
    temperature: float
    seed: int
    m: int = 1            # drafts per prompt (multi)
    N: int = 0            # tree nodes
    level_sizes: tuple = ()

    @property
    def race_elements(self) -> int:
        """Logits read by one pass (the unit of the throughput metric)."""
        if self.variant == "tree":
            return self.B * 2 * self.N * self.V
        if self.variant == "arrival_tree":  # one target row per context, one draft row per context with a child
            with_child = len(set(int(p) for p in tree_parents(self)))
            return self.B * (self.N + 1 + with_child) * self.V
        return self.B * self.m * (2 * self.k + 1) * self.V

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == torch.float32 else 2

    @property
    def logit_bytes(self) -> int:
        return self.race_elements * self.elem_bytes


WORKLOADS = (
    Workload(0, "seq_B1_k4_V32000_f32", "sequence", B=1, k=4, V=32000, dtype=torch.float32, temperature=1.0, seed=0),
    Workload(1, "seq_B64_k8_V128256_bf16", "sequence", B=64, k=8, V=128256, dtype=torch.bfloat16, temperature=1.0,
             seed=1),
    Workload(2, "seq_B256_k16_V152064_f32", "sequence", B=256, k=16, V=152064, dtype=torch.float32, temperature=0.7,
             seed=2),
    Workload(3, "multi_B32_m8_k8_V128256_bf16", "multi", B=32, k=8, V=128256, dtype=torch.bfloat16, temperature=1.0,
             seed=3, m=8),
    Workload(4, "tree_B16_N64_V256000_bf16", "tree", B=16, k=0, V=256000, dtype=torch.bfloat16, temperature=1.0,
             seed=4, N=64, level_sizes=(4, 8, 12, 14, 14, 12)),
)


# The tree of workload 4 verified as Algorithm 5 states it: one row per context (N + 1 of them), the children of a
# context are the first arrivals of its race under the draft model (rank = order among siblings).
ARRIVAL_TREE = Workload(5, "arrival_tree_B16_N64_V256000_bf16", "arrival_tree", B=16, k=0, V=256000,
                        dtype=torch.bfloat16, temperature=1.0, seed=4, N=64, level_sizes=(4, 8, 12, 14, 14, 12))


def shrink(w: Workload, **kw) -> Workload:
    """Same recipe at another shape (parity tests use smaller B / k / V / N)."""
    if "N" in kw and "level_sizes" not in kw:
        kw["level_sizes"] = ()
    return replace(w, **kw)


def tree_parents(w: Workload) -> np.ndarray:
    """Flat parent array: nodes numbered level by level, depth-1 nodes hang off the root (-1),
    deeper nodes pick a parent uniformly in the previous level."""
    rng = np.random.default_rng(w.seed)
    sizes = list(w.level_sizes)
    if not sizes:  # shrunken tree: spread N nodes over at most 6 levels, at least one node per level used
        depth = min(6, w.N)
        base, extra = divmod(w.N, depth)
        sizes = [base + (1 if i < extra else 0) for i in range(depth)]
    assert sum(sizes) == w.N
    parent = np.empty(w.N, dtype=np.int32)
    start_prev, n = 0, 0
    for lvl, sz in enumerate(sizes):
        for _ in range(sz):
            parent[n] = -1 if lvl == 0 else start_prev + rng.integers(0, sizes[lvl - 1])
            n += 1
        if lvl > 0:
            start_prev += sizes[lvl - 1]
    return parent


def sibling_ranks(parent: np.ndarray) -> np.ndarray:
    """rank[n] = how many earlier nodes share n's parent (children of a context take its arrivals in order)."""
    seen = {}
    rank = np.empty(len(parent), dtype=np.int32)
    for n, p in enumerate(parent):
        rank[n] = seen.get(int(p), 0)
        seen[int(p)] = rank[n] + 1
    return rank


def _randn(shape, gen, device, chunk_rows=None):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def make_inputs(w: Workload, device="cpu"):
    """-> dict(draft, target[, parent]) of tensors on `device` in the workload dtype.

    sequence: draft [B,k,V], target [B,k+1,V];  multi: draft [B,m,k,V], target [B,m,k+1,V];
    tree: draft, target [B,N,V] and parent int32 [N];  arrival_tree: draft, target [B,N+1,V], parent, rank int32 [N].
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000 + w.index)
    B, k, V, m = w.B, w.k, w.V, w.m
    if w.index == 0:
        target = 3.0 * _randn((B, k + 1, V), gen, dev)
        draft = target[:, :k] + 0.5 * _randn((B, k, V), gen, dev)
    elif w.index == 1:
        perm = torch.randperm(V, generator=gen, device=dev)
        rank = torch.empty(V, device=dev, dtype=torch.float32)
        rank[perm] = torch.arange(1, V + 1, device=dev, dtype=torch.float32)
        prior = -1.1 * torch.log(rank)  # Zipf(s = 1.1) log-prior, one frequency order for the vocabulary
        target = 2.5 * _randn((B, k + 1, V), gen, dev) + prior
        draft = target[:, :k] + 0.7 * _randn((B, k, V), gen, dev)
    elif w.index == 2:
        target = 4.0 * _randn((B, k + 1, V), gen, dev)
        idx = torch.randint(0, V, (B, k + 1, 20), generator=gen, device=dev)
        target.scatter_(-1, idx, target.gather(-1, idx) + 8.0)  # duplicates collapse to one boost
        draft = 0.8 * target[:, :k] + _randn((B, k, V), gen, dev)
    elif w.index == 3:
        base = 3.0 * _randn((B, 1, k + 1, V), gen, dev)
        target = base + 0.3 * _randn((B, m, k + 1, V), gen, dev)
        draft = target[:, :, :k] + 0.8 * _randn((B, m, k, V), gen, dev)
    elif w.index == 4:
        N = w.N
        target = 3.0 * _randn((B, N, V), gen, dev)
        draft = target + 0.6 * _randn((B, N, V), gen, dev)
    elif w.index == 5:
        C = w.N + 1
        target = 3.0 * _randn((B, C, V), gen, dev)
        draft = target + 0.6 * _randn((B, C, V), gen, dev)
    else:
        raise ValueError(w.index)
    out = dict(draft=draft.to(w.dtype).contiguous(), target=target.to(w.dtype).contiguous())
    if w.variant in ("tree", "arrival_tree"):
        par = tree_parents(w)
        out["parent"] = torch.from_numpy(par).to(dev)
        if w.variant == "arrival_tree":
            out["rank"] = torch.from_numpy(sibling_ranks(par)).to(dev)
    return out


def describe(w: Workload) -> str:
    shape = {"sequence": f"B={w.B} k={w.k}", "multi": f"B={w.B} m={w.m} k={w.k}", "tree": f"B={w.B} N={w.N}",
             "arrival_tree": f"B={w.B} N={w.N}"}[w.variant]
    dt = "fp32" if w.dtype == torch.float32 else "bf16"
    return f"{w.variant} {shape} V={w.V} {dt} T={w.temperature} seed={w.seed}"
