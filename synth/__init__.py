"""Seeded synthetic inputs for the decode hot path (shared by the tests, the oracle-side
checks and the bench).  This module holds no arithmetic of the method: it only draws random
tensors with the shapes, value distributions and structure of the workloads and lays them out
in memory.  Nothing here imports the HIP library or the oracle.

Value recipe: every bf16 tensor is an fp32 N(0,1) draw rounded to bf16 by torch on the target
device from a seeded ``torch.Generator`` (so CPU and GPU draws differ, but both sides of a
comparison always receive the same tensor).  Keys can carry "outlier" tokens (a Bernoulli
subset of whole rows scaled by 8).  Sequence lengths are fixed, uniform or log-uniform.  The
KV cache is either contiguous ``[B,Hkv,S_max,d]`` or a paged pool ``[n_pages,Hkv,page,d]``
with a shuffled page table.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import torch


@dataclass
class Workload:
    """Shape of one decode step of one attention layer."""
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int = 128
    Dg: int = 128
    block_size: int = 64
    seqlen: int = 0                    # fixed length, or 0 when a range is given
    seqlen_range: Optional[tuple] = None   # (lo, hi) inclusive
    seqlen_dist: str = "fixed"         # fixed | uniform | loguniform
    paged: bool = False
    budget_tokens: int = 0             # token budget (top-k mode), 0 = use budget_frac
    budget_frac: float = 0.0           # fraction of each sequence's blocks to keep
    outlier_frac: float = 0.0          # fraction of key rows scaled by outlier_scale
    outlier_scale: float = 8.0
    gate_inputs: str = "random"        # random | blockmean
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)


# The five configurations named by the benchmark definition, at full size.
CONFIGS = {
    "c1": Workload("c1", B=1, Hq=8, Hkv=2, block_size=64, seqlen=4096, budget_tokens=1024,
                   gate_inputs="blockmean", seed=1),
    "c2": Workload("c2", B=16, Hq=32, Hkv=8, block_size=64, seqlen=32768, budget_tokens=4096, seed=2),
    "c3": Workload("c3", B=32, Hq=32, Hkv=8, block_size=128, seqlen_range=(8192, 65536),
                   seqlen_dist="uniform", paged=True, budget_frac=0.10, outlier_frac=0.01, seed=3),
    "c4": Workload("c4", B=64, Hq=40, Hkv=8, block_size=64, seqlen=131072, budget_tokens=13107, seed=4),
    "c5": Workload("c5", B=128, Hq=32, Hkv=8, block_size=64, seqlen_range=(4096, 131072),
                   seqlen_dist="loguniform", paged=True, budget_frac=0.10, seed=5),
}


def scaled(w: Workload, **overrides) -> Workload:
    """A copy of a workload with some fields replaced (used for small parity cases)."""
    d = dict(w.__dict__)
    d.update(overrides)
    d["extra"] = dict(w.extra)
    return Workload(**d)


def generator(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def randn_bf16(shape, device, gen: torch.Generator) -> torch.Tensor:
    """N(0,1) rounded to bf16, drawn in place to avoid an fp32 temporary of the same shape."""
    t = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = t.view(-1)
    step = 1 << 28
    for s in range(0, flat.numel(), step):
        flat[s:s + step].normal_(0.0, 1.0, generator=gen)
    return t


def draw_seqlens(w: Workload, gen_cpu: torch.Generator) -> torch.Tensor:
    """[B] int32 sequence lengths (tokens already in the cache, the current one included)."""
    if w.seqlen_dist == "fixed":
        return torch.full((w.B,), w.seqlen, dtype=torch.int32)
    lo, hi = w.seqlen_range
    u = torch.rand(w.B, generator=gen_cpu, dtype=torch.float64)
    if w.seqlen_dist == "uniform":
        s = lo + torch.floor(u * (hi - lo + 1))
    elif w.seqlen_dist == "loguniform":
        s = torch.round(torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))
    else:
        raise ValueError(w.seqlen_dist)
    return s.clamp(lo, hi).to(torch.int32)


@dataclass
class DecodeInputs:
    w: Workload
    seqlens: torch.Tensor              # [B] int32 (on device)
    seqlens_cpu: torch.Tensor
    q: torch.Tensor                    # [B,Hq,d] bf16
    k: torch.Tensor                    # contiguous [B,Hkv,S_max,d] or pool [n_pages,Hkv,page,d]
    v: torch.Tensor
    page_table: Optional[torch.Tensor]  # [B,max_pages] int32 or None
    page_size: int
    q_gate: torch.Tensor               # [B,Hkv,Dg] bf16
    kc: torch.Tensor                   # [B,Hkv,nb_max,Dg] bf16
    nb_max: int
    budget_blocks: Optional[torch.Tensor]  # [B] int32 (device) or None
    budget_blocks_cpu: Optional[torch.Tensor]
    max_sel: int


def _block_means(k: torch.Tensor, block: int, nb_max: int) -> torch.Tensor:
    """Per-block mean of a contiguous cache [B,Hkv,S,d] -> [B,Hkv,nb_max,d] bf16 (the tail
    block, if partial, averages what is there).  Used only to give a tiny workload a gate
    input that is correlated with the keys."""
    B, H, S, d = k.shape
    out = torch.zeros(B, H, nb_max, d, dtype=torch.float32, device=k.device)
    nfull = S // block
    if nfull:
        out[:, :, :nfull] = k[:, :, :nfull * block].float().view(B, H, nfull, block, d).mean(3)
    if nfull < nb_max and S > nfull * block:
        out[:, :, nfull] = k[:, :, nfull * block:].float().mean(2)
    return out.to(torch.bfloat16)


def make_inputs(w: Workload, device="cpu", seed: Optional[int] = None) -> DecodeInputs:
    """Draw every tensor of one decode step for workload ``w`` on ``device``."""
    seed = w.seed if seed is None else seed
    dev = torch.device(device)
    gen = generator(dev, seed)
    gen_cpu = generator("cpu", seed + 7919)
    seqlens_cpu = draw_seqlens(w, gen_cpu)
    S_max = int(seqlens_cpu.max().item()) if w.B else 0
    b = w.block_size
    nb_max = max(1, (S_max + b - 1) // b)

    q = randn_bf16((w.B, w.Hq, w.d), dev, gen)
    page_table = None
    page_size = 0
    if not w.paged:
        S_alloc = nb_max * b
        k = randn_bf16((w.B, w.Hkv, S_alloc, w.d), dev, gen)
        v = randn_bf16((w.B, w.Hkv, S_alloc, w.d), dev, gen)
    else:
        page_size = b
        pages_per_seq = (seqlens_cpu.to(torch.int64) + page_size - 1) // page_size
        n_pages = int(pages_per_seq.sum().item()) + 1       # page 0 is a spare nobody maps
        k = randn_bf16((n_pages, w.Hkv, page_size, w.d), dev, gen)
        v = randn_bf16((n_pages, w.Hkv, page_size, w.d), dev, gen)
        perm = torch.randperm(n_pages - 1, generator=gen_cpu) + 1
        pt = torch.zeros(w.B, nb_max, dtype=torch.int32)
        o = 0
        for i in range(w.B):
            n = int(pages_per_seq[i])
            pt[i, :n] = perm[o:o + n].to(torch.int32)
            o += n
        page_table = pt.to(dev)

    if w.outlier_frac > 0:
        rows = k.shape[0] * k.shape[1] * k.shape[2]
        mask = torch.rand(rows, device=dev, generator=gen) < w.outlier_frac
        kf = k.view(rows, w.d)
        kf[mask] = (kf[mask].float() * w.outlier_scale).to(torch.bfloat16)

    if w.gate_inputs == "blockmean":
        assert not w.paged
        q_gate = q.float().view(w.B, w.Hkv, w.g, w.d).mean(2).to(torch.bfloat16)
        kc = _block_means(k[:, :, :S_max], b, nb_max)
    else:
        q_gate = randn_bf16((w.B, w.Hkv, w.Dg), dev, gen)
        kc = randn_bf16((w.B, w.Hkv, nb_max, w.Dg), dev, gen)

    budget_blocks = budget_blocks_cpu = None
    if w.budget_tokens > 0:
        max_sel = min((w.budget_tokens + b - 1) // b, nb_max)
    else:
        budget_blocks_cpu = block_budgets(seqlens_cpu, b, w.budget_frac)
        budget_blocks = budget_blocks_cpu.to(dev)
        max_sel = int(budget_blocks_cpu.max().item())

    return DecodeInputs(w=w, seqlens=seqlens_cpu.to(dev), seqlens_cpu=seqlens_cpu, q=q, k=k, v=v,
                        page_table=page_table, page_size=page_size, q_gate=q_gate, kc=kc,
                        nb_max=nb_max, budget_blocks=budget_blocks,
                        budget_blocks_cpu=budget_blocks_cpu, max_sel=max_sel)


def block_budgets(seqlens_cpu: torch.Tensor, block_size: int, frac: float) -> torch.Tensor:
    """[B] int32 per-sequence block budgets: the fraction ``frac`` (in thousandths) of each sequence's
    blocks, rounded up, at least one.  Integer arithmetic only."""
    nb_i = (seqlens_cpu.to(torch.int64) + block_size - 1) // block_size
    num = int(round(frac * 1000))
    return torch.clamp((nb_i * num + 999) // 1000, min=1).to(torch.int32)


def random_block_lists(B: int, Hkv: int, nb_per_seq, k_per_seq, max_sel: int, gen_cpu: torch.Generator,
                       ascending: bool = True):
    """Uniformly random block lists: for each (sequence, kv head) ``k_per_seq[i]`` distinct block
    ids below ``nb_per_seq[i]``; -1 padded to max_sel.  Returns (block_idx int32, nblk int32)."""
    idx = torch.full((B, Hkv, max_sel), -1, dtype=torch.int32)
    cnt = torch.zeros(B, Hkv, dtype=torch.int32)
    for i in range(B):
        nb = int(nb_per_seq[i])
        k = min(int(k_per_seq[i]), nb, max_sel)
        for h in range(Hkv):
            sel = torch.randperm(nb, generator=gen_cpu)[:k]
            if ascending:
                sel = torch.sort(sel).values
            idx[i, h, :k] = sel.to(torch.int32)
            cnt[i, h] = k
    return idx, cnt


def rope_tables(n_pos: int, dim: int, base: float = 1.0e6, device="cpu"):
    """cos/sin tables [n_pos, dim/2] fp32 of the rotary embedding: angle = pos * base^(-2c/dim),
    evaluated in fp64 and rounded once (base 1e6 as in the Qwen3 family).  These are inputs of the
    gate front-end calls, like any other tensor."""
    c = torch.arange(dim // 2, dtype=torch.float64)
    inv = torch.pow(torch.tensor(base, dtype=torch.float64), -2.0 * c / dim)
    ang = torch.arange(n_pos, dtype=torch.float64)[:, None] * inv[None, :]
    return torch.cos(ang).float().to(device), torch.sin(ang).float().to(device)


def gate_weights(w: Workload, device, gen: torch.Generator):
    """Random bf16 gate projections: Wq [Hkv, Dg, g*d] and Wk [Hkv, Dg, 3d], N(0,1)/sqrt(fan-in)."""
    wq = torch.empty(w.Hkv, w.Dg, w.g * w.d, dtype=torch.float32, device=device).normal_(generator=gen)
    wk = torch.empty(w.Hkv, w.Dg, 3 * w.d, dtype=torch.float32, device=device).normal_(generator=gen)
    return ((wq / math.sqrt(w.g * w.d)).to(torch.bfloat16), (wk / math.sqrt(3 * w.d)).to(torch.bfloat16))
