"""Seeded synthetic inputs shaped like the paper's long-reasoning KV caches.

This module only draws random numbers and shapes tensors; none of the method's arithmetic lives
here.  It serves both the GPU path and the CPU oracle (each receives the same tensors / index
lists as plain inputs).

Recipe (per KV head, i.e. per unit): M Gaussian modes with centers 2*N(0,1) in 128 dimensions;
four fixed "outlier" channels per head whose center coordinates are multiplied by 8; every token
draws a mode uniformly and adds N(0, 0.3) noise; values are N(0,1); a query head is a noisy copy
(N(0, 0.3)) of one independently drawn center.  Everything is rounded to bf16.
"""
from __future__ import annotations

import dataclasses

import torch

HEAD_DIM = 128


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    context: int
    levels: int
    n_fine: int
    n_coarse: int
    modes: int
    key_budgets: tuple
    block_w: int = 8192
    block_alpha: int = 4096
    kmeans_iters: int = 10
    # config 4 only
    gen_tokens: int = 0
    update_every: int = 128
    new_fine_per_update: int = 16
    new_coarse_per_update: int = 2
    refine_iters: int = 3

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five workloads of the benchmark definition.  Budgets are in keys.
WORKLOADS = {
    "cfg0_tiny": Workload("cfg0_tiny", 1, 4, 1, 4096, 1, 64, 0, 64, (256,), block_w=0, block_alpha=0),
    "cfg1_qwen3_8b_32k": Workload("cfg1_qwen3_8b_32k", 1, 32, 8, 32768, 2, 1024, 64, 1024, (4096,)),
    "cfg2_14b_64k": Workload("cfg2_14b_64k", 4, 40, 8, 65536, 2, 2048, 128, 2048, (4096,)),
    "cfg3_128k_b16": Workload("cfg3_128k_b16", 16, 32, 8, 131072, 2, 4096, 256, 4096, (8192, 4096)),
    "cfg4_online": Workload("cfg4_online", 8, 32, 8, 8192, 2, 256, 32, 256, (1024,), gen_tokens=16384),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_modes(units: int, modes: int, device, seed: int):
    """Mode centers [units, modes, 128] (fp32) with the four outlier channels already scaled."""
    g = _gen(device, seed)
    centers = 2.0 * torch.randn(units, modes, HEAD_DIM, generator=g, device=device)
    gc = _gen("cpu", seed + 7)
    for u in range(units):
        ch = torch.randperm(HEAD_DIM, generator=gc)[:4].to(device)
        centers[u, :, ch] *= 8.0
    return centers


def make_tree_modes(units: int, modes: int, fan: int, device, seed: int, spread: float = 0.6):
    """Mode centers with two scales of structure, for accuracy studies: modes / fan parent centers
    2*N(0,1)*sqrt(1 - spread^2), every mode = its parent + 2*N(0,1)*spread (same overall variance as
    :func:`make_modes`, no outlier channels).  Returns key centers and, drawn the same way from other
    random numbers, value centers (both [units, modes, 128] fp32), so that tokens of one mode, and
    to a lesser degree of sibling modes, carry similar values."""
    g = _gen(device, seed)
    parents = modes // fan
    out = []
    for _ in range(2):
        top = 2.0 * (1.0 - spread * spread) ** 0.5 * torch.randn(units, parents, 1, HEAD_DIM, generator=g, device=device)
        sub = 2.0 * spread * torch.randn(units, parents, fan, HEAD_DIM, generator=g, device=device)
        out.append((top + sub).reshape(units, parents * fan, HEAD_DIM))
    return out[0], out[1]


def draw_tokens(centers: torch.Tensor, n_tokens: int, seed: int, noise: float = 0.3, chunk_units: int = 8,
                value_centers: torch.Tensor = None, value_scale: float = 0.5):
    """Keys and values for every unit: K, V bf16 [units, n_tokens, 128].  With value_centers
    ([units, modes, 128]) a token's value is value_scale * (the value center of its mode + N(0,1))
    instead of plain N(0,1)."""
    units, modes, d = centers.shape
    device = centers.device
    g = _gen(device, seed)
    K = torch.empty(units, n_tokens, d, dtype=torch.bfloat16, device=device)
    V = torch.empty(units, n_tokens, d, dtype=torch.bfloat16, device=device)
    for u0 in range(0, units, chunk_units):
        u1 = min(units, u0 + chunk_units)
        mode = torch.randint(0, modes, (u1 - u0, n_tokens), generator=g, device=device)
        idx = mode.unsqueeze(-1).expand(-1, -1, d)
        k = torch.gather(centers[u0:u1], 1, idx)
        k += noise * torch.randn(u1 - u0, n_tokens, d, generator=g, device=device)
        K[u0:u1] = k.to(torch.bfloat16)
        v = torch.randn(u1 - u0, n_tokens, d, generator=g, device=device)
        if value_centers is not None:
            v = value_scale * (v + torch.gather(value_centers[u0:u1], 1, idx))
        del k, idx, mode
        V[u0:u1] = v.to(torch.bfloat16)
    return K, V


def draw_queries(centers: torch.Tensor, group: int, n_sets: int, seed: int, noise: float = 0.3,
                 softness: float = 1.0):
    """Queries bf16 [n_sets, units, group, 128]; each head copies one random center plus noise.
    softness < 1 shrinks the query so that attention is less peaked (centroid terms carry mass)."""
    units, modes, d = centers.shape
    device = centers.device
    g = _gen(device, seed)
    m = torch.randint(0, modes, (n_sets, units, group), generator=g, device=device)
    base = centers[torch.arange(units, device=device).view(1, units, 1), m]
    q = base + noise * torch.randn(n_sets, units, group, d, generator=g, device=device)
    return (softness * q).to(torch.bfloat16)


def drift_modes(centers: torch.Tensor, seed: int, step: float = 0.05):
    """One random-walk step of every mode center (generation phase of the online workload)."""
    g = _gen(centers.device, seed)
    return centers + step * torch.randn(centers.shape, generator=g, device=centers.device)


def sample_distinct(n: int, k: int, seed: int) -> torch.Tensor:
    """k distinct integers from range(n) as int32 (CPU), seeded."""
    g = _gen("cpu", seed)
    return torch.randperm(n, generator=g)[:k].to(torch.int32)


def plan_blocks(n_tokens: int, block_w: int, block_alpha: int, n_fine: int, n_coarse: int):
    """Token ranges and cluster counts per clustering block (only integer bookkeeping, used to
    shape the seed lists): blocks of block_w tokens, the last one holding the remainder of
    block_alpha .. block_w+block_alpha-1 tokens; totals split by cumulative integer division."""
    if block_w <= 0 or n_tokens < block_w + block_alpha:
        bounds = [0, n_tokens]
    else:
        m = (n_tokens - block_alpha) // block_w
        bounds = [i * block_w for i in range(m + 1)] + [n_tokens]
    out = []
    for b in range(len(bounds) - 1):
        t0, t1 = bounds[b], bounds[b + 1]
        out.append(dict(t0=t0, t1=t1, f0=(n_fine * t0) // n_tokens, f1=(n_fine * t1) // n_tokens,
                        c0=(n_coarse * t0) // n_tokens, c1=(n_coarse * t1) // n_tokens))
    return out


def draw_seeds(units: int, blocks, levels: int, seed: int):
    """k-means seeds for every unit: init_fine int32 [units, n_fine] (block-local token indices,
    block after block) and init_coarse int32 [units, n_coarse] (block-local fine-cluster indices)."""
    n_fine = blocks[-1]["f1"]
    n_coarse = blocks[-1]["c1"] if levels == 2 else 0
    fine = torch.zeros(units, n_fine, dtype=torch.int32)
    coarse = torch.zeros(units, max(n_coarse, 1), dtype=torch.int32)
    for u in range(units):
        for bi, b in enumerate(blocks):
            kf = b["f1"] - b["f0"]
            fine[u, b["f0"]:b["f1"]] = sample_distinct(b["t1"] - b["t0"], kf, seed + 1000003 * u + 2 * bi)
            if levels == 2:
                kc = b["c1"] - b["c0"]
                coarse[u, b["c0"]:b["c1"]] = sample_distinct(kf, kc, seed + 1000003 * u + 2 * bi + 1)
    return fine, coarse[:, :n_coarse]


def make_workload(w: Workload, device, seed: int, n_query_sets: int = 1, softness: float = 1.0):
    """All tensors of a workload: dict with K, V [B,Hkv,N,128], q [sets,B,Hq,128], centers, seeds."""
    centers = make_modes(w.units, w.modes, device, seed)
    K, V = draw_tokens(centers, w.context, seed + 1)
    q = draw_queries(centers, w.group, n_query_sets, seed + 2, softness=softness)
    blocks = plan_blocks(w.context, w.block_w, w.block_alpha, w.n_fine, w.n_coarse)
    init_fine, init_coarse = draw_seeds(w.units, blocks, w.levels, seed + 3)
    return dict(
        K=K.view(w.batch, w.n_kv_heads, w.context, HEAD_DIM),
        V=V.view(w.batch, w.n_kv_heads, w.context, HEAD_DIM),
        q=q.view(n_query_sets, w.batch, w.n_q_heads, HEAD_DIM),
        centers=centers, blocks=blocks, init_fine=init_fine, init_coarse=init_coarse)
