"""The five synthetic workloads and the recipe that builds them.

Graph: R-MAT CSR (rows = in-neighbours).  Features: fp32 N(0,1).  Train set: the first
``train_frac * N`` nodes of a hashed ordering.  Batches: each epoch is a hashed shuffle of
the train set cut into consecutive batches of ``batch`` seeds (the last batch of an epoch is
short); a superbatch of ``S`` batches runs on into the next epoch when the epoch ends.
"""
from __future__ import annotations

import sys
from dataclasses import dataclass, field

import torch

from .rmat import mix64, mix64_int, rmat_csr


@dataclass
class Config:
    name: str
    num_nodes: int
    num_edges: int          # directed R-MAT edges drawn (doubled when symmetrised)
    abc: tuple
    feat_dim: int
    train_frac: float
    batch: int
    fanout: tuple
    S: int
    cap: int
    symmetrise: bool = False
    offsets_64: bool = False
    seed: int = 0


CONFIGS = [
    Config("c1-tiny-rmat14", 1 << 14, 262_144, (0.57, 0.19, 0.19), 64, 0.10, 256,
           (10, 10, 10), 8, 2048),
    Config("c2-rmat20", 1 << 20, 16 << 20, (0.57, 0.19, 0.19), 128, 0.10, 1000,
           (10, 10, 10), 20, (1 << 20) // 10),
    Config("c3-rmat24", 1 << 24, 16 << 24, (0.57, 0.19, 0.19), 128, 0.05, 1000,
           (10, 10, 10), 100, (1 << 24) // 5, offsets_64=True),
    Config("c4-papers-shape", 111_000_000, 1_600_000_000, (0.57, 0.19, 0.19), 128, 0.011,
           1000, (10, 10, 10), 200, 111_000_000 // 4, offsets_64=True),
    Config("c5-friendster-shape", 65_600_000, 1_800_000_000, (0.45, 0.22, 0.22), 256, 0.01,
           1000, (10, 10, 10), 200, 65_600_000 // 5, symmetrise=True, offsets_64=True),
]


@dataclass
class Workload:
    cfg: Config
    offsets: torch.Tensor           # [N+1] int32/int64, on the build device
    indices: torch.Tensor           # [E] int32
    seeds: torch.Tensor             # flat int32 (CPU)
    seed_offsets: torch.Tensor      # [S+1] int64 (CPU)
    features: torch.Tensor | None = None   # [N, F] fp32 on the host (pinned if possible)
    extra: dict = field(default_factory=dict)


def train_nodes(num_nodes: int, frac: float, seed: int, device="cpu") -> torch.Tensor:
    v = torch.arange(num_nodes, dtype=torch.int64, device=device)
    order = torch.argsort(mix64(v ^ (mix64_int(seed ^ 0x7A11) >> 1)))
    return order[: int(num_nodes * frac)].to(torch.int32)


def seed_batches(train: torch.Tensor, batch: int, S: int, seed: int, first_batch: int = 0):
    """Batches ``first_batch .. first_batch+S-1`` of the endless epoch sequence.
    Returns (flat seeds int32, seed_offsets int64[S+1]) on the CPU."""
    n = train.numel()
    per_epoch = (n + batch - 1) // batch
    t64 = train.to(torch.int64)
    out, offs, cache = [], [0], {}
    for g in range(first_batch, first_batch + S):
        epoch, j = divmod(g, per_epoch)
        if epoch not in cache:
            key = mix64_int(seed ^ (0xE90C << 20) ^ epoch) >> 1
            cache[epoch] = train[torch.argsort(mix64(t64 ^ key))]
        b = cache[epoch][j * batch: min((j + 1) * batch, n)]
        out.append(b)
        offs.append(offs[-1] + b.numel())
    return torch.cat(out).to(torch.int32).cpu(), torch.tensor(offs, dtype=torch.int64)


def make_features(num_nodes: int, feat_dim: int, seed: int, device="cpu",
                  pin: bool | None = None, chunk_rows: int = 1 << 22) -> torch.Tensor:
    """fp32 N(0,1) table on the host; generated on ``device`` in chunks."""
    if pin is None:
        pin = torch.cuda.is_available()
    out = torch.empty((num_nodes, feat_dim), dtype=torch.float32, pin_memory=pin)
    g = torch.Generator(device=device)
    g.manual_seed(mix64_int(seed ^ 0xFEA7) >> 1)
    for lo in range(0, num_nodes, chunk_rows):
        hi = min(lo + chunk_rows, num_nodes)
        out[lo:hi].copy_(torch.randn((hi - lo, feat_dim), generator=g, device=device,
                                     dtype=torch.float32))
    return out


def make_workload(index: int, device="cpu", features: bool = True, S: int | None = None,
                  first_batch: int = 0, verbose: bool = False) -> Workload:
    """Build workload ``index`` (1-based, as the configs are numbered)."""
    cfg = CONFIGS[index - 1]
    offsets, indices = rmat_csr(cfg.num_nodes, cfg.num_edges, cfg.abc, cfg.seed, device,
                                symmetrise=cfg.symmetrise, offsets_64=cfg.offsets_64,
                                verbose=verbose)
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed, device)
    seeds, seed_offsets = seed_batches(train, cfg.batch, S or cfg.S, cfg.seed, first_batch)
    if verbose:
        print("[workload] graph and seeds ready; filling the feature table", file=sys.stderr,
              flush=True)
    feats = make_features(cfg.num_nodes, cfg.feat_dim, cfg.seed, device) if features else None
    return Workload(cfg, offsets, indices, seeds, seed_offsets, feats)
