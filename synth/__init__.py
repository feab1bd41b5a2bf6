"""Seeded synthetic IVF workloads (inputs only; none of the search arithmetic).

The paper measures on question-answering query sets over a Wikipedia passage
corpus embedded with a sentence-embedding model (Section 6.1); none of that is
available here.  These generators produce stand-ins with the same shape: unit
(or near-unit) high-dimensional embeddings clustered around centroids, an IVF
partition with skewed list sizes, skewed cluster popularity (Section 3.3), and
multi-hop query sequences that drift a little per round (Section 3.2).

Recipe, per config:
  centroids  ~ N(0, I), normalised to unit length;
  a database vector of list l = centroid_l + N(0, (noise^2/d) I), then
  normalised (unless ``normalize`` is False), then rounded to the storage dtype;
  list sizes: ``uniform`` (N/nlist each) or ``zipf``: deterministic rank weights
  r^-s, floor(N*w_r/sum w) with the remainder handed out by largest fractional
  part, at least one vector per list; rank r is mapped to a list id by a seeded
  permutation so that large lists are scattered in memory;
  labels (list_ids) are a seeded permutation of 0..N-1, so a label never equals
  its row number by construction;
  queries are generated like database vectors from a chosen cluster: chosen
  uniformly, by the same Zipf ranks as the sizes (popular clusters are the large
  ones), or with probability proportional to list size.

Everything is generated with ``torch`` on the requested device from one
``torch.Generator`` per purpose; both the HIP path and the oracle receive the
same bytes (the oracle gets a host copy).
"""
from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 20250709


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    d: int
    nlist: int
    size_dist: str          # "uniform" | "zipf"
    size_s: float
    normalize: bool
    dtype: str              # "f32" | "f16" | "bf16"  (storage of list_vectors)
    metric: str             # "ip" | "l2"
    nq: int
    query_dist: str         # "uniform" | "zipf" | "size"
    query_s: float
    nprobe: int
    k: int
    rounds: int = 1
    noise: float = 0.3
    drift: float = 0.05
    seed: int = BASE_SEED
    index_of: str = ""      # reuse the index of another config (same bytes)


CONFIGS = {
    "C1": Config("C1", 65536, 768, 256, "zipf", 1.0, True, "f32", "ip", 64, "uniform", 0.0,
                 16, 10, seed=BASE_SEED + 1),
    "C2": Config("C2", 1048576, 768, 1024, "uniform", 0.0, True, "f32", "ip", 1024, "uniform",
                 0.0, 32, 10, seed=BASE_SEED + 2),
    "C3": Config("C3", 4194304, 768, 4096, "zipf", 1.1, True, "f16", "ip", 4096, "zipf", 1.1,
                 64, 10, seed=BASE_SEED + 3),
    "C4": Config("C4", 4194304, 768, 4096, "zipf", 1.1, True, "f16", "ip", 512, "uniform", 0.0,
                 32, 10, rounds=8, seed=BASE_SEED + 3, index_of="C3"),
    "C5": Config("C5", 16777216, 768, 16384, "zipf", 1.05, False, "bf16", "l2", 8192, "size",
                 0.0, 128, 100, seed=BASE_SEED + 5),
    # the paper's own shape (Section 6.1): ~38 M passages, 1024-dimensional embeddings, IVF4096,
    # nprobe 128..512, top-1, requests arriving in small batches.  77 GB of binary16 rows.
    "P1": Config("P1", 37748736, 1024, 4096, "zipf", 0.5, True, "f16", "ip", 256, "size", 0.0,
                 128, 1, seed=BASE_SEED + 6),
}

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def scaled(cfg, **kw):
    """A smaller (or otherwise altered) copy of a config, for tests."""
    return replace(cfg, **kw)


def list_sizes(cfg):
    """Sizes by popularity rank (rank 0 = largest), int64 numpy, sums to N."""
    if cfg.size_dist == "uniform":
        base = cfg.N // cfg.nlist
        sizes = np.full(cfg.nlist, base, np.int64)
        sizes[: cfg.N - base * cfg.nlist] += 1
        return sizes
    r = np.arange(1, cfg.nlist + 1, dtype=np.float64)
    w = r ** (-cfg.size_s)
    w /= w.sum()
    if cfg.N < cfg.nlist:
        raise ValueError("N < nlist")
    exact = w * cfg.N
    sizes = np.floor(exact).astype(np.int64)
    rem = int(cfg.N - sizes.sum())
    order = np.argsort(-(exact - sizes), kind="stable")
    sizes[order[:rem]] += 1
    short = sizes < 1                   # at least one vector per list, taken from the largest
    sizes[0] -= int(short.sum())
    sizes[short] = 1
    return sizes


@dataclass
class Index:
    cfg: Config
    centroids: torch.Tensor      # [nlist, d] float32
    list_offsets: torch.Tensor   # [nlist+1] int64, host
    list_vectors: torch.Tensor   # [N, d] storage dtype
    list_ids: torch.Tensor       # [N] int64
    rank_to_list: torch.Tensor   # [nlist] int64, host: popularity rank -> list id


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _unit(x):
    return x / x.norm(dim=1, keepdim=True)


def make_index(cfg, device="cpu", chunk_rows=None):
    device = torch.device(device)
    g = _gen(device, cfg.seed)
    gh = _gen("cpu", cfg.seed + 1000)
    cent = _unit(torch.randn(cfg.nlist, cfg.d, generator=g, device=device, dtype=torch.float32))
    rank_to_list = torch.randperm(cfg.nlist, generator=gh)
    sizes_by_rank = torch.from_numpy(list_sizes(cfg))
    sizes = torch.empty(cfg.nlist, dtype=torch.int64)
    sizes[rank_to_list] = sizes_by_rank
    offsets = torch.zeros(cfg.nlist + 1, dtype=torch.int64)
    offsets[1:] = torch.cumsum(sizes, 0)
    row_list = torch.repeat_interleave(torch.arange(cfg.nlist), sizes).to(device)
    vecs = torch.empty(cfg.N, cfg.d, dtype=TORCH_DTYPE[cfg.dtype], device=device)
    if chunk_rows is None:
        chunk_rows = 1 << 19 if device.type == "cuda" else 1 << 15
    sigma = cfg.noise / cfg.d ** 0.5
    for r0 in range(0, cfg.N, chunk_rows):
        r1 = min(cfg.N, r0 + chunk_rows)
        x = torch.randn(r1 - r0, cfg.d, generator=g, device=device, dtype=torch.float32)
        x.mul_(sigma).add_(cent[row_list[r0:r1]])
        if cfg.normalize:
            x = _unit(x)
        vecs[r0:r1] = x.to(vecs.dtype)
    ids = torch.randperm(cfg.N, generator=gh).to(device)
    return Index(cfg, cent, offsets, vecs, ids, rank_to_list)


def _pick_clusters(cfg, index, n, gh):
    if cfg.query_dist == "uniform":
        return torch.randint(0, cfg.nlist, (n,), generator=gh)
    if cfg.query_dist == "zipf":
        w = torch.arange(1, cfg.nlist + 1, dtype=torch.float64) ** (-cfg.query_s)
        ranks = torch.multinomial(w, n, replacement=True, generator=gh)
        return index.rank_to_list[ranks]
    if cfg.query_dist == "size":
        sizes = (index.list_offsets[1:] - index.list_offsets[:-1]).to(torch.float64)
        return torch.multinomial(sizes, n, replacement=True, generator=gh)
    raise ValueError(cfg.query_dist)


def make_queries(cfg, index, device=None):
    """List of ``cfg.rounds`` tensors [nq, d] float32 on ``device``."""
    device = index.centroids.device if device is None else torch.device(device)
    g = _gen(device, cfg.seed + 2000 + (17 if cfg.index_of else 0))
    gh = _gen("cpu", cfg.seed + 3000 + (17 if cfg.index_of else 0))
    cl = _pick_clusters(cfg, index, cfg.nq, gh).to(device)
    sigma = cfg.noise / cfg.d ** 0.5
    q = torch.randn(cfg.nq, cfg.d, generator=g, device=device, dtype=torch.float32)
    q.mul_(sigma).add_(index.centroids.to(device)[cl])
    if cfg.normalize:
        q = _unit(q)
    out = [q]
    dsig = cfg.drift / cfg.d ** 0.5
    for _ in range(1, cfg.rounds):
        step = torch.randn(cfg.nq, cfg.d, generator=g, device=device, dtype=torch.float32)
        q = q + step * dsig
        if cfg.normalize:
            q = _unit(q)
        out.append(q)
    return out


def to_numpy(t):
    """Host numpy view of a tensor; bfloat16 becomes its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
