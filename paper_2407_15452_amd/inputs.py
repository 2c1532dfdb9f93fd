"""Seeded synthetic inputs for the walk + SGNS path.

This module only *makes inputs*: graphs as edge lists, start nodes, noise
weights, initial embedding tables and the five workload descriptions.  It
contains none of the method's arithmetic (no Philox, no alias sampling, no
walk, no SGNS) and is used unchanged by the HIP path, by the CPU reference in
the tests and by the benchmark, so that both sides always see the same bytes.

Everything is a pure function of (seed, index) through a 64-bit integer mixer
written with torch integer ops, so the same tensors come out on the CPU and on
the GPU.  The mixer is the SplitMix64 finaliser (Steele, Lea, Flood 2014).

The graphs stand in for the public datasets of GraphScale §4 ("Datasets"):
the R-MAT graph of workload 2 has the shape of ogbn-products, the directed one
of workload 4 the shape of ogbn-papers100M, and the weighted bipartite graph of
workload 3 that of a user-item interaction graph.  None of the real datasets is
read anywhere.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

_MASK32 = (1 << 32) - 1


def _s64(x: int) -> int:
    """Python int -> the same 64 bits as a signed value torch can hold."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift on int64 tensors."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """SplitMix64 finaliser on an int64 tensor (arithmetic wraps modulo 2**64)."""
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def hashed_u32(seed: int, index: torch.Tensor, stream: int) -> torch.Tensor:
    """32 pseudo-random bits (as int64 in [0, 2**32)) per (seed, index, stream)."""
    base = _s64(seed * 0x2545F4914F6CDD1D + stream * 0x9E3779B97F4A7C15)
    return _lsr(mix64(mix64(index + base) ^ _s64(seed)), 32)


def hashed_unit(seed: int, index: torch.Tensor, stream: int) -> torch.Tensor:
    """fp64 uniform in (0, 1) per (seed, index, stream)."""
    return (hashed_u32(seed, index, stream).to(torch.float64) + 0.5) * (1.0 / 4294967296.0)


# ---------------------------------------------------------------------------
# Workloads
# ---------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    kind: str               # "rmat" | "bipartite"
    num_nodes: int
    num_edges: int          # undirected edges (directed edges if directed=True)
    directed: bool
    offset_bits: int
    walks_per_node: int
    walk_len: int
    window: int
    num_neg: int
    dim: int
    dtype: str              # "f32" | "bf16"
    lr: float
    lr_decay: bool
    batch_pairs: int
    node2vec: bool = False
    p: float = 1.0
    q: float = 1.0
    weighted: bool = False
    num_users: int = 0      # bipartite only
    num_items: int = 0
    graph_seed: int = 0x67530001
    init_seed: int = 0x67531000
    walk_seed: int = 0x67532000
    neg_seed: int = 0x67533000

    def scaled(self, factor: float, name: str | None = None) -> "Workload":
        """Same recipe with nodes/edges (and users/items) scaled by `factor`."""
        f = lambda v: max(1, int(round(v * factor)))  # noqa: E731
        return dataclasses.replace(
            self, name=name or f"{self.name}@{factor:g}", num_nodes=f(self.num_nodes),
            num_edges=f(self.num_edges), num_users=f(self.num_users) if self.num_users else 0,
            num_items=f(self.num_items) if self.num_items else 0)


WORKLOADS = [
    Workload("cfg0-deepwalk-10k", "rmat", 10_000, 100_000, False, 32, 4, 20, 5, 5, 64, "f32",
             0.025, True, 65_536, graph_seed=0x67530001),
    Workload("cfg1-deepwalk-1m", "rmat", 1_000_000, 10_000_000, False, 32, 10, 40, 5, 5, 128,
             "f32", 0.025, False, 1_048_576, graph_seed=0x67530002),
    Workload("cfg2-node2vec-4m", "rmat", 4_000_000, 64_000_000, False, 32, 10, 80, 10, 5, 128,
             "f32", 0.025, False, 2_000_000, node2vec=True, p=0.5, q=2.0,
             graph_seed=0x67530003),
    Workload("cfg3-bipartite-25m", "bipartite", 25_000_000, 500_000_000, False, 32, 5, 40, 5, 10,
             256, "bf16", 0.025, False, 2_000_000, weighted=True, num_users=20_000_000,
             num_items=5_000_000, graph_seed=0x67530004),
    Workload("cfg4-shard-100m", "rmat", 100_000_000, 1_600_000_000, True, 64, 2, 40, 5, 5, 128,
             "f32", 0.025, False, 4_000_000, graph_seed=0x67530005),
]


def pairs_per_full_walk(walk_len: int, window: int) -> int:
    """Number of (centre, context) pairs of a walk without dead end."""
    return sum(min(a, window) + min(walk_len - 1 - a, window) for a in range(walk_len))


# ---------------------------------------------------------------------------
# Graph generators (edge lists; CSR construction is part of the method)
# ---------------------------------------------------------------------------
RMAT_A, RMAT_B, RMAT_C = 0.57, 0.19, 0.19


def _relabel(num_nodes: int, seed: int, device) -> torch.Tensor:
    """A fixed pseudo-random permutation of the vertex ids (R-MAT puts its hubs
    at low ids; relabelling removes that accidental locality)."""
    ids = torch.arange(num_nodes, dtype=torch.int64, device=device)
    return torch.argsort(hashed_u32(seed, ids, 7) * num_nodes + ids)


def rmat_candidates(num_nodes: int, first: int, count: int, seed: int, device="cpu",
                    a: float = RMAT_A, b: float = RMAT_B, c: float = RMAT_C):
    """R-MAT candidate edges number first .. first+count-1 (before any filtering).

    One quadrant choice per bit level; level l of candidate e compares
    hashed_u32(seed, e * 64 + l) with the cumulative quadrant thresholds.
    Returns int64 (src, dst) in the 2**scale id space.
    """
    scale = max(1, math.ceil(math.log2(max(2, num_nodes))))
    e = torch.arange(first, first + count, dtype=torch.int64, device=device)
    src = torch.zeros_like(e)
    dst = torch.zeros_like(e)
    ta = int(a * 4294967296.0)
    tab = int((a + b) * 4294967296.0)
    tabc = int((a + b + c) * 4294967296.0)
    for level in range(scale):
        r = hashed_u32(seed, e * 64 + level, 1)
        src = (src << 1) | (r >= tab).to(torch.int64)
        dst = (dst << 1) | ((r >= ta) & (r < tab) | (r >= tabc)).to(torch.int64)
    return src, dst


def rmat_edge_list(wl: Workload, device="cpu", chunk: int = 1 << 24):
    """Edge list (int32 src, dst) of an R-MAT workload, vertex ids relabelled.

    Candidates with an endpoint >= num_nodes or src == dst are dropped here;
    duplicates are left in (CSR construction removes them), except for the
    smallest workload, which takes the first `num_edges` distinct undirected
    edges in candidate order so that its edge count is exact.
    """
    n = wl.num_nodes
    perm = _relabel(n, wl.graph_seed, device)
    exact = wl.num_edges <= 200_000 and not wl.directed
    want = wl.num_edges * 4 if exact else int(math.ceil(wl.num_edges * 1.15))
    srcs, dsts = [], []
    for first in range(0, want, chunk):
        cnt = min(chunk, want - first)
        s, d = rmat_candidates(n, first, cnt, wl.graph_seed, device)
        ok = (s < n) & (d < n) & (s != d)
        srcs.append(perm[s[ok]].to(torch.int32))
        dsts.append(perm[d[ok]].to(torch.int32))
    s = torch.cat(srcs)
    del srcs
    d = torch.cat(dsts)
    del dsts
    if exact:
        key = torch.minimum(s, d).long() * n + torch.maximum(s, d).long()
        uniq, inv = torch.unique(key, return_inverse=True)
        pos = torch.arange(key.numel(), dtype=torch.int64, device=key.device)
        first_pos = torch.full((uniq.numel(),), key.numel(), dtype=torch.int64, device=key.device)
        first_pos.scatter_reduce_(0, inv, pos, reduce="amin")
        keep = torch.sort(first_pos).values[:wl.num_edges]
        if keep.numel() < wl.num_edges:
            raise RuntimeError("not enough distinct R-MAT edges; raise the candidate factor")
        s, d = s[keep], d[keep]
    return s, d


def _zipf_rank(u: torch.Tensor, n: int, s: float) -> torch.Tensor:
    """Rank in [0, n) with P(rank = r) roughly proportional to (r + 1) ** -s
    (inverse of the continuous power-law CDF on [1, n + 1))."""
    one_minus = 1.0 - s
    top = (n + 1.0) ** one_minus
    x = (1.0 + u * (top - 1.0)) ** (1.0 / one_minus)
    return torch.clamp(x.floor().to(torch.int64) - 1, 0, n - 1)


def bipartite_edge_list(wl: Workload, device="cpu", chunk: int = 1 << 24, max_rounds: int = 8):
    """Weighted user-item interactions: endpoints drawn independently with
    Zipf(1.1) user ranks and Zipf(0.9) item ranks.  The product of two Zipf laws
    repeats its popular pairs heavily, so draws are made in rounds and
    de-duplicated until at least 95 % of `num_edges` distinct interactions
    exist (the realised count is what the benchmark reports).  The weight of an
    interaction is lognormal(0, 1) hashed from its (user, item) key.  Users are
    nodes [0, num_users), items [num_users, num_nodes); both id ranges are
    relabelled.  The list comes out sorted by (user, item)."""
    nu, ni = wl.num_users, wl.num_items
    pu = _relabel(nu, wl.graph_seed, device)
    pi = _relabel(ni, wl.graph_seed + 1, device)
    keys = torch.empty(0, dtype=torch.int64, device=device)
    drawn = 0
    for _ in range(max_rounds):
        if keys.numel() >= 0.95 * wl.num_edges:
            break
        todo = max(1024, int((wl.num_edges - keys.numel()) * 1.6))
        parts = [keys]
        for first in range(drawn, drawn + todo, chunk):
            cnt = min(chunk, drawn + todo - first)
            e = torch.arange(first, first + cnt, dtype=torch.int64, device=device)
            user = pu[_zipf_rank(hashed_unit(wl.graph_seed, e, 2), nu, 1.1)]
            item = pi[_zipf_rank(hashed_unit(wl.graph_seed, e, 3), ni, 0.9)]
            parts.append(torch.unique(user * ni + item))
        drawn += todo
        keys = torch.unique(torch.cat(parts))
        del parts
    user = torch.div(keys, ni, rounding_mode="floor")
    item = keys - user * ni + nu
    z = torch.sqrt(-2.0 * torch.log(hashed_unit(wl.graph_seed, keys, 4))) * \
        torch.cos(2.0 * math.pi * hashed_unit(wl.graph_seed, keys, 5))
    return user.to(torch.int32), item.to(torch.int32), torch.exp(z).to(torch.float32)


def edge_list(wl: Workload, device="cpu"):
    """(src, dst, weights-or-None) for a workload."""
    if wl.kind == "bipartite":
        return bipartite_edge_list(wl, device)
    s, d = rmat_edge_list(wl, device)
    return s, d, None


# ---------------------------------------------------------------------------
# Other inputs
# ---------------------------------------------------------------------------
def walk_starts(num_nodes: int, first_walk: int, count: int, device="cpu") -> torch.Tensor:
    """Walk i starts at node i mod num_nodes (every node, round after round)."""
    i = torch.arange(first_walk, first_walk + count, dtype=torch.int64, device=device)
    return (i % num_nodes).to(torch.int32)


def noise_weights(offsets: torch.Tensor) -> torch.Tensor:
    """degree ** 0.75 per node as fp32 (degree-0 nodes get weight 0).

    Computed once, on the host in fp64, and handed to every consumer as data:
    pow is not correctly rounded, so it must not be evaluated twice."""
    deg = (offsets[1:] - offsets[:-1]).to(torch.float64).cpu().numpy()
    w = np.where(deg > 0, np.power(deg, 0.75), 0.0).astype(np.float32)
    return torch.from_numpy(w).to(offsets.device)


def _fill_uniform(table: torch.Tensor, seed: int, half_width: float, chunk_rows: int = 1 << 20):
    """table[r, e] = (u - 0.5) * 2 * half_width, u a 24-bit hashed uniform of (seed, r, e)."""
    n, dim = table.shape
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        idx = torch.arange(r0 * dim, r1 * dim, dtype=torch.int64, device=table.device)
        bits = hashed_u32(seed, idx, 9) >> 8
        vals = (bits.to(torch.float32) * (1.0 / 16777216.0) - 0.5) * (2.0 * half_width)
        table[r0:r1] = vals.view(-1, dim).to(table.dtype)


def init_tables(num_nodes: int, dim: int, seed: int, device="cpu", dtype: str = "f32",
                context_seed: int | None = None):
    """Input table U(-0.5/dim, 0.5/dim) (24-bit uniforms; exact in fp32 for
    power-of-two dims), context table zero -- or, with `context_seed`, filled
    the same way from that seed (a lived-in table for throughput runs)."""
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    w_in = torch.empty((num_nodes, dim), dtype=tdtype, device=device)
    _fill_uniform(w_in, seed, 0.5 / dim)
    if context_seed is None:
        w_out = torch.zeros((num_nodes, dim), dtype=tdtype, device=device)
    else:
        w_out = torch.empty((num_nodes, dim), dtype=tdtype, device=device)
        _fill_uniform(w_out, context_seed, 0.5 / dim)
    return w_in, w_out


def random_tables(num_nodes: int, dim: int, seed: int, scale: float = 0.5, device="cpu"):
    """Both tables filled with U(-scale, scale): a mid-training-like state for tests."""
    out = []
    for stream in (11, 12):
        idx = torch.arange(num_nodes * dim, dtype=torch.int64, device=device)
        u = hashed_u32(seed, idx, stream).to(torch.float32) * (1.0 / 4294967296.0)
        out.append(((u - 0.5) * (2.0 * scale)).view(num_nodes, dim).contiguous())
    return out[0], out[1]


LR_REFERENCE_PAIRS = 16_384


def learning_rate(wl: Workload, batch_index: int, num_batches: int) -> float:
    """fp32 step size handed to the SGNS step for one batch.

    The step *sums* the gradients of the pairs of a batch, so the nominal rate
    of a workload is read as the rate for a batch of LR_REFERENCE_PAIRS pairs
    and scaled down in proportion for larger batches (with the nominal 0.025 a
    summed batch of 65,536 pairs on 10,000 nodes diverges within 20 batches).
    Optionally decayed linearly in the batch index with a floor of 1e-4."""
    scale = min(1.0, LR_REFERENCE_PAIRS / wl.batch_pairs)
    decay = max(1.0 - batch_index / num_batches, 1e-4) if wl.lr_decay else 1.0
    return float(np.float32(wl.lr * scale * decay))
