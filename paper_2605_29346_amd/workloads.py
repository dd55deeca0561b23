"""Seeded synthetic inputs for the mini-batch construction path.

Everything here produces *inputs* (graphs, feature tables, seed batches); none of
the method's arithmetic (sampling RNG, relabeling, aggregation) lives here, so the
CPU checker and the HIP path may both be fed from this module.

The generators are written with torch integer tensor ops only, so the same call
gives bit-identical results on the CPU and on a GPU: the random source is a small
counter-based 32-bit mixer evaluated in int64 containers (every product stays
below 2**63, so there is no reliance on wrap-around), and floating point is
limited to exactly representable integers, one double multiply and one
double->float rounding.

Shapes follow the datasets of the paper's Table 1 (Reddit, OGBN-Products,
OGBN-papers100M) as restated by the five benchmark configurations; the datasets
themselves are not available, these graphs stand in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import torch

_M32 = 0xFFFFFFFF
# odd 31-bit multipliers (arbitrary; products of a 32-bit value with them fit in 63 bits)
_K1, _K2, _K3 = 0x6A5D39EB, 0x2F1B8C27, 0x4E7C9A53
_KB = 0x3C6EF373  # stride applied to the second hash argument


def _mix32_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * _K1) & _M32
    x ^= x >> 13
    x = (x * _K2) & _M32
    x ^= x >> 17
    x = (x * _K3) & _M32
    x ^= x >> 15
    return x


def mix32(x: torch.Tensor) -> torch.Tensor:
    """Avalanche a tensor of values in [0, 2**32) held in int64."""
    x = x ^ (x >> 16)
    x = (x * _K1) & _M32
    x = x ^ (x >> 13)
    x = (x * _K2) & _M32
    x = x ^ (x >> 17)
    x = (x * _K3) & _M32
    x = x ^ (x >> 15)
    return x


def _seed_words(seed: int) -> Tuple[int, int]:
    s0 = _mix32_int(seed ^ 0x5EED0001)
    s1 = _mix32_int((seed >> 32) ^ s0 ^ 0x0BADC0DE)
    return s0, s1


def hash32(seed: int, a: torch.Tensor, b) -> torch.Tensor:
    """32 uniform bits per element from (seed, a, b); a < 2**32, 0 <= b < 2**30."""
    s0, s1 = _seed_words(seed)
    h = mix32((a ^ s0) & _M32)
    return mix32((h + b * _KB + s1) & _M32)


# --------------------------------------------------------------------------------------
# graphs
# --------------------------------------------------------------------------------------
@dataclass
class Graph:
    num_nodes: int
    offsets: torch.Tensor  # int32 or int64 [num_nodes+1]
    indices: torch.Tensor  # int32 [num_edges], each row ascending and duplicate-free
    hubs: Optional[torch.Tensor] = None  # int64 ids of designated hubs (stress graph)

    @property
    def num_edges(self) -> int:
        return int(self.indices.numel())


def _permutation(n: int, seed: int, device) -> torch.Tensor:
    """Seeded permutation of [0, n): new_id[old_id]."""
    i = torch.arange(n, dtype=torch.int64, device=device)
    key = (hash32(seed, i, 0) << 31) | i  # unique keys -> order independent of sort stability
    order = torch.argsort(key)
    del key
    perm = torch.empty_like(order)
    perm[order] = i
    return perm


def _csr_from_keys(keys: torch.Tensor, num_nodes: int, offsets_dtype) -> Tuple[torch.Tensor, torch.Tensor]:
    """keys = src*num_nodes+dst (any order, duplicates allowed) -> sorted duplicate-free CSR."""
    keys = torch.unique(keys, sorted=True)
    src = torch.div(keys, num_nodes, rounding_mode="floor")
    dst = (keys - src * num_nodes).to(torch.int32)
    del keys
    counts = torch.bincount(src, minlength=num_nodes)
    del src
    offsets = torch.zeros(num_nodes + 1, dtype=torch.int64, device=dst.device)
    torch.cumsum(counts, 0, out=offsets[1:])
    return offsets.to(offsets_dtype), dst


def _rmat_edges(num_nodes: int, first: int, count: int, seed: int, abcd, device) -> torch.Tensor:
    """R-MAT draws number first..first+count-1 -> keys src*num_nodes+dst of the draws whose
    endpoints both fall below num_nodes (the rest are rejected)."""
    a, b, c, _ = abcd
    scale = max(1, (num_nodes - 1).bit_length())
    A = int(a * 2**32)
    AB = int((a + b) * 2**32)
    ABC = int((a + b + c) * 2**32)
    s0, s1 = _seed_words(seed)
    e = torch.arange(first, first + count, dtype=torch.int64, device=device)
    h0 = mix32((e ^ s0) & _M32)
    del e
    src = torch.zeros(count, dtype=torch.int64, device=device)
    dst = torch.zeros(count, dtype=torch.int64, device=device)
    for level in range(scale):
        h = mix32((h0 + level * _KB + s1) & _M32)
        sbit = (h >= AB).to(torch.int64)
        dbit = (((h >= A) & (h < AB)) | (h >= ABC)).to(torch.int64)
        src = src * 2 + sbit
        dst = dst * 2 + dbit
    ok = (src < num_nodes) & (dst < num_nodes)
    return src[ok], dst[ok]


def rmat_graph(num_nodes: int, num_draws: int, seed: int, *, abcd=(0.57, 0.19, 0.19, 0.05),
               offsets_dtype=torch.int64, device="cpu", exact_edges: Optional[int] = None,
               chunk: int = 1 << 26) -> Graph:
    """Directed R-MAT graph on `num_nodes` vertices from `num_draws` edge draws.

    Vertex ids go through a seeded permutation so hubs are not the low ids; rows are sorted
    ascending and de-duplicated; self-loops and zero-degree vertices are kept.  With
    `exact_edges`, draws continue until that many distinct edges exist and exactly the first
    `exact_edges` distinct ones (in draw order) are kept.
    """
    perm = _permutation(num_nodes, seed ^ 0x9E3779B9, device)
    parts: List[torch.Tensor] = []
    first = 0
    if exact_edges is None:
        while first < num_draws:
            cnt = min(chunk, num_draws - first)
            s, d = _rmat_edges(num_nodes, first, cnt, seed, abcd, device)
            parts.append(perm[s] * num_nodes + perm[d])
            first += cnt
        keys = torch.cat(parts) if len(parts) > 1 else parts[0]
        del parts
    else:
        keys = torch.empty(0, dtype=torch.int64, device=device)
        while True:
            cnt = max(1024, int(exact_edges * 1.5))
            s, d = _rmat_edges(num_nodes, first, cnt, seed, abcd, device)
            keys = torch.cat([keys, perm[s] * num_nodes + perm[d]])
            first += cnt
            uniq, inv = torch.unique(keys, sorted=True, return_inverse=True)
            if uniq.numel() >= exact_edges:
                pos = torch.arange(keys.numel(), dtype=torch.int64, device=device)
                first_pos = torch.full((uniq.numel(),), keys.numel(), dtype=torch.int64, device=device)
                first_pos.scatter_reduce_(0, inv, pos, reduce="amin")
                keep = torch.argsort(first_pos)[:exact_edges]
                keys = uniq[keep]
                break
    offsets, indices = _csr_from_keys(keys, num_nodes, offsets_dtype)
    return Graph(num_nodes, offsets, indices)


def chung_lu_graph(num_nodes: int, num_edges: int, seed: int, *, gamma: float = 2.1, i0: float = 10.0,
                   num_hubs: int = 100, hub_degree=(100_000, 200_000), offsets_dtype=torch.int64,
                   device="cpu") -> Graph:
    """Symmetric Chung-Lu power-law graph (expected degree of vertex i proportional to
    (i+i0)**(-1/(gamma-1))) with `num_hubs` designated hubs, each wired to a uniform random
    set of about hub_degree[0]..hub_degree[1] distinct vertices.  `num_edges` is the total
    directed edge budget (both directions, hubs included)."""
    dev = device
    perm = _permutation(num_nodes, seed ^ 0x51ED270B, dev)
    keys: List[torch.Tensor] = []
    hub_old = torch.arange(num_nodes - num_hubs, num_nodes, dtype=torch.int64, device=dev)
    lo, hi = hub_degree
    lo, hi = min(lo, num_nodes // 2), min(hi, num_nodes // 2)
    used = 0
    for k in range(num_hubs):
        target = lo + (_mix32_int(seed * 1000003 + k) % max(1, hi - lo + 1))
        draws = int(-num_nodes * math.log1p(-target / num_nodes)) + 1
        j = torch.arange(draws, dtype=torch.int64, device=dev)
        h = hash32(seed ^ 0x48554253, j, k)
        nb = (h * num_nodes) >> 32  # uniform in [0, num_nodes)
        hub = int(hub_old[k])
        keys.append(perm[torch.full_like(nb, hub)] * num_nodes + perm[nb])
        keys.append(perm[nb] * num_nodes + perm[torch.full_like(nb, hub)])
        used += 2 * draws
    pairs = max(0, (num_edges - used) // 2)
    w = (torch.arange(num_nodes, dtype=torch.float64, device="cpu") + i0) ** (-1.0 / (gamma - 1.0))
    cdf = torch.cumsum(w, 0)
    cdf = (cdf / cdf[-1]).to(dev)  # built on the CPU so the table is the same for any device
    done = 0
    chunk = 1 << 24
    while done < pairs:
        cnt = min(chunk, pairs - done)
        e = torch.arange(done, done + cnt, dtype=torch.int64, device=dev)
        ends = []
        for side in (1, 2):
            hi32 = hash32(seed ^ 0x434C5500, e, side)
            lo32 = hash32(seed ^ 0x434C55FF, e, side)
            u = (hi32.to(torch.float64) + lo32.to(torch.float64) * 2.0**-32) * 2.0**-32
            ends.append(torch.searchsorted(cdf, u).clamp_(max=num_nodes - 1))
        s, d = perm[ends[0]], perm[ends[1]]
        keys.append(s * num_nodes + d)
        keys.append(d * num_nodes + s)
        done += cnt
    allk = torch.cat(keys)
    del keys
    offsets, indices = _csr_from_keys(allk, num_nodes, offsets_dtype)
    return Graph(num_nodes, offsets, indices, hubs=perm[hub_old].clone())


# --------------------------------------------------------------------------------------
# features
# --------------------------------------------------------------------------------------
_FEAT_SCALE = 1.0 / math.sqrt((65536.0**2 - 1.0) / 3.0)


def feature_rows(ids: torch.Tensor, dim: int, seed: int) -> torch.Tensor:
    """fp32 feature rows of the given vertex ids: feat(v, j) is a pure function of
    (seed, v, j): the sum of four uniform 16-bit integers, centred and scaled to unit
    variance (bell-shaped on about +-3.46), so any row can be regenerated anywhere."""
    ids = ids.to(torch.int64)
    j = torch.arange(dim, dtype=torch.int64, device=ids.device)
    v = ids[:, None].expand(-1, dim)
    h1 = hash32(seed ^ 0x46454131, v, j[None, :])
    h2 = hash32(seed ^ 0x46454132, v, j[None, :])
    s = (h1 & 0xFFFF) + (h1 >> 16) + (h2 & 0xFFFF) + (h2 >> 16)
    x = (s - 131070).to(torch.float64) * _FEAT_SCALE
    return x.to(torch.float32)


def feature_table(num_nodes: int, dim: int, seed: int, device="cpu", row_chunk: Optional[int] = None,
                  ld: Optional[int] = None) -> torch.Tensor:
    """Full [num_nodes, dim] fp32 table (row stride `ld` >= dim elements), built in row chunks."""
    ld = dim if ld is None else ld
    if row_chunk is None:
        row_chunk = max(1, (1 << 25) // max(dim, 1))
    out = torch.empty((num_nodes, ld), dtype=torch.float32, device=device)
    if ld != dim:
        out.zero_()
    for r0 in range(0, num_nodes, row_chunk):
        r1 = min(num_nodes, r0 + row_chunk)
        ids = torch.arange(r0, r1, dtype=torch.int64, device=device)
        out[r0:r1, :dim] = feature_rows(ids, dim, seed)
    return out


# --------------------------------------------------------------------------------------
# seed batches
# --------------------------------------------------------------------------------------
class SeedPool:
    """Distinct seed vertices per step: a seeded shuffle of a vertex pool, step s takes
    slice s (wrapping).  With hubs, each hub enters a batch independently with
    probability hub_prob and the rest of the batch comes from the non-hub pool."""

    def __init__(self, graph: Graph, batch: int, seed: int, pool_size: Optional[int] = None,
                 hub_prob: float = 0.0):
        n = graph.num_nodes
        dev = graph.indices.device
        self.batch = batch
        self.seed = seed
        self.hub_prob = hub_prob
        order = torch.argsort((hash32(seed ^ 0x5EED5EED, torch.arange(n, dtype=torch.int64, device=dev), 1) << 31)
                              | torch.arange(n, dtype=torch.int64, device=dev))
        self.hubs = None
        if graph.hubs is not None and hub_prob > 0:
            is_hub = torch.zeros(n, dtype=torch.bool, device=dev)
            is_hub[graph.hubs] = True
            order = order[~is_hub[order]]
            self.hubs = graph.hubs.to(dev)
        if pool_size is not None:
            order = order[:pool_size]
        assert order.numel() >= batch, "seed pool smaller than the batch"
        self.pool = order.to(torch.int32)

    def batch_for(self, step: int) -> torch.Tensor:
        """int32 [batch] distinct vertex ids for this step (on the graph's device)."""
        slots = self.pool.numel() // self.batch
        s = step % slots
        plain = self.pool[s * self.batch:(s + 1) * self.batch]
        if self.hubs is None:
            return plain.clone()
        k = torch.arange(self.hubs.numel(), dtype=torch.int64, device=self.hubs.device)
        pick = hash32(self.seed ^ 0x48500000, k, step) < int(self.hub_prob * 2**32)
        chosen = self.hubs[pick].to(torch.int32)
        return torch.cat([chosen, plain[: self.batch - chosen.numel()]])

    def seed_prob(self, num_nodes: int) -> torch.Tensor:
        """float32 [num_nodes]: the chance that a vertex is a seed of a step picked at random (the pool's
        vertices share the batch's places evenly; a hub enters with hub_prob)."""
        p = torch.zeros(num_nodes, dtype=torch.float32, device=self.pool.device)
        slots = self.pool.numel() // self.batch
        p[self.pool[: slots * self.batch].long()] = 1.0 / slots
        if self.hubs is not None:
            p[self.hubs.long()] = self.hub_prob
        return p


# --------------------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    kind: str  # "rmat" | "chung_lu"
    num_nodes: int
    num_draws: int  # R-MAT draws, or the directed edge budget of the Chung-Lu graph
    offsets_dtype: torch.dtype
    dim: int
    batch: int
    fanouts: Tuple[int, ...]
    steps: int
    exact_edges: Optional[int] = None
    pool_size: Optional[int] = None
    hub_prob: float = 0.0
    graph_seed: int = 20260529
    feat_seed: int = 346
    pool_seed: int = 77
    base_key: int = 0x2605_2934_6000_0000
    extra: Dict = field(default_factory=dict)

    def build_graph(self, device="cpu") -> Graph:
        if self.kind == "rmat":
            return rmat_graph(self.num_nodes, self.num_draws, self.graph_seed, offsets_dtype=self.offsets_dtype,
                              device=device, exact_edges=self.exact_edges)
        return chung_lu_graph(self.num_nodes, self.num_draws, self.graph_seed, offsets_dtype=self.offsets_dtype,
                              device=device, **self.extra)

    def seed_pool(self, graph: Graph) -> SeedPool:
        return SeedPool(graph, self.batch, self.pool_seed, self.pool_size, self.hub_prob)

    def key_for(self, step: int) -> int:
        return (self.base_key + step) & 0xFFFFFFFFFFFFFFFF

    def scaled(self, factor: float, **over) -> "Config":
        """A shrunken copy (vertex and edge counts times `factor`) for quick checks."""
        import dataclasses
        c = dataclasses.replace(
            self, name=f"{self.name}@{factor:g}", num_nodes=max(64, int(self.num_nodes * factor)),
            num_draws=max(256, int(self.num_draws * factor)),
            exact_edges=None if self.exact_edges is None else max(64, int(self.exact_edges * factor)),
            pool_size=None if self.pool_size is None else max(self.batch, int(self.pool_size * factor)))
        if c.kind == "chung_lu":
            ex = dict(c.extra)
            lo, hi = ex.get("hub_degree", (100_000, 200_000))
            ex["hub_degree"] = (max(4, int(lo * factor)), max(8, int(hi * factor)))
            c = dataclasses.replace(c, extra=ex)
        return dataclasses.replace(c, **over) if over else c


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", "rmat", 10_000, 150_000, torch.int32, 32, 64, (5, 5), 1, exact_edges=100_000),
    "medium_dense": Config("medium_dense", "rmat", 250_000, 150_000_000, torch.int64, 600, 1024, (25, 10), 100,
                           exact_edges=100_000_000),
    "large_sparse": Config("large_sparse", "rmat", 2_400_000, 180_000_000, torch.int64, 100, 1024, (15, 10, 5), 200,
                           exact_edges=120_000_000, pool_size=204_800),
    "very_large": Config("very_large", "rmat", 110_000_000, 1_600_000_000, torch.int64, 128, 4096, (15, 10, 5), 100),
    "envelope_stress": Config("envelope_stress", "chung_lu", 1_000_000, 50_000_000, torch.int64, 256, 4096, (25, 10),
                              500, hub_prob=0.10,
                              extra=dict(gamma=2.1, num_hubs=100, hub_degree=(100_000, 200_000))),
}
