"""Seeded synthetic inputs shaped like the paper's workloads (Sec. 5 "Datasets").

This module holds NO arithmetic of the method (no sampler, no mean, no gradient): it only
builds CSR graphs, feature tables, seed batches and upstream gradients.  Both the HIP path
and the CPU oracle are fed from it; when a graph is generated on the GPU the very same
bytes are copied to the host for the oracle.

Every array is a pure function of (recipe parameters, seed, device type).  Randomness comes
from a counter-based 64-bit mixer evaluated with wrapping int64 tensor arithmetic, so a
chunk can be generated anywhere without carrying generator state; only the tiny unit-test
graph uses numpy's own generators.

Recipes (none reproduces a real dataset; they only take its published shape):
  * ``tiny_graph``       -- unit-scale directed graph, Zipf out-degrees clipped to [0, 200].
  * ``chung_lu_graph``   -- power-law expected-degree (Chung-Lu) directed graph; stands in for
                            the product-co-purchase, social and citation graphs.
  * ``kg_graph``         -- (head, tail) pairs with Zipf-popular endpoints stored in both
                            directions; stands in for the KG-completion graphs.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int -> the signed 64-bit value with the same bit pattern."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MIX_A = _s64(0xBF58476D1CE4E5B9)
_MIX_B = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def hash64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Counter-based 64-bit mixer (the splitmix64 finaliser) of (seed, stream, idx)."""
    base = _s64((seed * 0xD1342543DE82EF95 + stream * 0xA0761D6478BD642F + 0x1234567) & _MASK64)
    z = idx.to(torch.int64) * _GOLDEN + base
    z = (z ^ _lsr(z, 30)) * _MIX_A
    z = (z ^ _lsr(z, 27)) * _MIX_B
    return z ^ _lsr(z, 31)


def hash_u01(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Uniform float64 in [0, 1) from the top 53 bits of ``hash64``."""
    return _lsr(hash64(seed, stream, idx), 11).to(torch.float64) * (2.0 ** -53)


# ----------------------------------------------------------------------------------------
# graphs
# ----------------------------------------------------------------------------------------

@dataclass
class Graph:
    indptr: torch.Tensor    # [N+1] int32 or int64
    indices: torch.Tensor   # [E]   int32
    num_nodes: int

    @property
    def num_edges(self) -> int:
        return int(self.indices.shape[0])

    def degrees(self) -> torch.Tensor:
        return (self.indptr[1:] - self.indptr[:-1]).to(torch.int64)


def tiny_graph(num_nodes: int = 10_000, zipf_a: float = 2.0, max_deg: int = 200,
               seed: int = 0) -> Graph:
    """Unit-scale graph: out-degree min(max_deg, Z-1) with Z ~ Zipf(zipf_a), so that empty
    rows, rows shorter than, equal to and far longer than the fanout all occur; neighbors
    uniform over the other nodes."""
    rng = np.random.default_rng(seed)
    deg = np.minimum(max_deg, rng.zipf(zipf_a, size=num_nodes) - 1).astype(np.int64)
    # make sure the boundary cases around a fanout of 10 exist whatever the draw
    deg[:6] = np.array([0, 1, 9, 10, 11, max_deg])
    indptr = np.zeros(num_nodes + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    E = int(indptr[-1])
    src = np.repeat(np.arange(num_nodes, dtype=np.int64), deg)
    off = rng.integers(1, num_nodes, size=E, dtype=np.int64)   # 1..N-1: never a self-loop
    dst = (src + off) % num_nodes
    return Graph(torch.from_numpy(indptr.astype(np.int32)), torch.from_numpy(dst.astype(np.int32)),
                 num_nodes)


def _affine_bijection(n: int) -> Tuple[int, int, int]:
    """(a, b, a^-1 mod n) with gcd(a, n) = 1: a fixed relabelling that scatters hubs."""
    a = max(1, int(n * 0.6180339887) | 1)
    while math.gcd(a, n) != 1:
        a += 2
    b = int(n * 0.2360679775)
    return a % n if n > 1 else 0, b % n, pow(a, -1, n) if n > 1 else 0


def solve_power_law(num_nodes: int, mean_deg: float, max_deg: float, alpha: float) -> Tuple[float, float]:
    """(c, i0) of the weight sequence w_i = c (i + i0)^-alpha, i = 0..N-1, whose largest
    weight is max_deg and whose mean is mean_deg (integral approximation of the sum)."""
    def mean_for(i0: float) -> float:
        c = max_deg * i0 ** alpha
        return c / num_nodes * ((num_nodes + i0) ** (1 - alpha) - i0 ** (1 - alpha)) / (1 - alpha)
    lo, hi = 1e-6, float(num_nodes) * 10
    for _ in range(200):          # mean_for is increasing in i0
        mid = math.sqrt(lo * hi)
        if mean_for(mid) < mean_deg:
            lo = mid
        else:
            hi = mid
    i0 = math.sqrt(lo * hi)
    return max_deg * i0 ** alpha, i0


def chung_lu_graph(num_nodes: int, mean_deg: float, max_deg: float, *, alpha: float = 0.8,
                   seed: int = 0, zero_frac: float = 0.01, device: str = "cpu",
                   wide_indptr: bool = False, edge_chunk: int = 1 << 26) -> Graph:
    """Directed Chung-Lu graph with power-law expected degrees.

    Node v has rank (a v + b) mod N and weight w = c (rank + i0)^-alpha; its out-degree is
    floor(w + u) with u hashed from v (stochastic rounding), or 0 for a hashed ``zero_frac``
    of the nodes; every target is drawn with probability proportional to the weights by
    inverting the continuous CDF; a self-loop moves to the next node.  Neighbor order inside
    a row is the generation order (unsorted); repeated targets are kept (multigraph)."""
    dev = torch.device(device)
    N = num_nodes
    c, i0 = solve_power_law(N, mean_deg / max(1e-9, 1.0 - zero_frac), max_deg, alpha)
    a, b, a_inv = _affine_bijection(N)
    v = torch.arange(N, dtype=torch.int64, device=dev)
    rank = (v * a + b) % N
    w = c * (rank.to(torch.float64) + i0) ** (-alpha)
    deg = torch.floor(w + hash_u01(seed, 0, v)).to(torch.int64)
    if zero_frac > 0:
        deg = torch.where(hash_u01(seed, 1, v) < zero_frac, torch.zeros_like(deg), deg)
    del rank, w
    indptr = torch.zeros(N + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=indptr[1:])
    E = int(indptr[-1].item())
    if not wide_indptr and E >= 2 ** 31:
        raise ValueError("graph needs a 64-bit indptr")
    indices = torch.empty(E, dtype=torch.int32, device=dev)
    lo_p = i0 ** (1 - alpha)
    hi_p = (N + i0) ** (1 - alpha)
    inv_exp = 1.0 / (1 - alpha)
    # chunk by whole rows so that repeat_interleave can name each edge's source
    row0 = 0
    while row0 < N:
        e0 = int(indptr[row0].item())
        row1 = int(torch.searchsorted(indptr, torch.tensor([e0 + edge_chunk], device=dev),
                                      right=True).item()) - 1
        row1 = min(N, max(row0 + 1, row1))
        e1 = int(indptr[row1].item())
        if e1 > e0:
            src = torch.repeat_interleave(torch.arange(row0, row1, dtype=torch.int64, device=dev),
                                          deg[row0:row1])
            e = torch.arange(e0, e1, dtype=torch.int64, device=dev)
            u = hash_u01(seed, 2, e)
            j = torch.floor((u * (hi_p - lo_p) + lo_p) ** inv_exp - i0).to(torch.int64)
            j = j.clamp_(0, N - 1)
            dst = (((j - b) % N) * a_inv) % N
            dst = torch.where(dst == src, (dst + 1) % N, dst)
            indices[e0:e1] = dst.to(torch.int32)
            del src, e, u, j, dst
        row0 = row1
    return Graph(indptr if wide_indptr else indptr.to(torch.int32), indices, N)


def kg_graph(num_entities: int, num_triples: int, *, zipf_a: float = 1.1, num_relations: int = 535,
             seed: int = 0, device: str = "cpu") -> Graph:
    """(head, tail) pairs whose endpoints follow a discrete Zipf(zipf_a) law over a scattered
    entity ranking, stored in both directions (2 * num_triples CSR entries).  Relation ids
    are drawn but ignored, as the mean aggregator ignores them; parallel edges are kept."""
    dev = torch.device(device)
    N = num_entities
    ranks = torch.arange(1, N + 1, dtype=torch.float64, device=dev)
    cdf = torch.cumsum(ranks ** (-zipf_a), 0)
    cdf = cdf / cdf[-1]
    del ranks
    a, b, _ = _affine_bijection(N)
    t = torch.arange(num_triples, dtype=torch.int64, device=dev)

    def endpoint(stream: int) -> torch.Tensor:
        r = torch.searchsorted(cdf, hash_u01(seed, stream, t)).clamp_(0, N - 1)
        return (r * a + b) % N

    head = endpoint(0)
    tail = endpoint(1)
    tail = torch.where(tail == head, (tail + 1) % N, tail)
    _relation = hash64(seed, 2, t) % num_relations            # generated, unused by the method
    del cdf, t, _relation
    src = torch.cat([head, tail])
    dst = torch.cat([tail, head])
    del head, tail
    order = torch.sort(src, stable=True).indices
    indices = dst[order].to(torch.int32)
    counts = torch.bincount(src, minlength=N)
    indptr = torch.zeros(N + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=indptr[1:])
    return Graph(indptr.to(torch.int32), indices, N)


# ----------------------------------------------------------------------------------------
# features, seeds, gradients
# ----------------------------------------------------------------------------------------

def features(num_rows: int, dim: int, *, dist: str = "normal", dtype: torch.dtype = torch.float32,
             seed: int = 1, device: str = "cpu", scale: float = 0.1,
             chunk_rows: Optional[int] = None) -> torch.Tensor:
    """[num_rows, dim] table: N(0,1) (Box-Muller on hashed uniforms) or U(-scale, scale)."""
    dev = torch.device(device)
    out = torch.empty((num_rows, dim), dtype=dtype, device=dev)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // max(1, dim))
    for r0 in range(0, num_rows, chunk_rows):
        r1 = min(num_rows, r0 + chunk_rows)
        idx = torch.arange(r0 * dim, r1 * dim, dtype=torch.int64, device=dev)
        u1 = hash_u01(seed, 0, idx)
        if dist == "normal":
            u2 = hash_u01(seed, 1, idx)
            z = torch.sqrt(-2.0 * torch.log1p(-u1)) * torch.cos((2.0 * math.pi) * u2)
        elif dist == "uniform":
            z = (u1 * 2.0 - 1.0) * scale
        else:
            raise ValueError(dist)
        out[r0:r1] = z.reshape(r1 - r0, dim).to(dtype)
    return out


def edge_weights(num_edges: int, *, seed: int = 11, device: str = "cpu") -> torch.Tensor:
    """Per-edge weights for the weighted mean: hashed uniforms in [0, 1), fp32, aligned with `indices`."""
    out = torch.empty(num_edges, dtype=torch.float32, device=device)
    step = 1 << 27
    for e0 in range(0, num_edges, step):
        e1 = min(num_edges, e0 + step)
        out[e0:e1] = hash_u01(seed, 0, torch.arange(e0, e1, dtype=torch.int64, device=device)).float()
    return out


def seed_batches(num_nodes: int, batch: int, num_batches: int = 1, *, seed: int = 2) -> torch.Tensor:
    """[num_batches, batch] int32 node ids, each batch uniform without replacement."""
    rng = np.random.default_rng(seed)
    rows = [rng.choice(num_nodes, size=batch, replace=False) for _ in range(num_batches)]
    return torch.from_numpy(np.stack(rows).astype(np.int32))


def upstream_grad(shape, *, seed: int = 3, device: str = "cpu") -> torch.Tensor:
    """Upstream gradient ~ N(0,1), float32."""
    n = 1
    for s in shape:
        n *= int(s)
    return features(n, 1, dist="normal", seed=seed, device=device).reshape(*shape)


# ----------------------------------------------------------------------------------------
# the five workload shapes
# ----------------------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    graph: Graph
    x: torch.Tensor
    batch: int
    fanouts: Tuple[int, ...]
    sampler_seed: int = 0


WORKLOADS = ("tiny", "products", "social", "kg", "citation")

# (num_nodes, mean_deg, max_deg, D, dtype, dist, B, fanouts, wide_indptr); scale < 1 shrinks
# num_nodes (and, for the KG shape, the triple count) for CPU-sized rehearsals.
_SHAPES = {
    "products": dict(n=2_449_029, mean=50.5, max=17_000, D=100, dtype=torch.float32,
                     dist="normal", B=1024, fan=(15, 10), wide=False),
    "social":   dict(n=232_965, mean=492.0, max=21_700, D=602, dtype=torch.float32,
                     dist="normal", B=1024, fan=(25, 10), wide=False),
    "citation": dict(n=111_000_000, mean=14.5, max=100_000, D=128, dtype=torch.bfloat16,
                     dist="normal", B=4096, fan=(15, 10), wide=True),
}


def make_workload(name: str, *, device: str = "cpu", scale: float = 1.0) -> Workload:
    """Build one of the five workload shapes (graph seed 0, feature seed 1)."""
    if name == "tiny":
        g = tiny_graph()
        g = Graph(g.indptr.to(device), g.indices.to(device), g.num_nodes)
        x = features(g.num_nodes, 64, seed=1, device=device)
        return Workload(name, g, x, 1024, (10,))
    if name == "kg":
        n = max(64, int(2_500_000 * scale))
        t = max(64, int(16_100_000 * scale))
        g = kg_graph(n, t, seed=0, device=device)
        x = features(n, 128, dist="uniform", scale=0.1, seed=1, device=device)
        return Workload(name, g, x, 4096 if scale == 1.0 else min(4096, n // 2), (15,))
    s = _SHAPES[name]
    n = max(64, int(s["n"] * scale))
    max_deg = min(s["max"], max(4.0, n / 8))
    mean = min(s["mean"], max_deg / 4)
    g = chung_lu_graph(n, mean, max_deg, seed=0, device=device, wide_indptr=s["wide"])
    x = features(n, s["D"], dist=s["dist"], dtype=s["dtype"], seed=1, device=device)
    return Workload(name, g, x, s["B"] if scale == 1.0 else min(s["B"], n // 2), s["fan"])
