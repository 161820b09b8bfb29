"""Seeded synthetic inputs: community-structured graphs, features, weights, batches.

This module only manufactures inputs.  It holds none of the sampling method's
arithmetic and is the one piece of code that both the CPU oracle's tests and
the HIP path's tests/bench use, so that the two sides see identical bytes.

The graphs stand in for the public graphs the paper trains on (Section 5.1,
Table 1): nodes are split evenly over partitions by contiguous id range, as the
paper divides nodes evenly among GPUs, and a planted community structure makes
most edges intra-partition.  The propagation matrix is the symmetric
normalisation with self-loops, P = D^-1/2 (A + I) D^-1/2, of the GCN the paper
builds on (Section 3, "P is the normalized Laplacian matrix of the graph").
"""
from __future__ import annotations

import dataclasses
import numpy as np

__all__ = [
    "Graph", "Config", "CONFIGS", "partition_bounds", "make_sbm", "make_chung_lu",
    "make_graph", "make_features", "to_bf16_bits", "glorot_uniform", "make_batch",
    "layer_dims",
]


@dataclasses.dataclass
class Graph:
    """CSR of P with ascending column ids per row, plus the partition map."""
    n_nodes: int
    rowptr: np.ndarray        # int64 [n_nodes + 1]
    colidx: np.ndarray        # int32 [nnz]
    val: np.ndarray           # float32 [nnz]
    part_bounds: np.ndarray   # int32 [P + 1], partition p owns ids [b[p], b[p+1])
    local_part: int = 0
    rownorm2_max: float = 1.0  # upper bound on max_i sum_j P_ij^2

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])

    @property
    def local_lo(self) -> int:
        return int(self.part_bounds[self.local_part])

    @property
    def local_hi(self) -> int:
        return int(self.part_bounds[self.local_part + 1])


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    kind: str                 # "sbm" | "chung_lu"
    seed: int
    n_nodes: int
    n_parts: int
    feat_dim: int
    hidden: int
    n_layers: int
    n_classes: int            # 0: last layer outputs `hidden`
    batch: int
    samples: int
    skew: float
    feat_dtype: str = "f32"   # "f32" | "bf16"
    # sbm
    p_in: float = 0.0
    p_out: float = 0.0
    mean_degree: float = 0.0
    intra_frac: float = 0.0
    # chung-lu
    exponent: float = 0.0
    skews: tuple = ()


CONFIGS = {
    "tiny": Config("tiny", "sbm", 0, 4096, 4, 64, 64, 2, 0, 256, 256, 4.0,
                   p_in=0.004, p_out=0.0005),
    "medium": Config("medium", "sbm", 1, 262_144, 8, 128, 256, 2, 0, 1024, 1024, 8.0,
                     mean_degree=50.0, intra_frac=0.80),
    "dense": Config("dense", "chung_lu", 2, 232_965, 8, 602, 256, 2, 41, 2048, 2048, 8.0,
                    mean_degree=490.0, intra_frac=0.85, exponent=2.1,
                    skews=(1.0, 2.0, 4.0, 8.0, 16.0)),
    "mid": Config("mid", "sbm", 3, 716_847, 8, 300, 512, 3, 100, 4096, 4096, 8.0,
                  mean_degree=19.0, intra_frac=0.75),
    "large": Config("large", "chung_lu", 4, 2_449_029, 16, 100, 256, 3, 47, 8192, 8192, 16.0,
                    feat_dtype="bf16", mean_degree=51.0, intra_frac=0.80, exponent=2.2),
}


def layer_dims(cfg: Config) -> list[tuple[int, int]]:
    """(F_in, F_out) of each GCN layer, bottom layer first."""
    dims = []
    f = cfg.feat_dim
    for l in range(cfg.n_layers):
        last = l == cfg.n_layers - 1
        out = cfg.n_classes if (last and cfg.n_classes) else cfg.hidden
        dims.append((f, out))
        f = out
    return dims


def partition_bounds(n_nodes: int, n_parts: int) -> np.ndarray:
    return np.array([(p * n_nodes) // n_parts for p in range(n_parts + 1)], dtype=np.int32)


# ---------------------------------------------------------------------------
# CSR assembly shared by both graph families
# ---------------------------------------------------------------------------

def _finish(n: int, und_keys: np.ndarray, bounds: np.ndarray) -> Graph:
    """und_keys: unique int64 keys (u << 32) | v with u < v.  Symmetrise, add
    self-loops, normalise symmetrically, emit CSR with ascending columns."""
    mask = np.int64(0xFFFFFFFF)
    u = und_keys >> 32
    v = und_keys & mask
    deg = np.bincount(u, minlength=n) + np.bincount(v, minlength=n) + 1  # self-loop counted
    loops = np.arange(n, dtype=np.int64)
    keys = np.concatenate([und_keys, (v << 32) | u, (loops << 32) | loops])
    del u, v, und_keys, loops
    keys.sort()
    col = (keys & mask).astype(np.int32)
    del keys
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    dinv = 1.0 / np.sqrt(deg.astype(np.float64))
    val = (np.repeat(dinv, deg) * dinv[col]).astype(np.float32)
    return Graph(n, rowptr, col, val, bounds.astype(np.int32), 0, 1.0)


def _uniform_pairs(rng, lo_a, n_a, lo_b, n_b, m, same):
    if m == 0:
        return np.empty(0, np.int64), np.empty(0, np.int64)
    a = rng.integers(0, n_a, size=m, dtype=np.int64) + lo_a
    b = rng.integers(0, n_b, size=m, dtype=np.int64) + lo_b
    if same:
        keep = a != b
        a, b = a[keep], b[keep]
    return np.minimum(a, b), np.maximum(a, b)


def make_sbm(n_nodes: int, n_parts: int, p_in: float, p_out: float, seed: int) -> Graph:
    """Stochastic block model on contiguous equal blocks.  For every block pair
    the edge count is Binomial(#pairs, p) and that many uniform node pairs are
    drawn; repeated pairs collapse (a negligible deficit at these densities)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    bounds = partition_bounds(n_nodes, n_parts)
    chunks = []
    for a in range(n_parts):
        lo_a, n_a = int(bounds[a]), int(bounds[a + 1] - bounds[a])
        for b in range(a, n_parts):
            lo_b, n_b = int(bounds[b]), int(bounds[b + 1] - bounds[b])
            same = a == b
            pairs = n_a * (n_a - 1) // 2 if same else n_a * n_b
            m = int(rng.binomial(pairs, p_in if same else p_out))
            u, v = _uniform_pairs(rng, lo_a, n_a, lo_b, n_b, m, same)
            chunks.append((u << 32) | v)
    keys = np.unique(np.concatenate(chunks)) if chunks else np.empty(0, np.int64)
    return _finish(n_nodes, keys, bounds)


def sbm_probs(n_nodes: int, n_parts: int, mean_degree: float, intra_frac: float):
    """Block probabilities that give the requested mean degree (self-loop
    excluded) and intra-partition edge fraction."""
    m = n_nodes * mean_degree / 2.0
    nb = n_nodes / n_parts
    intra_pairs = n_parts * nb * (nb - 1) / 2.0
    inter_pairs = n_parts * (n_parts - 1) / 2.0 * nb * nb
    return intra_frac * m / intra_pairs, (1.0 - intra_frac) * m / inter_pairs


def make_chung_lu(n_nodes: int, n_parts: int, mean_degree: float, intra_frac: float,
                  exponent: float, seed: int) -> Graph:
    """Chung-Lu style power-law graph with a planted contiguous partition.

    Expected degrees follow theta(r) ~ (r + r0)^(-1/(exponent-1)) over ranks r,
    with r0 set so that the largest expected degree is min(sqrt(2m), partition
    size).  Rank r lives in partition r mod P at a shuffled slot, so every
    partition carries the same degree mix.  Each undirected edge picks one
    endpoint by rank, then the second endpoint by an independent rank draw that
    is snapped into the first endpoint's partition with a probability chosen so
    that the overall intra-partition edge fraction is `intra_frac`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    bounds = partition_bounds(n_nodes, n_parts)
    sizes = np.diff(bounds).astype(np.int64)
    n = n_nodes
    m = int(round(n * mean_degree / 2.0))
    alpha = 1.0 / (exponent - 1.0)
    cap = min(np.sqrt(2.0 * m), float(sizes.min()))

    def top_degree(r0):
        a, b = r0 ** (1 - alpha), (n + r0) ** (1 - alpha)
        p0 = ((1 + r0) ** (1 - alpha) - a) / (b - a)
        return 2.0 * m * p0

    lo_r, hi_r = 1e-3, float(n)
    for _ in range(200):
        mid = np.sqrt(lo_r * hi_r)
        if top_degree(mid) > cap:
            lo_r = mid
        else:
            hi_r = mid
    r0 = hi_r
    a, b = r0 ** (1 - alpha), (n + r0) ** (1 - alpha)

    def draw_ranks(k):
        uu = rng.random(k)
        r = np.floor((uu * (b - a) + a) ** (1.0 / (1 - alpha)) - r0).astype(np.int64)
        return np.clip(r, 0, n - 1)

    # slot shuffles: rank r -> partition r % P, slot perm_p[(r // P) % size_p]
    perms = [rng.permutation(int(s)) for s in sizes]
    perm_flat = np.concatenate([p.astype(np.int64) + int(bounds[i]) for i, p in enumerate(perms)])
    perm_off = np.concatenate([[0], np.cumsum(sizes)])[:-1]

    def rank_to_node(r, part=None):
        p = (r % n_parts) if part is None else part
        slot = (r // n_parts) % sizes[p]
        return perm_flat[perm_off[p] + slot], p

    # a free second endpoint lands in the same partition with probability ~1/P
    snap = (intra_frac - 1.0 / n_parts) / (1.0 - 1.0 / n_parts)
    def draw_edges(m_draw):
        chunks = []
        step = 8_000_000
        for start in range(0, m_draw, step):
            k = min(step, m_draw - start)
            u, pu = rank_to_node(draw_ranks(k))
            r2 = draw_ranks(k)
            forced = rng.random(k) < snap
            p2 = np.where(forced, pu, r2 % n_parts)
            v, _ = rank_to_node(r2, p2)
            keep = u != v
            u, v = u[keep], v[keep]
            chunks.append((np.minimum(u, v) << 32) | np.maximum(u, v))
        return chunks

    # repeated pairs collapse (hubs lose the most); top up until within 0.5 % of m
    keys = np.unique(np.concatenate(draw_edges(m)))
    for _ in range(4):
        deficit = m - keys.shape[0]
        if deficit <= 0.005 * m:
            break
        keys = np.unique(np.concatenate([keys] + draw_edges(int(deficit * 1.1))))
    return _finish(n, keys, bounds)


def make_graph(cfg: Config) -> Graph:
    if cfg.kind == "sbm":
        if cfg.p_in > 0:
            p_in, p_out = cfg.p_in, cfg.p_out
        else:
            p_in, p_out = sbm_probs(cfg.n_nodes, cfg.n_parts, cfg.mean_degree, cfg.intra_frac)
        return make_sbm(cfg.n_nodes, cfg.n_parts, p_in, p_out, cfg.seed)
    if cfg.kind == "chung_lu":
        return make_chung_lu(cfg.n_nodes, cfg.n_parts, cfg.mean_degree, cfg.intra_frac,
                             cfg.exponent, cfg.seed)
    raise ValueError(cfg.kind)


# ---------------------------------------------------------------------------
# features, weights, batches
# ---------------------------------------------------------------------------

def make_features(n_rows: int, dim: int, seed: int) -> np.ndarray:
    """float32 [n_rows, dim], i.i.d. N(0,1)."""
    rng = np.random.Generator(np.random.PCG64([seed, 0xFEA7]))
    return rng.standard_normal((n_rows, dim), dtype=np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest-even) and return the 16-bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def glorot_uniform(fan_in: int, fan_out: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64([seed, 0x61070, fan_in, fan_out]))
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=(fan_in, fan_out)).astype(np.float32)


def make_batch(g: Graph, batch: int, seed: int, it: int = 0) -> np.ndarray:
    """`batch` distinct uniform local target nodes, ascending, int32."""
    rng = np.random.Generator(np.random.PCG64([seed, 0xBA7C4, it]))
    n_local = g.local_hi - g.local_lo
    batch = min(batch, n_local)
    ids = rng.choice(n_local, size=batch, replace=False).astype(np.int64) + g.local_lo
    ids.sort()
    return ids.astype(np.int32)
