"""Synthetic power-law graphs with the shapes of the paper's workloads (Table 3).

The public datasets the paper trains on are not available here; only their
sizes, relation counts and degree skew are taken.  Every generator is a pure
function of (workload, seed).

Recipe
------
* A node *rank* k in [0, V) is drawn from the continuous Zipf-Mandelbrot density
  p(x) ~ (x + q)^(-s) on [0, V) by inverse-CDF sampling and floored.  ``s = 0``
  gives the uniform distribution.
* Ranks are sent through a seeded permutation to node ids, so that hubs are
  spread over the node partitions instead of all sitting in partition 0.
* Relation ids are drawn the same way (no permutation).
* Multi-edges and self loops are kept.
* Edges are independent draws, so their generation order is already a uniform
  shuffle; bucketing is a stable partition by (src // R_p, dst // R_p) and node
  ids inside a bucket are stored partition-local.
"""

from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

SCORE_DOT, SCORE_DISTMULT, SCORE_COMPLEX, SCORE_TRANSE_L1 = 0, 1, 2, 3
LOSS_SOFTMAX, LOSS_LOGISTIC, LOSS_SOFTMAX_POS = 0, 1, 2
CORRUPT_DST, CORRUPT_SRC, CORRUPT_BOTH = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    num_nodes: int
    num_relations: int          # 0: graph without relation types
    num_edges: int
    dim: int
    num_partitions: int
    batch_size: int
    chunk_size: int
    num_negs: int               # negatives per chunk and corrupted side
    num_degree_negs: int        # how many of them are degree-weighted (the last ones)
    score: int
    loss: int = LOSS_SOFTMAX
    corrupt: int = CORRUPT_DST
    lr: float = 0.1
    eps: float = 1e-10
    init_std: float = 1e-3
    src_skew: Tuple[float, float] = (0.0, 1.0)   # (s, q) of the rank density
    dst_skew: Tuple[float, float] = (0.0, 1.0)
    rel_skew: Tuple[float, float] = (0.0, 1.0)
    stands_for: str = ""

    @property
    def rows_per_partition(self) -> int:
        return rows_per_partition(self.num_nodes, self.num_partitions)

    @property
    def sides(self) -> int:
        return 2 if self.corrupt == CORRUPT_BOTH else 1


def rows_per_partition(num_nodes: int, num_partitions: int) -> int:
    return -(-num_nodes // num_partitions)


WORKLOADS: Dict[str, Workload] = {
    # Tiny graph: Zipf(1.1) out-degree, uniform destinations.
    "c1": Workload("c1", 10_000, 0, 100_000, 32, 1, 1_000, 100, 64, 0, SCORE_DOT,
                   src_skew=(1.1, 1.0), stands_for="tiny synthetic"),
    # Social-graph shape (4.8 M nodes, 68 M edges); alpha ~ 2.1  =>  s = 1/(alpha-1) ~ 0.91;
    # q = 100 puts the largest degree at a few 1e4.
    "c2": Workload("c2", 4_800_000, 0, 68_000_000, 100, 4, 50_000, 50, 1_000, 500, SCORE_DOT,
                   src_skew=(0.91, 100.0), dst_skew=(0.91, 100.0), stands_for="LiveJournal shape"),
    # Knowledge-graph shape.
    "c3": Workload("c3", 15_000, 1_345, 483_000, 400, 1, 10_000, 100, 1_000, 0, SCORE_DISTMULT,
                   corrupt=CORRUPT_BOTH, src_skew=(0.7, 1.0), dst_skew=(0.7, 1.0), rel_skew=(1.0, 1.0),
                   stands_for="FB15k shape"),
    # Billion-edge social shape; alpha ~ 2.0 => s = 1, q ~ 34 => max degree ~ 3 M.
    "c4": Workload("c4", 41_600_000, 0, 1_460_000_000, 100, 16, 50_000, 50, 1_000, 0, SCORE_DOT,
                   src_skew=(1.0, 34.0), dst_skew=(1.0, 34.0), stands_for="Twitter shape"),
    # Large knowledge-graph shape.
    "c5": Workload("c5", 86_000_000, 14_824, 338_000_000, 100, 16, 50_000, 50, 1_000, 0, SCORE_COMPLEX,
                   corrupt=CORRUPT_BOTH, src_skew=(0.8, 1.0), dst_skew=(0.8, 1.0), rel_skew=(1.0, 1.0),
                   stands_for="Freebase86M shape"),
}


def scaled(w: Workload, node_div: int, edge_div: Optional[int] = None, **overrides) -> Workload:
    """The same workload with fewer nodes/edges (degree structure and all
    per-batch parameters unchanged).  Used where a full-size graph does not fit
    the host or the time budget; the name records the scale."""
    edge_div = node_div if edge_div is None else edge_div
    return dataclasses.replace(
        w,
        name=f"{w.name}/nodes÷{node_div},edges÷{edge_div}",
        num_nodes=max(w.num_partitions, w.num_nodes // node_div),
        num_edges=max(1, w.num_edges // edge_div),
        **overrides,
    )


def _sample_ranks(rng: np.random.Generator, count: int, size: int, skew: Tuple[float, float]) -> np.ndarray:
    """Inverse-CDF draw from p(x) ~ (x+q)^(-s) on [0, size), floored to int64."""
    s, q = skew
    u = rng.random(count)
    if s == 0.0:
        x = u * size
    elif abs(s - 1.0) < 1e-12:
        x = q * np.power((size + q) / q, u) - q
    else:
        a = q ** (1.0 - s)
        b = (size + q) ** (1.0 - s)
        x = np.power(a + u * (b - a), 1.0 / (1.0 - s)) - q
    k = x.astype(np.int64)
    np.clip(k, 0, size - 1, out=k)
    return k


def generate_edges(w: Workload, seed: int, block: int = 1 << 24, progress=None):
    """Global edge list as three int64/int32 arrays (src, rel, dst), seeded.
    `progress(done, total)` is called after every block (long generations report through it)."""
    rng = np.random.default_rng([seed, 0xE])
    perm = np.random.default_rng([seed, 0xF]).permutation(w.num_nodes)
    src = np.empty(w.num_edges, np.int64)
    dst = np.empty(w.num_edges, np.int64)
    rel = np.zeros(w.num_edges, np.int32)
    for lo in range(0, w.num_edges, block):
        hi = min(w.num_edges, lo + block)
        src[lo:hi] = perm[_sample_ranks(rng, hi - lo, w.num_nodes, w.src_skew)]
        dst[lo:hi] = perm[_sample_ranks(rng, hi - lo, w.num_nodes, w.dst_skew)]
        if w.num_relations > 1:
            rel[lo:hi] = _sample_ranks(rng, hi - lo, w.num_relations, w.rel_skew)
        if progress is not None:
            progress(hi, w.num_edges)
    return src, rel, dst


def _rank_cdf(x: np.ndarray, size: int, skew: Tuple[float, float]) -> np.ndarray:
    """CDF of the rank density p(x) ~ (x+q)^(-s) on [0, size) at the points x (float64)."""
    s, q = skew
    x = np.asarray(x, np.float64)
    if s == 0.0:
        return x / size
    if abs(s - 1.0) < 1e-12:
        return np.log((x + q) / q) / np.log((size + q) / q)
    a = q ** (1.0 - s)
    b = (size + q) ** (1.0 - s)
    return (np.power(x + q, 1.0 - s) - a) / (b - a)


def generate_bucket_edges(w: Workload, seed: int, wanted):
    """Edges of the buckets in `wanted` (pairs (i, j)) only, for graphs too large to generate whole.

    The edges of generate_edges are independent draws with independent endpoints, so the edges of
    bucket (i, j) are independent draws too: their number is Binomial(E, P(src in i) P(dst in j)), and
    each endpoint follows the rank distribution restricted to its partition (rank -> node through the
    same seeded permutation).  This samples exactly that law (another random stream than
    generate_edges: the same distribution, not the same edges).
    Returns ({(i, j): int32 [m_ij, 3]}, {(i, j): expected share of all edges})."""
    n, rp = w.num_partitions, w.rows_per_partition
    perm = np.random.default_rng([seed, 0xF]).permutation(w.num_nodes)
    part_of_rank = perm // rp
    cache = {}

    def side(p, skew):
        key = (p, skew)
        if key not in cache:
            ranks = np.flatnonzero(part_of_rank == p)
            pmf = _rank_cdf(ranks + 1.0, w.num_nodes, skew) - _rank_cdf(ranks, w.num_nodes, skew)
            cdf = np.cumsum(pmf)
            mass = float(cdf[-1])
            cache[key] = (ranks, cdf / mass, mass)
        return cache[key]

    out, share = {}, {}
    for (i, j) in wanted:
        rs, cs, ms = side(i, w.src_skew)
        rd, cd, md = side(j, w.dst_skew)
        rng = np.random.default_rng([seed, 0xB0C, i, j])
        m = int(rng.binomial(w.num_edges, ms * md))
        e = np.empty((m, 3), np.int32)
        e[:, 0] = perm[rs[np.minimum(np.searchsorted(cs, rng.random(m), side="right"), rs.size - 1)]] - i * rp
        e[:, 2] = perm[rd[np.minimum(np.searchsorted(cd, rng.random(m), side="right"), rd.size - 1)]] - j * rp
        e[:, 1] = _sample_ranks(rng, m, w.num_relations, w.rel_skew) if w.num_relations > 1 else 0
        out[(i, j)] = e
        share[(i, j)] = ms * md
    return out, share


def bucket_edges(w: Workload, src: np.ndarray, rel: np.ndarray, dst: np.ndarray, progress=None):
    """Stable partition of the edges into n*n buckets.

    Returns {(i, j): int32 [m_ij, 3]} with columns (src_local, rel, dst_local);
    the order inside a bucket is the generation order."""
    n = w.num_partitions
    rp = w.rows_per_partition
    pi = src // rp
    pj = dst // rp
    bid = (pi * n + pj).astype(np.int16 if n * n < 32768 else np.int32)
    del pi, pj
    if progress is not None:
        progress(0, n * n)
    order = np.argsort(bid, kind="stable")
    counts = np.bincount(bid, minlength=n * n)
    out = {}
    pos = 0
    for b in range(n * n):
        idx = order[pos:pos + counts[b]]
        pos += counts[b]
        i, j = divmod(b, n)
        e = np.empty((idx.size, 3), np.int32)
        e[:, 0] = src[idx] - i * rp
        e[:, 1] = rel[idx]
        e[:, 2] = dst[idx] - j * rp
        out[(i, j)] = e
        if progress is not None:
            progress(b + 1, n * n)
    return out


def init_tables(w: Workload, seed: int):
    """Initial node and relation embeddings, N(0, init_std^2), fp32.

    Relation rows use the same distribution (never zero: a zero relation row
    would null every first-step node gradient of a multiplicative score)."""
    rng = np.random.default_rng([seed, 0xA])
    node = rng.standard_normal((w.num_nodes, w.dim), dtype=np.float32)
    node *= np.float32(w.init_std)
    nrel = max(w.num_relations, 1)
    relt = np.random.default_rng([seed, 0xB]).standard_normal((nrel, w.dim), dtype=np.float32)
    relt *= np.float32(w.init_std)
    return node, relt
