"""Negative sampling of one batch: integer-only, stateless (oracle; test infrastructure).

The paper samples negatives on the GPU per batch (Sec. 2.1 stage 2, Sec. 3 step 3)
but fixes no generator.  The reading used here: a counter hash over the tuple
(seed, epoch, src partition, dst partition, batch, chunk, side, k) built from the
splitmix64 output function, reduced to a range by the high half of a 64x64-bit
product.  No floating point takes part in index generation.
"""

from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15

SIDE_DST = 0   # the destination is replaced by a sampled node of partition j
SIDE_SRC = 1   # the source is replaced by a sampled node of partition i


def _u64(x):
    return np.asarray(x, dtype=np.uint64)


def mix64(z):
    """splitmix64 output function on uint64 arrays (wrap-around arithmetic)."""
    z = _u64(z).copy()
    with np.errstate(over="ignore"):
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return z


def fold(h, field):
    """Absorb one integer field into the running hash: mix64(h + GOLDEN + field)."""
    with np.errstate(over="ignore"):
        return mix64(_u64(h) + np.uint64(GOLDEN) + _u64(field))


def mulhi64(a, b: int):
    """High 64 bits of a*b for a uint64 array a and a Python int 0 <= b < 2^64."""
    a = _u64(a)
    m32 = np.uint64(0xFFFFFFFF)
    s32 = np.uint64(32)
    al, ah = a & m32, a >> s32
    bl, bh = np.uint64(b & 0xFFFFFFFF), np.uint64(b >> 32)
    with np.errstate(over="ignore"):
        ll = al * bl
        hl = ah * bl
        lh = al * bh
        hh = ah * bh
        cross = (ll >> s32) + (hl & m32) + (lh & m32)
        return hh + (hl >> s32) + (lh >> s32) + (cross >> s32)


def chunk_hash(seed: int, epoch: int, i: int, j: int, b: int, c: int, side: int, num: int):
    """H(seed, epoch, i, j, b, c, side, k) for k = 0..num-1."""
    h = np.uint64(seed & MASK64)
    for f in (epoch, i, j, b, c, side):
        h = fold(h, f)
    return fold(h, np.arange(num, dtype=np.uint64))


def rows_valid(num_nodes: int, num_partitions: int, part: int) -> int:
    """Rows of a partition that hold a real node (the last partition is padded)."""
    rp = -(-num_nodes // num_partitions)
    return max(0, min(rp, num_nodes - part * rp))


def chunk_negatives(cfg, epoch, i, j, b, c, side, bucket_edges):
    """Local row ids of the chunk's shared negatives for one corrupted side.

    The first num_negs - num_degree_negs ids are uniform over the valid rows of
    the side's partition; the rest are the side's endpoint of a uniformly drawn
    edge of the current bucket (in-bucket degree-proportional)."""
    n_all = cfg.num_negs
    n_uni = n_all - cfg.num_degree_negs
    h = chunk_hash(cfg.seed, epoch, i, j, b, c, side, n_all)
    part = j if side == SIDE_DST else i
    ids = np.empty(n_all, np.int64)
    ids[:n_uni] = mulhi64(h[:n_uni], rows_valid(cfg.num_nodes, cfg.num_partitions, part)).astype(np.int64)
    if n_uni < n_all:
        q = mulhi64(h[n_uni:], bucket_edges.shape[0]).astype(np.int64)
        col = 2 if side == SIDE_DST else 0
        ids[n_uni:] = bucket_edges[q, col]
    return ids


def sides_of(cfg):
    """Corrupted sides in processing order for the config's corruption mode."""
    return {0: (SIDE_DST,), 1: (SIDE_SRC,), 2: (SIDE_DST, SIDE_SRC)}[cfg.corrupt]


def batch_negatives(cfg, epoch, i, j, b, batch_edges, bucket_edges):
    """ids[side_slot][chunk][k] for every chunk of batch b (int64 array)."""
    p = batch_edges.shape[0]
    nchunks = -(-p // cfg.chunk_size)
    sides = sides_of(cfg)
    out = np.empty((len(sides), nchunks, cfg.num_negs), np.int64)
    for si, side in enumerate(sides):
        for c in range(nchunks):
            out[si, c] = chunk_negatives(cfg, epoch, i, j, b, c, side, bucket_edges)
    return out


def touched_rows(cfg, i, j, batch_edges, neg_ids):
    """Sorted unique (table, row) pairs the batch updates, as a single int64 key.

    Table 0 is node partition i, table 1 is node partition j (folded into table
    0 when i == j), table 2 is the relation table (only for scores that use it).
    key = table * 2^32 + row."""
    keys = []
    t_dst = 0 if i == j else 1
    keys.append(batch_edges[:, 0].astype(np.int64))
    keys.append((t_dst << 32) + batch_edges[:, 2].astype(np.int64))
    if cfg.score != 0:
        keys.append((2 << 32) + batch_edges[:, 1].astype(np.int64))
    for si, side in enumerate(sides_of(cfg)):
        t = t_dst if side == SIDE_DST else 0
        keys.append((t << 32) + neg_ids[si].reshape(-1))
    return np.unique(np.concatenate(keys))
