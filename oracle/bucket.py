"""The per-edge-bucket training step, batch by batch (oracle; test infrastructure).

Follows the six stages of Sec. 2.1 (positive selection, negative sampling,
embedding retrieval, batch assembly, batch computation, embedding update) with
the synchronous-update semantics of Sec. 3: every read of a batch sees the
tables as they were when the batch started, every write happens in the update
stage, and the next batch sees the update.  Relation embeddings and their
optimiser state live beside the node partitions and follow the same rule
(Sec. 3, storage arrangement item 3).

Adagrad (named in Sec. 2.1; the paper prints no formula) is the textbook rule
with a zero initial accumulator: all gradient rows addressed to one table row
in the batch are summed first (float64, rounded once to fp32), then
    S <- S + G*G ;  theta <- theta - lr * G / (sqrt(S) + eps)
in fp32 steps in exactly this order.  Rows no gradient addresses are not written.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from . import model, negatives


@dataclass
class OracleConfig:
    num_nodes: int
    num_relations: int
    dim: int
    num_partitions: int
    batch_size: int
    chunk_size: int
    num_negs: int
    num_degree_negs: int = 0
    score: int = model.DOT
    loss: int = model.SOFTMAX
    corrupt: int = 0              # 0 dst, 1 src, 2 both
    lr: float = 0.1
    eps: float = 1e-10
    neg_weight: float = -1.0      # logistic only; < 0 means 1 / num_negs
    margin: float = 1.0           # margin loss only
    seed: int = 0
    round_composed: bool = True   # translational score: u, v as fp32 numbers (False only for derivative checks)

    @property
    def rows_per_partition(self) -> int:
        return -(-self.num_nodes // self.num_partitions)

    @property
    def w_neg(self) -> float:
        return self.neg_weight if self.neg_weight >= 0 else 1.0 / self.num_negs

    @staticmethod
    def from_workload(w, seed: int, **kw) -> "OracleConfig":
        return OracleConfig(
            num_nodes=w.num_nodes, num_relations=w.num_relations, dim=w.dim,
            num_partitions=w.num_partitions, batch_size=w.batch_size, chunk_size=w.chunk_size,
            num_negs=w.num_negs, num_degree_negs=w.num_degree_negs, score=w.score, loss=w.loss,
            corrupt=w.corrupt, lr=w.lr, eps=w.eps, seed=seed, **kw)


class Tables:
    """Node partitions [E_p | S_p] (padded to equal size) and the relation table."""

    def __init__(self, cfg: OracleConfig, node_emb: np.ndarray, rel_emb: Optional[np.ndarray]):
        rp, n, d = cfg.rows_per_partition, cfg.num_partitions, cfg.dim
        assert node_emb.shape == (cfg.num_nodes, d)
        self.cfg = cfg
        self.E: List[np.ndarray] = []
        self.S: List[np.ndarray] = []
        for p in range(n):
            e = np.zeros((rp, d), np.float32)
            lo = p * rp
            hi = min(cfg.num_nodes, lo + rp)
            e[: hi - lo] = node_emb[lo:hi]
            self.E.append(e)
            self.S.append(np.zeros((rp, d), np.float32))
        nrel = max(cfg.num_relations, 1)
        self.RE = np.zeros((nrel, d), np.float32) if rel_emb is None else rel_emb.astype(np.float32).copy()
        self.RS = np.zeros_like(self.RE)

    def node_table(self, which: int) -> np.ndarray:
        """All node rows in global id order (which: 0 embeddings, 1 optimiser state)."""
        src = self.E if which == 0 else self.S
        return np.concatenate(src, axis=0)[: self.cfg.num_nodes]


def adagrad_rows(theta: np.ndarray, state: np.ndarray, rows: np.ndarray, grad64: np.ndarray, lr, eps):
    """Sparse Adagrad on unique `rows` with summed float64 gradients `grad64`."""
    g = grad64.astype(np.float32)
    s_new = state[rows] + g * g
    step = (np.float32(lr) * g) / (np.sqrt(s_new) + np.float32(eps))
    state[rows] = s_new
    theta[rows] = theta[rows] - step


def _coalesce(keys: List[np.ndarray], grads: List[np.ndarray]):
    k = np.concatenate(keys)
    g = np.concatenate(grads, axis=0)
    uniq, inv = np.unique(k, return_inverse=True)
    acc = np.zeros((uniq.size, g.shape[1]), np.float64)
    np.add.at(acc, inv, g)
    return uniq, acc


def batch_gradients(tab: Tables, i: int, j: int, bucket_edges: np.ndarray, b: int, epoch: int,
                    record: Optional[dict] = None):
    """Stages 1-5 for batch b of bucket (i, j): loss and coalesced gradients.

    Returns (loss, node, rel): loss is the float64 batch sum; node maps a table
    slot (0: partition i, 1: partition j when j != i) to (unique rows, summed
    float64 gradient rows); rel is the same pair for the relation table or None.
    record, when given, receives the batch's gradients, negative ids and touched rows; a
    callable under record["observer"] is shown every chunk's inputs and results
    (side index, corrupted side is dst, chunk, the chunk's edge rows, negative ids, the
    gathered float64 rows s, r, d, negs, and chunk_side's result) and takes no part in
    the computation."""
    cfg = tab.cfg
    lo = b * cfg.batch_size
    e = bucket_edges[lo: lo + cfg.batch_size]
    p = e.shape[0]
    uses_rel = cfg.score != model.DOT
    Ei, Ej = tab.E[i], tab.E[j]

    # stages 1-4: positives in stored order, negatives, row retrieval (snapshot reads)
    neg = negatives.batch_negatives(cfg, epoch, i, j, b, e, bucket_edges)
    s_all = Ei[e[:, 0]].astype(np.float64)
    d_all = Ej[e[:, 2]].astype(np.float64)
    r_all = tab.RE[e[:, 1]].astype(np.float64) if uses_rel else None

    ti, tj = 0, (0 if i == j else 1)      # node table slot of each role
    node_keys = [[], []]
    node_grads = [[], []]
    rel_keys, rel_grads = [], []
    loss = 0.0
    observer = record.get("observer") if record is not None else None

    # stage 5: batch computation, chunk by chunk, side by side
    nchunks = -(-p // cfg.chunk_size)
    for si, side in enumerate(negatives.sides_of(cfg)):
        is_dst = side == negatives.SIDE_DST
        neg_table, neg_slot = (Ej, tj) if is_dst else (Ei, ti)
        for c in range(nchunks):
            sl = slice(c * cfg.chunk_size, min(p, (c + 1) * cfg.chunk_size))
            ids = neg[si, c]
            neg_rows = neg_table[ids].astype(np.float64)
            out = model.chunk_side(cfg.score, cfg.loss, cfg.w_neg, is_dst,
                                   s_all[sl], r_all[sl] if uses_rel else None, d_all[sl],
                                   neg_rows, rounded=cfg.round_composed, margin=cfg.margin)
            loss += float(out["loss"].sum())
            node_keys[ti].append(e[sl, 0].astype(np.int64)); node_grads[ti].append(out["g_s"])
            node_keys[tj].append(e[sl, 2].astype(np.int64)); node_grads[tj].append(out["g_d"])
            node_keys[neg_slot].append(ids); node_grads[neg_slot].append(out["g_neg"])
            if uses_rel:
                rel_keys.append(e[sl, 1].astype(np.int64)); rel_grads.append(out["g_r"])
            if observer is not None:
                observer(si, is_dst, c, e[sl], ids, s_all[sl], r_all[sl] if uses_rel else None, d_all[sl], neg_rows, out)

    node = {}
    for slot in (0, 1):
        if node_keys[slot]:
            node[slot] = _coalesce(node_keys[slot], node_grads[slot])
    rel = None
    if uses_rel and rel_keys:
        rel = _coalesce(rel_keys, rel_grads)
    if record is not None:
        record["grads"] = (node, rel)
        record["neg_ids"] = neg
        record["touched"] = negatives.touched_rows(cfg, i, j, e, neg)
    return loss, node, rel


def train_batch(tab: Tables, i: int, j: int, bucket_edges: np.ndarray, b: int, epoch: int,
                record: Optional[dict] = None) -> float:
    """One batch of bucket (i, j), stages 1-6.  Returns the batch loss (float64 sum)."""
    cfg = tab.cfg
    loss, node, rel = batch_gradients(tab, i, j, bucket_edges, b, epoch, record)
    # stage 6: coalesced sparse Adagrad on every touched table
    for slot, part in ((0, i), (1, j)):
        if slot in node:
            rows, g = node[slot]
            adagrad_rows(tab.E[part], tab.S[part], rows, g, cfg.lr, cfg.eps)
    if rel is not None:
        adagrad_rows(tab.RE, tab.RS, rel[0], rel[1], cfg.lr, cfg.eps)
    return loss


def train_bucket(tab: Tables, i: int, j: int, bucket_edges: np.ndarray, epoch: int,
                 max_batches: Optional[int] = None) -> Dict[str, float]:
    """All batches of bucket (i, j) in stored order.  Returns loss sum and counts."""
    cfg = tab.cfg
    m = bucket_edges.shape[0]
    nb = -(-m // cfg.batch_size)
    if max_batches is not None:
        nb = min(nb, max_batches)
    loss = 0.0
    for b in range(nb):
        loss += train_batch(tab, i, j, bucket_edges, b, epoch)
    return dict(loss_sum=loss, batches=nb, edges=min(m, nb * cfg.batch_size))


def gather_global(tab: Tables, ids: np.ndarray) -> np.ndarray:
    """Embedding rows of global node ids (float64 copies)."""
    cfg = tab.cfg
    rp = cfg.rows_per_partition
    ids = np.asarray(ids, np.int64)
    out = np.zeros((ids.size, cfg.dim), np.float64)
    part = ids // rp
    for p in np.unique(part):
        m = part == p
        out[m] = tab.E[int(p)][ids[m] - int(p) * rp]
    return out


def score_edges(tab: Tables, src: np.ndarray, rel: Optional[np.ndarray], dst: np.ndarray) -> np.ndarray:
    """f(theta_s, theta_r, theta_d) for global node ids (float64)."""
    cfg = tab.cfg
    s = gather_global(tab, src)
    d = gather_global(tab, dst)
    r = tab.RE[np.asarray(rel, np.int64)].astype(np.float64) if cfg.score != model.DOT else None
    return model.positive_scores(cfg.score, s, r, d)
