"""Shared helpers of the GPU parity tests (oracle side + comparison rules)."""

from __future__ import annotations

import numpy as np

from oracle import model
from oracle.bucket import OracleConfig, Tables, train_batch

# Tolerances (spec: scores 1e-5 relative in fp32, embeddings 1e-5 relative).
#   embeddings:  |gpu - oracle| <= 1e-5 * max(|oracle|, lr)
#   state:       |gpu - oracle| <= 3e-5 * |oracle| + 1e-30   (a sum of squares: twice the relative error)
# An element whose batch gradient nearly cancels, |G| < 1e-4 * sum|terms| in some batch, is
# ill-conditioned under any reordering of the fp32 arithmetic (Adagrad's first step is
# lr * G / (|G| + eps), i.e. sign-like); such elements are excluded and counted, and their
# share must stay below 2e-3.
EMB_RTOL = 1e-5
STATE_RTOL = 3e-5
COND = 1e-4
MAX_EXCLUDED = 2e-3


def oracle_config(**kw) -> OracleConfig:
    return OracleConfig(**kw)


class OracleRun:
    """Trains batches with the oracle and tracks ill-conditioned elements per table."""

    def __init__(self, cfg: OracleConfig, node: np.ndarray, rel):
        self.cfg = cfg
        self.tab = Tables(cfg, node, rel)
        rp, d = cfg.rows_per_partition, cfg.dim
        self.bad_node = [np.zeros((rp, d), bool) for _ in range(cfg.num_partitions)]
        self.bad_rel = np.zeros_like(self.tab.RE, dtype=bool)
        self.touched_node = [np.zeros(rp, bool) for _ in range(cfg.num_partitions)]
        self.touched_rel = np.zeros(self.tab.RE.shape[0], bool)
        self.loss = 0.0

    def train_bucket(self, i, j, edges, epoch, max_batches=None):
        cfg = self.cfg
        nb = -(-edges.shape[0] // cfg.batch_size)
        if max_batches is not None:
            nb = min(nb, max_batches)
        loss = 0.0
        for b in range(nb):
            rec = {}
            loss += train_batch(self.tab, i, j, edges, b, epoch, record=rec)
            node, rel = rec["grads"]
            mags = rec["grad_abs_sums"]
            for slot, part in ((0, i), (1, j)):
                if slot in node:
                    rows, g = node[slot]
                    self.bad_node[part][rows] |= np.abs(g) < COND * mags[slot]
                    self.touched_node[part][rows] = True
            if rel is not None:
                rows, g = rel
                self.bad_rel[rows] |= np.abs(g) < COND * mags[2]
                self.touched_rel[rows] = True
        self.loss += loss
        return loss


def compare_table(name, got, want, bad, rtol, floor, atol=0.0):
    """Element-wise comparison; returns the excluded fraction."""
    assert got.shape == want.shape, (name, got.shape, want.shape)
    got64, want64 = got.astype(np.float64), want.astype(np.float64)
    tol = rtol * np.maximum(np.abs(want64), floor) + atol
    err = np.abs(got64 - want64)
    viol = (err > tol) & ~bad
    if viol.any():
        idx = np.argwhere(viol)[:5]
        lines = [f"{tuple(k)}: gpu={got64[tuple(k)]!r} oracle={want64[tuple(k)]!r}" for k in idx]
        raise AssertionError(f"{name}: {int(viol.sum())} of {viol.size} elements outside tolerance; first: " + "; ".join(lines))
    return float(bad.mean())


def check_scores(got, want, s64, r64, d64, score):
    """|gpu - oracle| <= 1e-5 * max(|oracle|, ||u|| ||d||): norm-wise bound of a dot product."""
    u = model.compose_u(score, s64, r64)
    bound = np.linalg.norm(u, axis=1) * np.linalg.norm(d64, axis=1)
    tol = 1e-5 * np.maximum(np.abs(want), bound)
    err = np.abs(got.astype(np.float64) - want)
    assert (err <= tol).all(), f"score mismatch: max err {err.max():.3e}, worst tol {tol[err.argmax()]:.3e}"
