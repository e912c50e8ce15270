"""Shared helpers of the GPU parity tests (oracle side + comparison rules)."""

from __future__ import annotations

import numpy as np

from oracle import model
from oracle.bucket import OracleConfig, Tables, train_batch

# Tolerances (spec: scores 1e-5 relative in fp32, embeddings 1e-5 relative).
#
#   embeddings:  |gpu - oracle| <= 1e-5 * max(|oracle|, lr) + forward_error
#   state:       |gpu - oracle| <= 3e-5 * |oracle| + forward_error_state
#
# forward_error is the first-order effect, on the Adagrad step, of evaluating the batch
# gradient G of an element in fp32 in any order: every gradient element is a sum of
# products whose absolute values add up to M (computed by the oracle next to G), and an
# fp32 evaluation of it (a length-d dot product behind every softmax weight, then sums over
# the chunk and over the occurrences of the row) is off by at most KAPPA * M with KAPPA a
# few dozen roundoffs.  The step theta -= lr * G / (sqrt(S) + eps) then moves by at most
# lr * KAPPA * M / (sqrt(S) + eps), and the accumulator S += G*G by 2 |G| KAPPA M + (KAPPA M)^2
# (the square matters only where G itself vanishes: the translational score with all signs equal
# and sum_k W_k = 1).  For an
# element without cancellation (M ~ |G| ~ sqrt(S)) this adds 2e-7 to a tolerance of 1e-6;
# it only matters where the gradient terms nearly cancel, which no fp32 order can reproduce.
# The error of an fp32 dot product grows with the square root of its length: KAPPA is 32 roundoffs
# up to dim 128 and grows like sqrt(dim / 128) beyond (45 roundoffs at 256, 57 at 400, 64 at 512).
# Softmax weights and dl/df are functions of score differences and inherit the absolute error of the
# fp32 scores, which scales with A = sum_j |q_j| |theta_j| and not with the score: the oracle widens
# their magnitudes by (1 + max A / 4) per row (8 roundoffs times A; 1.25 at the benchmark workloads'
# initial scale, two orders of magnitude once scores reach the hundreds), and the batch loss is allowed
# KAPPA * sum_e max A_e / 4 beside its 1e-5 relative bound.  For the translational score the same role
# is played by max |S| dim / 128.
# Below the normal range of fp32 (2^-126) results are spaced 2^-149 apart and a relative bound means
# nothing: every comparison allows two such steps on top.
EMB_RTOL = 1e-5
STATE_RTOL = 3e-5
KAPPA = 32 * 2.0 ** -24        # ~1.9e-6
FP32_SUBNORMAL_STEP = 2.0 ** -149


def kappa_for(dim: int) -> float:
    return KAPPA * max(1.0, (dim / 128.0) ** 0.5)


class OracleRun:
    """Trains batches with the oracle and accumulates the forward-error allowance per element."""

    def __init__(self, cfg: OracleConfig, node: np.ndarray, rel):
        self.cfg = cfg
        self.tab = Tables(cfg, node, rel)
        rp, d = cfg.rows_per_partition, cfg.dim
        n = cfg.num_partitions
        self.fe_node = [np.zeros((rp, d)) for _ in range(n)]      # allowance on embeddings
        self.fs_node = [np.zeros((rp, d)) for _ in range(n)]      # allowance on optimiser state
        self.fe_rel = np.zeros(self.tab.RE.shape)
        self.fs_rel = np.zeros(self.tab.RE.shape)
        self.touched_node = [np.zeros(rp, bool) for _ in range(n)]
        self.touched_rel = np.zeros(self.tab.RE.shape[0], bool)
        self.loss = 0.0

    def _allow(self, fe, fs, state, rows, g, mag):
        lr, eps = self.cfg.lr, self.cfg.eps
        s_new = state[rows].astype(np.float64)               # after the update
        kappa = kappa_for(self.cfg.dim)
        fe[rows] += lr * kappa * mag / (np.sqrt(s_new) + eps)
        fs[rows] += 2.0 * np.abs(g) * kappa * mag + (kappa * mag) ** 2      # |(G + e)^2 - G^2| <= 2 |G| e + e^2

    def set_state(self, node_E, node_S, rel_E=None, rel_S=None):
        """Restart from given tables (global node order) and clear the allowances."""
        cfg = self.cfg
        rp = cfg.rows_per_partition
        for p in range(cfg.num_partitions):
            lo, hi = p * rp, min(cfg.num_nodes, (p + 1) * rp)
            self.tab.E[p][: hi - lo] = node_E[lo:hi]
            self.tab.S[p][: hi - lo] = node_S[lo:hi]
            self.fe_node[p][:] = 0
            self.fs_node[p][:] = 0
            self.touched_node[p][:] = False
        if rel_E is not None:
            self.tab.RE[:] = rel_E
            self.tab.RS[:] = rel_S
        self.fe_rel[:] = 0
        self.fs_rel[:] = 0
        self.touched_rel[:] = False

    def train_bucket(self, i, j, edges, epoch, max_batches=None, batch_begin=0):
        cfg = self.cfg
        nb = -(-edges.shape[0] // cfg.batch_size)
        if max_batches is not None:
            nb = min(nb, batch_begin + max_batches)
        loss = 0.0
        self.last_loss_allowance = 0.0       # of this call's loss sum, absolute
        for b in range(batch_begin, nb):
            rec = {}
            loss += train_batch(self.tab, i, j, edges, b, epoch, record=rec)
            self.last_loss_allowance += kappa_for(cfg.dim) * rec["loss_magnitude"]
            node, rel = rec["grads"]
            mags = rec["grad_magnitudes"]
            for slot, part in ((0, i), (1, j)):
                if slot in node:
                    rows, g = node[slot]
                    self._allow(self.fe_node[part], self.fs_node[part], self.tab.S[part], rows, g, mags[slot])
                    self.touched_node[part][rows] = True
            if rel is not None:
                rows, g = rel
                self._allow(self.fe_rel, self.fs_rel, self.tab.RS, rows, g, mags[2])
                self.touched_rel[rows] = True
        self.loss += loss
        return loss

    def node_allowance(self, which):
        src = self.fe_node if which == 0 else self.fs_node
        return np.concatenate(src, 0)[: self.cfg.num_nodes]


def compare_table(name, got, want, allowance, rtol, floor):
    """Element-wise comparison: |got - want| <= rtol * max(|want|, floor) + allowance."""
    assert got.shape == want.shape, (name, got.shape, want.shape)
    got64, want64 = got.astype(np.float64), want.astype(np.float64)
    tol = rtol * np.maximum(np.abs(want64), floor) + allowance + 2 * FP32_SUBNORMAL_STEP
    err = np.abs(got64 - want64)
    viol = err > tol
    if viol.any():
        idx = np.argwhere(viol)[:5]
        lines = [f"{tuple(int(x) for x in k)}: gpu={got64[tuple(k)]!r} oracle={want64[tuple(k)]!r} tol={tol[tuple(k)]:.3e}"
                 for k in idx]
        raise AssertionError(f"{name}: {int(viol.sum())} of {viol.size} elements outside tolerance; first: " + "; ".join(lines))
    # how much of the comparison ran at the plain spec tolerance
    return float((allowance > rtol * np.maximum(np.abs(want64), floor)).mean())


def check_scores(got, want, s64, r64, d64, score):
    """|gpu - oracle| <= 1e-5 * max(|oracle|, ||u|| ||d||): norm-wise bound of a dot product
    (translational score: 1e-5 * (|u|_1 + |d|_1), the same bound for a sum of distances)."""
    u = model.compose_u(score, s64, r64)
    if score == model.TRANSE:
        bound = np.abs(u).sum(axis=1) + np.abs(d64).sum(axis=1)
    else:
        bound = np.linalg.norm(u, axis=1) * np.linalg.norm(d64, axis=1)
    tol = 1e-5 * np.maximum(np.abs(want), bound)
    err = np.abs(got.astype(np.float64) - want)
    assert (err <= tol).all(), f"score mismatch: max err {err.max():.3e}, worst tol {tol[err.argmax()]:.3e}"
