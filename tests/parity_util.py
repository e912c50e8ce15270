"""Shared helpers of the GPU parity tests (oracle side + comparison rules)."""

from __future__ import annotations

import numpy as np

import os

from oracle import model
from oracle.bucket import OracleConfig, Tables, train_batch
from tests.error_model import BatchMagnitudes

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
# The error of an fp32 dot product grows with the square root of its length: KAPPA (below) holds
# up to dim 128 and grows like sqrt(dim / 128) beyond (x1.41 at 256, x1.77 at 400, x2 at 512).
# Softmax weights and dl/df are functions of score differences and inherit the absolute error of the
# fp32 scores, which scales with A = sum_j |q_j| |theta_j| and not with the score: the error model
# (tests/error_model.py) widens their magnitudes by (1 + max A / 4) per row (8 roundoffs times A; 1.25 at the benchmark workloads'
# initial scale, two orders of magnitude once scores reach the hundreds), and the batch loss is allowed
# KAPPA * sum_e max A_e / 4 beside its 1e-5 relative bound.  For the translational score the same role
# is played by max |S| dim / 128.
# Below the normal range of fp32 (2^-126) results are spaced 2^-149 apart and a relative bound means
# nothing: every comparison allows two such steps on top.
EMB_RTOL = 1e-5
STATE_RTOL = 3e-5
# KAPPA, in roundoffs of 2^-24, is set from measurement with a factor of two of headroom: over every GPU parity
# case of this repository (the table the test run prints: column "allow. used" is the largest share of the
# allowance that any element outside the plain bound needed) the embedding tables used at most 5.3 roundoffs
# times M, the optimiser-state tables 15.4 (both in one case: ComplEx, d = 128, scores in the thousands); at the
# full-size workloads 1.5 and 2.2.  The atomic update mode stays inside the same allowance (0.8 / 9.2 roundoffs
# measured).  No batch loss of a committed case left its plain 1e-5 bound; its allowance (needed by randomised
# sweeps with initial standard deviations up to 4, scores of several hundred) is kept at 8 roundoffs.
KAPPA_EMB = 12 * 2.0 ** -24
KAPPA_STATE = 32 * 2.0 ** -24
KAPPA_LOSS = 8 * 2.0 ** -24
FP32_SUBNORMAL_STEP = 2.0 ** -149


def _dim_growth(dim: int) -> float:
    return max(1.0, (dim / 128.0) ** 0.5)


def kappa_for(dim: int, what: str = "state") -> float:
    return {"emb": KAPPA_EMB, "state": KAPPA_STATE, "loss": KAPPA_LOSS}[what] * _dim_growth(dim)


class OracleRun:
    """Trains batches with the oracle and accumulates the forward-error allowance per element
    (the allowance comes from tests/error_model.py, which watches the oracle's chunks; the oracle
    itself computes the method only).

    sparse=True keeps no dense per-partition allowance arrays: after each train_bucket call
    `last` maps a partition (or "rel") to (rows, allowance on embeddings, allowance on state) of
    the rows the call's LAST batch touched -- for tables too large to shadow three times."""

    def __init__(self, cfg: OracleConfig, node: np.ndarray, rel, sparse: bool = False, tables: Tables = None):
        self.cfg = cfg
        self.tab = tables if tables is not None else Tables(cfg, node, rel)
        self.sparse = sparse
        rp, d = cfg.rows_per_partition, cfg.dim
        n = cfg.num_partitions
        if not sparse:
            self.fe_node = [np.zeros((rp, d)) for _ in range(n)]      # allowance on embeddings
            self.fs_node = [np.zeros((rp, d)) for _ in range(n)]      # allowance on optimiser state
            self.touched_node = [np.zeros(rp, bool) for _ in range(n)]
        self.fe_rel = np.zeros(self.tab.RE.shape)
        self.fs_rel = np.zeros(self.tab.RE.shape)
        self.touched_rel = np.zeros(self.tab.RE.shape[0], bool)
        self.last = {}
        self.loss = 0.0

    def _allowances(self, state, rows, g, mag, band=None):
        """band: magnitude of gradient terms that may be present or absent as a whole (discrete decisions that
        fall either way within rounding, tests/error_model.py); it enters unscaled."""
        lr, eps = self.cfg.lr, self.cfg.eps
        s_new = state[rows].astype(np.float64)               # after the update
        ke, ks = kappa_for(self.cfg.dim, "emb"), kappa_for(self.cfg.dim, "state")
        ee = ke * mag + (band if band is not None else 0.0)
        es = ks * mag + (band if band is not None else 0.0)
        fe = lr * ee / (np.sqrt(s_new) + eps)
        fs = 2.0 * np.abs(g) * es + es ** 2                          # |(G + e)^2 - G^2| <= 2 |G| e + e^2
        return fe, fs

    def set_state(self, node_E, node_S, rel_E=None, rel_S=None):
        """Restart from given tables (global node order) and clear the allowances."""
        cfg = self.cfg
        rp = cfg.rows_per_partition
        for p in range(cfg.num_partitions):
            lo, hi = p * rp, min(cfg.num_nodes, (p + 1) * rp)
            self.tab.E[p][: hi - lo] = node_E[lo:hi]
            self.tab.S[p][: hi - lo] = node_S[lo:hi]
            if not self.sparse:
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
            watch = BatchMagnitudes(cfg.score, i == j, cfg.loss, cfg.margin)
            rec = {"observer": watch}
            loss += train_batch(self.tab, i, j, edges, b, epoch, record=rec)
            self.last_loss_allowance += kappa_for(cfg.dim, "loss") * watch.loss_magnitude
            node, rel = rec["grads"]
            mags = watch.coalesced()
            self.last = {}
            for slot, part in ((0, i), (1, j)):
                if slot in node:
                    rows, g = node[slot]
                    mrows, mag, band = mags[slot]
                    assert np.array_equal(rows, mrows)
                    fe, fs = self._allowances(self.tab.S[part], rows, g, mag, band)
                    if self.sparse:
                        self.last[part] = (rows, fe, fs)
                    else:
                        self.fe_node[part][rows] += fe
                        self.fs_node[part][rows] += fs
                        self.touched_node[part][rows] = True
            if rel is not None:
                rows, g = rel
                mrows, mag, band = mags[2]
                assert np.array_equal(rows, mrows)
                fe, fs = self._allowances(self.tab.RS, rows, g, mag, band)
                self.fe_rel[rows] += fe
                self.fs_rel[rows] += fs
                self.touched_rel[rows] = True
        self.loss += loss
        return loss

    def node_allowance(self, which):
        src = self.fe_node if which == 0 else self.fs_node
        return np.concatenate(src, 0)[: self.cfg.num_nodes]


# Every comparison leaves a record here; tests/conftest.py prints the table at the end of the run
# (and writes it to gpurun_out/parity_stats.json when that folder exists): how much of each comparison
# ran at the plain spec bound, and how much of the allowance the rest needed.
STATS = []


def compare_table(name, got, want, allowance, rtol, floor, untested_above=None, kind=None):
    """Element-wise comparison: |got - want| <= rtol * max(|want|, floor) + allowance.

    Returns the comparison's statistics (also appended to STATS):
      n                 elements compared
      share_plain       share of them inside the plain bound rtol * max(|want|, floor) (the spec bar)
      max_err_over_plain
      allowance_used    largest (err - plain) / allowance over the elements outside the plain bound:
                        the share of the allowance (hence of KAPPA) that this comparison needed
      share_allowance_dominant   share of elements whose allowance exceeds their plain bound
      share_untested    share of elements whose allowance exceeds `untested_above` (for embeddings: the learning
                        rate, the size of a whole Adagrad step -- such an element passes whatever its value)"""
    assert got.shape == want.shape, (name, got.shape, want.shape)
    got64, want64 = got.astype(np.float64), want.astype(np.float64)
    plain = rtol * np.maximum(np.abs(want64), floor) + 2 * FP32_SUBNORMAL_STEP
    tol = plain + allowance
    err = np.abs(got64 - want64)
    viol = err > tol
    if viol.any():
        idx = np.argwhere(viol)[:5]
        lines = [f"{tuple(int(x) for x in k)}: gpu={got64[tuple(k)]!r} oracle={want64[tuple(k)]!r} tol={tol[tuple(k)]:.3e}"
                 for k in idx]
        raise AssertionError(f"{name}: {int(viol.sum())} of {viol.size} elements outside tolerance; first: " + "; ".join(lines))
    beyond = err > plain
    allow = np.broadcast_to(np.asarray(allowance, np.float64), err.shape)
    used = float(((err[beyond] - plain[beyond]) / allow[beyond]).max()) if beyond.any() else 0.0
    st = dict(name=name, kind=kind or ("state" if floor == 0.0 else "emb"), n=int(err.size),
              share_plain=float(1.0 - beyond.mean()) if err.size else 1.0,
              max_err_over_plain=float((err / plain).max()) if err.size else 0.0,
              allowance_used=used,
              share_allowance_dominant=float((allow > plain).mean()) if err.size else 0.0,
              share_untested=float((allow > untested_above).mean()) if (untested_above is not None and err.size) else 0.0,
              test=os.environ.get("PYTEST_CURRENT_TEST", "").split(" ")[0])
    STATS.append(st)
    return st


def check_loss(name, got, want, allowance, rtol=1e-5):
    """Batch (or bucket) loss: |got - want| <= rtol * |want| + allowance; records how much of the allowance was used."""
    err = abs(got - want)
    plain = rtol * abs(want)
    assert err <= plain + allowance, (name, got, want, allowance)
    used = (err - plain) / allowance if (err > plain and allowance > 0) else 0.0
    STATS.append(dict(name=name, kind="loss", n=1, share_plain=1.0 if err <= plain else 0.0,
                      max_err_over_plain=err / plain if plain > 0 else 0.0, allowance_used=used,
                      share_allowance_dominant=1.0 if allowance > plain else 0.0, share_untested=0.0,
                      test=os.environ.get("PYTEST_CURRENT_TEST", "").split(" ")[0]))


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
