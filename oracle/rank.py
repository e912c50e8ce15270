"""Link-prediction ranks, MRR and Hits@k (oracle; float64; test infrastructure).

The paper evaluates embeddings by Mean Reciprocal Rank and Hits@k over test edges
(Sec. 7, "Metrics") and does not print the protocol; the textbook one is written out
here.  A test triple (s, r, d) is scored with f(theta_s, theta_r, theta_d) (Sec. 2.1);
its corrupted endpoint is replaced by every candidate node in turn, each replacement is
scored with the same f, and the triple's rank is its position among them:

    greater = #{c in candidates, c != true endpoint : f(corrupted with c) >  f(true)}
    equal   = #{c in candidates, c != true endpoint : f(corrupted with c) == f(true)}
    rank    = 1 + greater + equal / 2          (ties split evenly)
    MRR     = mean(1 / rank),   Hits@k = mean(rank <= k)

No filtering of candidates that happen to be true edges (same stance as training,
Sec. 2.1 stage 2).  Every replacement is scored by the plain definition of f on the
corrupted triple: no matrix-product shortcut.
"""

from __future__ import annotations

import numpy as np

from . import model

SIDE_DST, SIDE_SRC = 0, 1


def candidate_scores(score, node_emb, rel_emb, s, r, d, side, cand):
    """f of the triple (s, r, d) with its `side` endpoint replaced by each node of `cand`."""
    E = np.asarray(node_emb, dtype=np.float64)
    rows = E[np.asarray(cand, dtype=np.int64)]
    rr = np.zeros(E.shape[1]) if rel_emb is None else np.asarray(rel_emb, dtype=np.float64)[r]
    if side == SIDE_DST:
        return model.positive_scores(score, E[s][None, :], rr[None, :], rows)
    return model.positive_scores(score, rows, rr[None, :], E[d][None, :])


def rank_counts(score, node_emb, rel_emb, src, rel, dst, side, cand, band=0.0):
    """greater / equal counts per triple.  With band > 0 the comparison is taken with a
    dead zone: greater counts f_c > f + band, equal counts |f_c - f| <= band (used by tests
    to bracket an fp32 implementation; band = 0 is the definition)."""
    E = np.asarray(node_emb, dtype=np.float64)
    cand = np.arange(E.shape[0], dtype=np.int64) if cand is None else np.asarray(cand, dtype=np.int64)
    m = len(src)
    greater = np.zeros(m, dtype=np.int64)
    equal = np.zeros(m, dtype=np.int64)
    for e in range(m):
        s, d = int(src[e]), int(dst[e])
        r = 0 if rel is None else int(rel[e])
        true_id = d if side == SIDE_DST else s
        f_true = candidate_scores(score, E, rel_emb, s, r, d, side, [true_id])[0]
        f_c = candidate_scores(score, E, rel_emb, s, r, d, side, cand)
        other = cand != true_id
        greater[e] = np.count_nonzero(other & (f_c > f_true + band))
        equal[e] = np.count_nonzero(other & (np.abs(f_c - f_true) <= band))
    return greater, equal


def ranks_from_counts(greater, equal):
    return 1.0 + np.asarray(greater, dtype=np.float64) + 0.5 * np.asarray(equal, dtype=np.float64)


def metrics_from_ranks(ranks, ks=(1, 3, 10)):
    ranks = np.asarray(ranks, dtype=np.float64)
    out = {"mrr": float(np.mean(1.0 / ranks)) if ranks.size else 0.0}
    for k in ks:
        out[f"hits{k}"] = float(np.mean(ranks <= k)) if ranks.size else 0.0
    return out
