"""Pins of the ranking oracle (Sec. 7 "Metrics": MRR, Hits@k): a hand-worked example,
scipy's rankdata, numpy complex arithmetic, closed forms."""

import numpy as np
import pytest
from scipy.stats import rankdata

from oracle import model, rank


def test_hand_worked_example_dot():
    # five nodes in the plane; triple (4 -> 0): f = <(1,1), (1,0)> = 1
    E = np.array([[1, 0], [2, 0], [0, 5], [1, 0], [1, 1]], dtype=np.float64)
    src, dst = np.array([4]), np.array([0])
    # candidates replace the destination: scores 1 (true, left out), 2, 5, 1, 2
    g, q = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, None)
    assert (g[0], q[0]) == (3, 1)
    assert rank.ranks_from_counts(g, q)[0] == 4.5
    # candidates replace the source: <c, (1,0)> = 1, 2, 0, 1, 1(true, left out)
    g, q = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_SRC, None)
    assert (g[0], q[0]) == (1, 2)
    # an explicit candidate list; the true endpoint is skipped when it is listed, duplicates count twice
    g, q = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, [0, 2, 2, 3])
    assert (g[0], q[0]) == (2, 1)


def test_metrics_closed_form():
    m = rank.metrics_from_ranks([1, 2, 4])
    assert m["mrr"] == pytest.approx((1 + 0.5 + 0.25) / 3, rel=1e-15)
    assert m["hits1"] == pytest.approx(1 / 3) and m["hits3"] == pytest.approx(2 / 3) and m["hits10"] == 1.0
    assert rank.metrics_from_ranks([1.5])["hits1"] == 0.0     # a tie for first place is not a hit at 1


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.COMPLEX])
@pytest.mark.parametrize("side", [rank.SIDE_DST, rank.SIDE_SRC])
def test_against_rankdata_with_ties(score, side):
    # small integer embeddings: every score is exact, ties are frequent
    rng = np.random.default_rng(10 * score + side)
    V, R, d, m = 40, 3, 4, 25
    E = rng.integers(-2, 3, size=(V, d)).astype(np.float64)
    Rl = rng.integers(-2, 3, size=(R, d)).astype(np.float64)
    src, dst, rel = rng.integers(0, V, m), rng.integers(0, V, m), rng.integers(0, R, m)
    g, q = rank.rank_counts(score, E, Rl, src, rel, dst, side, None)
    assert q.sum() > 0
    for e in range(m):
        # the library's average rank of the true endpoint among all nodes, by descending score
        if side == rank.SIDE_DST:
            f = np.array([model.positive_scores(score, E[src[e]], Rl[rel[e]], E[c]) for c in range(V)])
            true_id = dst[e]
        else:
            f = np.array([model.positive_scores(score, E[c], Rl[rel[e]], E[dst[e]]) for c in range(V)])
            true_id = src[e]
        want = rankdata(-f, method="average")[true_id]
        assert rank.ranks_from_counts(g, q)[e] == want


def test_complex_candidates_against_numpy_complex():
    rng = np.random.default_rng(3)
    V, d = 30, 6
    h = d // 2
    E = rng.normal(size=(V, d))
    Rl = rng.normal(size=(2, d))
    z = E[:, :h] + 1j * E[:, h:]
    zr = Rl[:, :h] + 1j * Rl[:, h:]
    s, r, t = 4, 1, 7
    want_dst = np.real(np.sum(z[s] * zr[r] * np.conj(z), axis=1))
    want_src = np.real(np.sum(z * zr[r] * np.conj(z[t]), axis=1))
    got_dst = rank.candidate_scores(model.COMPLEX, E, Rl, s, r, t, rank.SIDE_DST, np.arange(V))
    got_src = rank.candidate_scores(model.COMPLEX, E, Rl, s, r, t, rank.SIDE_SRC, np.arange(V))
    np.testing.assert_allclose(got_dst, want_dst, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(got_src, want_src, rtol=1e-13, atol=1e-13)
    assert not np.allclose(want_dst, want_src)


def test_invariants():
    rng = np.random.default_rng(5)
    V, d, m = 50, 8, 12
    E = rng.normal(size=(V, d))
    src, dst = rng.integers(0, V, m), rng.integers(0, V, m)
    cand = rng.permutation(V)[:30]
    g, q = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, cand)
    g2, q2 = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, cand[::-1])
    assert (g == g2).all() and (q == q2).all()                  # the order of candidates does not matter
    # a true endpoint far along theta_s outranks everything
    E2 = E.copy()
    E2[dst[0]] = 100.0 * E[src[0]]
    g3, _ = rank.rank_counts(model.DOT, E2, None, src[:1], None, dst[:1], rank.SIDE_DST, None)
    assert g3[0] == 0
    # the dead zone brackets the definition
    lo, _ = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, cand, band=0.05)
    hi_g, hi_q = rank.rank_counts(model.DOT, E, None, src, None, dst, rank.SIDE_DST, cand, band=0.05)
    assert (lo <= g).all() and (g + q <= hi_g + hi_q).all()
