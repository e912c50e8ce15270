"""Pins for the oracle's scores, loss and gradients (Eq. 1, Sec. 6 operator structure)."""

import itertools

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import model, negatives
from oracle.bucket import OracleConfig, Tables, batch_gradients


# ---------------------------------------------------------------- scores

def test_closed_form_scores_on_three_node_graph():
    # d = 2, integer-valued rows: every product is exact.
    a, b, c = np.array([[1., 2.]]), np.array([[3., -1.]]), np.array([[-2., 5.]])
    r = np.array([[2., 3.]])
    assert model.positive_scores(model.DOT, a, None, b)[0] == 1 * 3 + 2 * -1
    assert model.positive_scores(model.DISTMULT, a, r, c)[0] == 1 * 2 * -2 + 2 * 3 * 5
    # ComplEx with one complex component: a = 1+2i, r = 2+3i, c = -2+5i, Re(a r conj(c))
    want = ((1 + 2j) * (2 + 3j) * np.conj(-2 + 5j)).real
    assert model.positive_scores(model.COMPLEX, a, r, c)[0] == want == 43.0


def test_complex_matches_numpy_complex_arithmetic():
    rng = np.random.default_rng(0)
    h = 5
    s, r, d = (rng.standard_normal((7, 2 * h)) for _ in range(3))
    cs, cr, cd = (x[:, :h] + 1j * x[:, h:] for x in (s, r, d))
    want = np.real(np.sum(cs * cr * np.conj(cd), axis=1))
    np.testing.assert_allclose(model.positive_scores(model.COMPLEX, s, r, d), want, rtol=1e-13, atol=1e-13)
    # u = s*r, v = conj(r)*d as complex numbers
    u = model.compose_u(model.COMPLEX, s, r)
    v = model.compose_v(model.COMPLEX, r, d)
    np.testing.assert_allclose(u[:, :h] + 1j * u[:, h:], cs * cr, rtol=1e-13)
    np.testing.assert_allclose(v[:, :h] + 1j * v[:, h:], np.conj(cr) * cd, rtol=1e-13)


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.COMPLEX])
def test_u_dot_d_equals_s_dot_v(score):
    rng = np.random.default_rng(1)
    s, r, d = (rng.standard_normal((9, 8)) for _ in range(3))
    u = model.compose_u(score, s, r)
    v = model.compose_v(score, r, d)
    np.testing.assert_allclose(np.sum(u * d, 1), np.sum(s * v, 1), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.COMPLEX])
def test_negative_block_is_the_score_of_the_corrupted_triple(score):
    rng = np.random.default_rng(2)
    s, r, d = (rng.standard_normal((4, 6)) for _ in range(3))
    negs = rng.standard_normal((5, 6))
    out_d = model.chunk_side(score, model.SOFTMAX, 1.0, True, s, r, d, negs)
    out_s = model.chunk_side(score, model.SOFTMAX, 1.0, False, s, r, d, negs)
    for e, k in itertools.product(range(4), range(5)):
        f_d = model.positive_scores(score, s[e:e + 1], r[e:e + 1], negs[k:k + 1])[0]
        f_s = model.positive_scores(score, negs[k:k + 1], r[e:e + 1], d[e:e + 1])[0]
        assert abs(out_d["S"][e, k] - f_d) < 1e-12
        assert abs(out_s["S"][e, k] - f_s) < 1e-12


# ---------------------------------------------------------------- loss

def test_softmax_single_and_double_negative_closed_forms():
    f = np.array([0.25, -1.0])
    S = np.array([[0.75], [2.0]])
    l, a, W = model.side_loss(model.SOFTMAX, f, S, 1.0)
    np.testing.assert_allclose(l, S[:, 0] - f, rtol=0, atol=1e-15)
    assert (W == 1.0).all() and (a == -1.0).all()
    S2 = np.repeat(S, 2, axis=1)
    l2, _, W2 = model.side_loss(model.SOFTMAX, f, S2, 1.0)
    np.testing.assert_allclose(l2, S[:, 0] - f + np.log(2.0), atol=1e-15)
    np.testing.assert_allclose(W2, 0.5, atol=1e-15)


def test_softmax_matches_scipy_and_is_shift_invariant():
    rng = np.random.default_rng(3)
    f = rng.standard_normal(6)
    S = 5 * rng.standard_normal((6, 11))
    l, _, W = model.side_loss(model.SOFTMAX, f, S, 1.0)
    np.testing.assert_allclose(l, -f + logsumexp(S, axis=1), rtol=1e-13)
    np.testing.assert_allclose(W.sum(1), 1.0, rtol=1e-13)
    l3, _, W3 = model.side_loss(model.SOFTMAX, f, S + 3.5, 1.0)
    np.testing.assert_allclose(l3, l + 3.5, rtol=1e-12)
    np.testing.assert_allclose(W3, W, rtol=1e-12)
    # large scores do not overflow
    lbig, _, _ = model.side_loss(model.SOFTMAX, f, S + 800.0, 1.0)
    assert np.isfinite(lbig).all()


def test_logistic_closed_forms():
    f = np.array([0.0, 2.0])
    S = np.array([[0.0, 0.0], [-1.0, 3.0]])
    l, a, W = model.side_loss(model.LOGISTIC, f, S, 0.5)
    sp = lambda x: np.log1p(np.exp(x))
    np.testing.assert_allclose(l, sp(-f) + 0.5 * sp(S).sum(1), rtol=1e-13)
    np.testing.assert_allclose(a, -1 / (1 + np.exp(f)), rtol=1e-13)
    np.testing.assert_allclose(W, 0.5 / (1 + np.exp(-S)), rtol=1e-13)
    assert abs(l[0] - (np.log(2) + np.log(2))) < 1e-14


def test_logistic_coefficients_keep_their_precision_for_very_negative_scores():
    # sigmoid(x) = e^x (1 - e^x + ...) for x << 0: a distance-based score of -50 must not turn into weight 0
    f = np.array([-60.0])
    S = np.array([[-50.0, -37.0, -20.0, 0.0]])
    l, a, W = model.side_loss(model.LOGISTIC, f, S, 0.5)
    want = 0.5 * np.exp(S) / (1.0 + np.exp(S))
    np.testing.assert_allclose(W, want, rtol=1e-14)
    assert W[0, 0] > 0 and abs(W[0, 0] / (0.5 * np.exp(-50.0)) - 1.0) < 1e-15
    np.testing.assert_allclose(a, -1.0 / (1.0 + np.exp(-60.0)), rtol=1e-15)
    # softplus(60) + 0.5 * sum softplus(S)
    np.testing.assert_allclose(l, 60.0 + np.log1p(np.exp(-60.0)) + 0.5 * np.log1p(np.exp(S)).sum(), rtol=1e-15)


def test_softmax_with_positive_closed_forms_and_library_cross_entropy():
    # one negative scoring exactly like the positive: two equal logits
    l, a, W = model.side_loss(model.SOFTMAX_POS, np.array([0.3]), np.array([[0.3]]), 1.0)
    assert abs(l[0] - np.log(2.0)) < 1e-15 and abs(a[0] + 0.5) < 1e-15 and abs(W[0, 0] - 0.5) < 1e-15
    # a hopeless negative: loss -> 0, nothing to learn
    l, a, W = model.side_loss(model.SOFTMAX_POS, np.array([50.0]), np.array([[-50.0]]), 1.0)
    assert l[0] < 1e-40 + np.exp(-100.0) * 1.01 and abs(a[0]) < 1e-40 and W[0, 0] < 1e-40
    # a dominating positive: dl/df = -r / (1 + r) with r = sum_k e^(S_k - f) tiny; evaluated as -1 + e^f / z
    # it would keep two digits of r = 2e-14
    l, a, W = model.side_loss(model.SOFTMAX_POS, np.array([30.0]), np.array([[-2.0, -5.0]]), 1.0)
    r = np.exp(-32.0) + np.exp(-35.0)
    assert abs(a[0] / (-r / (1.0 + r)) - 1.0) < 1e-14 and abs(a[0] + W.sum()) < 1e-28
    # torch's cross entropy over the logits [f, S_1..S_N] with class 0 as the target
    rng = np.random.default_rng(3)
    f, S = rng.standard_normal(5) * 3, rng.standard_normal((5, 9)) * 3
    l, a, W = model.side_loss(model.SOFTMAX_POS, f, S, 1.0)
    logits = torch.tensor(np.concatenate([f[:, None], S], 1), requires_grad=True)
    ce = torch.nn.functional.cross_entropy(logits, torch.zeros(5, dtype=torch.long), reduction="none")
    np.testing.assert_allclose(l, ce.detach().numpy(), rtol=1e-13)
    ce.sum().backward()
    np.testing.assert_allclose(a, logits.grad[:, 0].numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(W, logits.grad[:, 1:].numpy(), rtol=1e-12, atol=1e-15)
    # overflow-free for large scores of either sign
    l, a, W = model.side_loss(model.SOFTMAX_POS, f + 900.0, S + 900.0, 1.0)
    np.testing.assert_allclose(l, ce.detach().numpy(), rtol=1e-10)
    # the coefficients of a row sum to zero: a + sum_k W_k = 0
    np.testing.assert_allclose(a + W.sum(1), 0.0, atol=1e-15)


def test_margin_ranking_loss_closed_forms_and_library_margin_ranking_loss():
    # one negative: it pays margin - f + S when it is less than the margin below the positive, else nothing
    l, a, W = model.side_loss(model.MARGIN, np.array([0.3]), np.array([[0.1]]), 1.0, margin=1.0)
    assert l[0] == pytest.approx(0.8) and a[0] == -1.0 and W[0, 0] == 1.0
    l, a, W = model.side_loss(model.MARGIN, np.array([2.0]), np.array([[0.5]]), 1.0, margin=1.0)
    assert l[0] == 0.0 and a[0] == 0.0 and W[0, 0] == 0.0
    l, a, W = model.side_loss(model.MARGIN, np.array([1.5]), np.array([[0.5]]), 1.0, margin=1.0)      # on the hinge itself
    assert l[0] == 0.0 and a[0] == 0.0 and W[0, 0] == 0.0
    # several: only the violators count, dl/df is minus their number
    l, a, W = model.side_loss(model.MARGIN, np.array([1.0, -1.0]), np.array([[0.5, -3.0, 0.9], [4.0, -2.5, -1.75]]), 1.0, margin=0.5)
    np.testing.assert_allclose(l, [0.0 + 0.0 + 0.4, 5.5 + 0.0 + 0.0])
    np.testing.assert_array_equal(W, [[0, 0, 1], [1, 0, 0]])
    np.testing.assert_array_equal(a, [-1, -1])
    # the library's pairwise ranking loss: max(0, -y (x1 - x2) + margin) with y = 1, x1 the positive, x2 a negative
    rng = np.random.default_rng(8)
    f, S = rng.standard_normal(7), rng.standard_normal((7, 11))
    tf = torch.tensor(f, requires_grad=True)
    tS = torch.tensor(S, requires_grad=True)
    lib = torch.nn.functional.margin_ranking_loss(tf[:, None].expand(7, 11), tS, torch.ones(7, 11, dtype=torch.float64),
                                                  margin=0.7, reduction="none")
    l, a, W = model.side_loss(model.MARGIN, f, S, 1.0, margin=0.7)
    np.testing.assert_allclose(l, lib.sum(1).detach().numpy(), rtol=1e-14)
    lib.sum().backward()
    np.testing.assert_allclose(a, tf.grad.numpy(), rtol=0, atol=0)
    np.testing.assert_allclose(W, tS.grad.numpy(), rtol=0, atol=0)


# ---------------------------------------------------------------- gradients

def _tiny(score, loss, corrupt, i, j, seed=0, degree_negs=0):
    cfg = OracleConfig(num_nodes=8, num_relations=3 if score else 0, dim=6, num_partitions=2,
                       batch_size=5, chunk_size=2, num_negs=3, num_degree_negs=degree_negs,
                       score=score, loss=loss, corrupt=corrupt, seed=seed, neg_weight=0.4)
    rng = np.random.default_rng(seed + 10)
    node = (0.7 * rng.standard_normal((8, 6))).astype(np.float32)
    rel = (0.7 * rng.standard_normal((3, 6))).astype(np.float32)
    edges = np.stack([rng.integers(0, 4, 5), rng.integers(0, 3, 5), rng.integers(0, 4, 5)], 1).astype(np.int32)
    return cfg, node, rel, edges


def _loss_only(cfg, node, rel, edges, i, j):
    tab = Tables(cfg, node.astype(np.float32), rel)
    # tables hold float32; for differences work in float64 copies
    tab.E = [node[p * 4:(p + 1) * 4].astype(np.float64) for p in range(2)]
    tab.RE = rel.astype(np.float64)
    return batch_gradients(tab, i, j, edges, 0, 0)[0]


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.COMPLEX, model.TRANSE])
@pytest.mark.parametrize("loss", [model.SOFTMAX, model.LOGISTIC, model.SOFTMAX_POS, model.MARGIN])
@pytest.mark.parametrize("corrupt", [0, 1, 2])
@pytest.mark.parametrize("bucket", [(0, 0), (0, 1), (1, 0)])
def test_gradients_match_central_finite_differences(score, loss, corrupt, bucket):
    i, j = bucket
    cfg, node32, rel32, edges = _tiny(score, loss, corrupt, i, j, degree_negs=1)
    if loss == model.MARGIN:
        # the hinge has kinks; the differences below are taken away from them: no sampled negative of these
        # tables sits within 1e-3 of its hinge (checked), the step is 1e-6
        cfg.margin = 0.8
        shortfalls = []
        batch_gradients(Tables(cfg, node32, rel32), i, j, edges, 0, 0,
                        record={"observer": lambda si, dst, c, er, ids, s, r, d, negs, out:
                                shortfalls.append(cfg.margin - out["f"][:, None] + out["S"])})
        assert min(float(np.abs(x).min()) for x in shortfalls) > 1e-3
        assert any((x > 0).any() for x in shortfalls)
    # the translational u, v are exact here: the differences perturb below fp32 resolution.  Its
    # kinks (a component of u equal to that of a row it meets: a negative that is the edge's own
    # endpoint and a zero relation component) do not occur in these continuous random tables.
    cfg.round_composed = False
    node, rel = node32.astype(np.float64), rel32.astype(np.float64)
    tab = Tables(cfg, node32, rel32)
    _, gnode, grel = batch_gradients(tab, i, j, edges, 0, 0)
    dense = np.zeros_like(node)
    for slot, part in ((0, i), (1, j)):
        if slot in gnode:
            rows, g = gnode[slot]
            dense[part * 4 + rows] += g
    h = 1e-6
    fd = np.zeros_like(node)
    for idx in np.ndindex(*node.shape):
        up, dn = node.copy(), node.copy()
        up[idx] += h
        dn[idx] -= h
        fd[idx] = (_loss_only(cfg, up, rel, edges, i, j) - _loss_only(cfg, dn, rel, edges, i, j)) / (2 * h)
    np.testing.assert_allclose(dense, fd, rtol=2e-6, atol=2e-8)
    if score != model.DOT:
        drel = np.zeros_like(rel)
        drel[grel[0]] = grel[1]
        fdr = np.zeros_like(rel)
        for idx in np.ndindex(*rel.shape):
            up, dn = rel.copy(), rel.copy()
            up[idx] += h
            dn[idx] -= h
            fdr[idx] = (_loss_only(cfg, node, up, edges, i, j) - _loss_only(cfg, node, dn, edges, i, j)) / (2 * h)
        np.testing.assert_allclose(drel, fdr, rtol=2e-6, atol=2e-8)
    else:
        assert grel is None


@pytest.mark.parametrize("score", [model.DOT, model.COMPLEX])
def test_margin_gradients_match_autograd_on_the_pairwise_hinge_written_edge_by_edge(score):
    i, j = 1, 0
    cfg, node32, rel32, edges = _tiny(score, model.MARGIN, 2, i, j, seed=6)
    cfg.margin = 0.6
    tab = Tables(cfg, node32, rel32)
    loss, gnode, grel = batch_gradients(tab, i, j, edges, 0, 0)
    neg = negatives.batch_negatives(cfg, 0, i, j, 0, edges, edges)
    tn = torch.tensor(node32, dtype=torch.float64, requires_grad=True)
    tr = torch.tensor(rel32, dtype=torch.float64, requires_grad=True)
    total = torch.zeros((), dtype=torch.float64)
    for e_idx, (sl, rl, dl) in enumerate(edges):
        c = e_idx // cfg.chunk_size
        s, r, d = tn[i * 4 + sl], tr[rl], tn[j * 4 + dl]
        f = _torch_score(score, s, r, d)
        for k in neg[0, c]:
            total = total + torch.clamp(cfg.margin - f + _torch_score(score, s, r, tn[j * 4 + int(k)]), min=0.0)
        for k in neg[1, c]:
            total = total + torch.clamp(cfg.margin - f + _torch_score(score, tn[i * 4 + int(k)], r, d), min=0.0)
    total.backward()
    assert float(total) > 0 and abs(float(total) - loss) < 1e-10
    kinds = []
    batch_gradients(Tables(cfg, node32, rel32), i, j, edges, 0, 0,
                    record={"observer": lambda si, dst, c, er, ids, s, r, d, negs, out: kinds.append(out["W"])})
    assert any((w == 1).any() for w in kinds) and any((w == 0).any() for w in kinds)      # violators and satisfied pairs
    dense = np.zeros((8, 6))
    for slot, part in ((0, i), (1, j)):
        if slot in gnode:
            rows, g = gnode[slot]
            dense[part * 4 + rows] += g
    np.testing.assert_allclose(dense, tn.grad.numpy(), rtol=1e-10, atol=1e-12)
    if score != model.DOT:
        drel = np.zeros((3, 6))
        drel[grel[0]] = grel[1]
        np.testing.assert_allclose(drel, tr.grad.numpy(), rtol=1e-10, atol=1e-12)


def _torch_score(score, s, r, d):
    if score == model.DOT:
        return (s * d).sum(-1)
    if score == model.DISTMULT:
        return (s * r * d).sum(-1)
    if score == model.TRANSE:
        return -(s + r - d).abs().sum(-1)
    h = s.shape[-1] // 2
    cs, cr, cd = (torch.complex(x[..., :h], x[..., h:]) for x in (s, r, d))
    return (cs * cr * torch.conj(cd)).real.sum(-1)


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.COMPLEX, model.TRANSE])
@pytest.mark.parametrize("bucket", [(0, 0), (1, 0)])
def test_gradients_match_autograd_on_eq1_written_edge_by_edge(score, bucket):
    # Eq. 1 with the sampled negatives, written per positive edge and per
    # corrupted triple with no shared intermediates, differentiated by autograd.
    i, j = bucket
    cfg, node32, rel32, edges = _tiny(score, model.SOFTMAX, 2, i, j, seed=4)
    cfg.round_composed = False            # autograd forms s + r - d in float64
    tab = Tables(cfg, node32, rel32)
    loss, gnode, grel = batch_gradients(tab, i, j, edges, 0, 0)
    neg = negatives.batch_negatives(cfg, 0, i, j, 0, edges, edges)

    tn = torch.tensor(node32, dtype=torch.float64, requires_grad=True)
    tr = torch.tensor(rel32, dtype=torch.float64, requires_grad=True)
    total = torch.zeros((), dtype=torch.float64)
    for e_idx, (sl, rl, dl) in enumerate(edges):
        c = e_idx // cfg.chunk_size
        s, r, d = tn[i * 4 + sl], tr[rl], tn[j * 4 + dl]
        f = _torch_score(score, s, r, d)
        dst_negs = torch.stack([_torch_score(score, s, r, tn[j * 4 + int(k)]) for k in neg[0, c]])
        src_negs = torch.stack([_torch_score(score, tn[i * 4 + int(k)], r, d) for k in neg[1, c]])
        total = total - (f - torch.logsumexp(dst_negs, 0)) - (f - torch.logsumexp(src_negs, 0))
    total.backward()
    assert abs(float(total) - loss) < 1e-10
    dense = np.zeros((8, 6))
    for slot, part in ((0, i), (1, j)):
        if slot in gnode:
            rows, g = gnode[slot]
            dense[part * 4 + rows] += g
    np.testing.assert_allclose(dense, tn.grad.numpy(), rtol=1e-10, atol=1e-12)
    if score != model.DOT:
        drel = np.zeros((3, 6))
        drel[grel[0]] = grel[1]
        np.testing.assert_allclose(drel, tr.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_softmax_gradient_invariants():
    rng = np.random.default_rng(5)
    s, r, d = (rng.standard_normal((4, 6)) for _ in range(3))
    negs = rng.standard_normal((7, 6))
    out = model.chunk_side(model.DISTMULT, model.SOFTMAX, 1.0, True, s, r, d, negs)
    u = s * r
    # sum_k W_ek = 1  =>  sum_k g_neg(k) = sum_e u_e
    np.testing.assert_allclose(out["g_neg"].sum(0), u.sum(0), rtol=1e-12)
    # g_u + d lies in the convex hull of the negatives: coefficients W >= 0 summing to 1
    g_u = out["W"] @ negs - d
    np.testing.assert_allclose(g_u + d, out["W"] @ negs, rtol=1e-12)
    assert (out["W"] >= 0).all()
    # g_d = -u for Eq. 1
    np.testing.assert_allclose(out["g_d"], -u, rtol=1e-15)


# ---------------------------------------------------------------- translational score

def test_translational_closed_forms():
    # d = 2, integers: s + r = (3, 1); f = -(|3-1| + |1-4|) = -5
    s, r, d = np.array([[1.0, 2.0]]), np.array([[2.0, -1.0]]), np.array([[1.0, 4.0]])
    assert model.positive_scores(model.TRANSE, s, r, d)[0] == -5.0
    # u meets d (destination side), s meets v = d - r (source side): the same number
    assert -np.abs(s - model.compose_v(model.TRANSE, r, d)).sum() == -5.0
    negs = np.array([[3.0, 1.0], [0.0, 0.0], [5.0, 1.0]])            # distances 0, 4, 2 from u
    out = model.chunk_side(model.TRANSE, model.SOFTMAX, 1.0, True, s, r, d, negs)
    np.testing.assert_array_equal(out["S"], [[0.0, -4.0, -2.0]])
    W = np.exp([0.0, -4.0, -2.0]) / np.exp([0.0, -4.0, -2.0]).sum()
    np.testing.assert_allclose(out["W"][0], W, rtol=1e-15)
    # d(-|u - n|)/dn = sign(u - n): (0,0) for the negative equal to u, (+,+) for the origin, (-,0) for (5,1)
    np.testing.assert_allclose(out["g_neg"], [[0, 0], [W[1], W[1]], [-W[2], 0]], rtol=1e-15)
    # Eq. 1: a = -1, d f/du = -sign(u - d) = (-1, +1); negatives pull u towards themselves
    want_gu = np.array([1.0, -1.0]) - (W[1] * np.array([1, 1]) + W[2] * np.array([-1, 0]))
    np.testing.assert_allclose(out["g_s"][0], want_gu, rtol=1e-15)
    np.testing.assert_allclose(out["g_r"][0], want_gu, rtol=1e-15)
    np.testing.assert_allclose(out["g_d"][0], [-1.0, 1.0], rtol=1e-15)   # a * sign(u - d)
    # source side: v = d - r = (-1, 5); the relation gradient changes sign
    out = model.chunk_side(model.TRANSE, model.SOFTMAX, 1.0, False, s, r, d, negs)
    np.testing.assert_allclose(out["g_r"], -out["g_d"], rtol=0, atol=0)


def test_translational_negative_block_is_the_score_of_the_corrupted_triple_and_scipy_cityblock():
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(12)
    s, r, d = (rng.standard_normal((4, 6)).astype(np.float32).astype(np.float64) for _ in range(3))
    negs = rng.standard_normal((5, 6)).astype(np.float32).astype(np.float64)
    out_d = model.chunk_side(model.TRANSE, model.SOFTMAX, 1.0, True, s, r, d, negs)
    out_s = model.chunk_side(model.TRANSE, model.SOFTMAX, 1.0, False, s, r, d, negs)
    for e, k in itertools.product(range(4), range(5)):
        assert out_d["S"][e, k] == model.positive_scores(model.TRANSE, s[e:e + 1], r[e:e + 1], negs[k:k + 1])[0]
        # source side through v = d - r: |n + r - d| and |n - fl(d - r)| agree to fp32 rounding of v
        f_s = model.positive_scores(model.TRANSE, negs[k:k + 1], r[e:e + 1], d[e:e + 1], rounded=False)[0]
        assert abs(out_s["S"][e, k] - f_s) < 1e-6
    u = model.compose_u(model.TRANSE, s, r)
    np.testing.assert_allclose(-out_d["S"], cdist(u, negs, metric="cityblock"), rtol=1e-14)
    # the composed operands are fp32 numbers, within half an ulp of the exact sums
    assert (u == u.astype(np.float32)).all() and np.abs(u - (s + r)).max() <= 2.0 ** -24 * np.abs(s + r).max()
