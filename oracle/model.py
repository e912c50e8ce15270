"""Scores, loss and analytic gradients of one chunk (oracle; float64; test infrastructure).

Notation follows Sec. 6 of the paper: the score has the form
(theta_s (x) theta_r) (+) theta_d, with (+) an inner product for the
multiplication-based models, so the negative block of a chunk is one real matrix
product.  u = theta_s (x) theta_r is the paper's "Intermediate Result 1"; its
mirror for source-side corruption is v = conj(theta_r) (x) theta_d, so that
f = <u, theta_d> = <theta_s, v>.  Embeddings of dimension d hold ComplEx numbers
as [real half | imaginary half] (Sec. 6, "first half / last half").

A translational score (Sec. 8 of the paper names such models as easy to integrate;
the form is the textbook one) fits the same frame with (x) an addition and (+) a
negative L1 distance: u = theta_s + theta_r, v = theta_d - theta_r,
f = -|u - theta_d|_1 = -|theta_s - v|_1; the negative block is then no matrix
product.  Its gradient is a sum of signs, a discrete decision: u and v are rounded to
fp32 (the storage precision, one IEEE addition of two fp32 numbers, so every
implementation gets the same u and v), after which the sign of u_j - n_j is exact in
any precision; sign(0) = 0.

Loss: Eq. 1 as printed (the log-sum-exp runs over the sampled negatives only),
the variant of Eq. 1 whose log-sum-exp also contains the positive score (the
usual sampled softmax / cross-entropy; not the paper's default), a logistic
loss, or a margin-based ranking loss (Sec. 8 says other objectives fit the same
frame and names none; the textbook pairwise hinge is used):
    l_e = sum_k max(0, margin - f_e + S_ek),
every sampled negative that is not at least `margin` below the positive pays for
the shortfall.  Its derivative is an indicator: dl/dS_ek = [margin - f_e + S_ek > 0]
(0 on the hinge itself), dl/df_e = minus their number.  All are sums, not means.
"""

from __future__ import annotations

import numpy as np

DOT, DISTMULT, COMPLEX, TRANSE = 0, 1, 2, 3
SOFTMAX, LOGISTIC, SOFTMAX_POS, MARGIN = 0, 1, 2, 3


def _halves(x):
    h = x.shape[-1] // 2
    return x[..., :h], x[..., h:]


def cmul(a, b):
    """Complex product a*b on [re | im] rows."""
    ar, ai = _halves(a)
    br, bi = _halves(b)
    return np.concatenate([ar * br - ai * bi, ar * bi + ai * br], axis=-1)


def cmul_conj(a, b):
    """conj(a)*b on [re | im] rows."""
    ar, ai = _halves(a)
    br, bi = _halves(b)
    return np.concatenate([ar * br + ai * bi, ar * bi - ai * br], axis=-1)


def _fp32(x):
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def compose_u(score, s, r, rounded=True):
    """u = theta_s (x) theta_r.  rounded: the translational u as the fp32 number (see above);
    False leaves it exact, for derivative checks, which perturb below fp32 resolution."""
    if score == TRANSE:
        return _fp32(np.asarray(s, np.float32) + np.asarray(r, np.float32)) if rounded else s + r
    if score == DOT:
        return s.copy()
    if score == DISTMULT:
        return s * r
    return cmul(s, r)


def compose_v(score, r, d, rounded=True):
    """v = conj(theta_r) (x) theta_d  (the operand that meets theta_s)."""
    if score == TRANSE:
        return _fp32(np.asarray(d, np.float32) - np.asarray(r, np.float32)) if rounded else d - r
    if score == DOT:
        return d.copy()
    if score == DISTMULT:
        return r * d
    return cmul_conj(r, d)


def pair_scores(score, q, rows):
    """q (+) row for every pair: q [C, dim], rows [N, dim] -> [C, N]."""
    if score == TRANSE:
        return -np.abs(q[:, None, :] - rows[None, :, :]).sum(axis=-1)
    return q @ rows.T


def positive_scores(score, s, r, d, rounded=True):
    if score == TRANSE:
        return -np.abs(compose_u(score, s, r, rounded) - d).sum(axis=-1)
    return np.sum(compose_u(score, s, r) * d, axis=-1)


def side_loss(loss, f, S, neg_weight, margin=1.0):
    """Loss terms and their derivatives for one chunk and one corrupted side.

    f: positive scores [C]; S: negative scores [C, N].
    Returns (loss_e [C], a_e = dl/df [C], W = dl/dS [C, N])."""
    if loss == MARGIN:
        short = margin - f[:, None] + S                      # how far each negative is from being `margin` below
        W = (short > 0.0).astype(np.float64)
        return np.maximum(short, 0.0).sum(axis=1), -W.sum(axis=1), W
    if loss == SOFTMAX:
        m = S.max(axis=1, keepdims=True)
        ex = np.exp(S - m)
        z = ex.sum(axis=1, keepdims=True)
        lse = (m + np.log(z))[:, 0]
        return -f + lse, -np.ones_like(f), ex / z
    if loss == SOFTMAX_POS:
        # -f + log(exp f + sum_k exp S_k): the positive competes with its negatives
        m = np.maximum(S.max(axis=1), f)[:, None]
        ex = np.exp(S - m)
        ef = np.exp(f[:, None] - m)
        z = ex.sum(axis=1, keepdims=True) + ef
        lse = (m + np.log(z))[:, 0]
        # dl/df = -1 + e^f / z = -(sum_k e^S_k) / z: the second form has no cancellation where the positive dominates
        return -f + lse, -(ex.sum(axis=1, keepdims=True) / z)[:, 0], ex / z
    # logistic: softplus(-f) + w * sum_k softplus(S_k)
    sp = lambda x: np.logaddexp(0.0, x)
    sig = lambda x: np.exp(-np.logaddexp(0.0, -x))       # 1 / (1 + e^-x), accurate for any x (e^x for x << 0)
    l = sp(-f) + neg_weight * sp(S).sum(axis=1)
    return l, -sig(-f), neg_weight * sig(S)


def chain_from_u(score, g_u, s, r):
    """(g_s, g_r) from the gradient with respect to u = s (x) r."""
    if score == TRANSE:
        return g_u, g_u
    if score == DOT:
        return g_u, None
    if score == DISTMULT:
        return r * g_u, s * g_u
    return cmul_conj(r, g_u), cmul_conj(s, g_u)


def chain_from_v(score, g_v, r, d):
    """(g_d, g_r) from the gradient with respect to v = conj(r) (x) d."""
    if score == TRANSE:
        return g_v, -g_v
    if score == DOT:
        return g_v, None
    if score == DISTMULT:
        return r * g_v, d * g_v
    return cmul(r, g_v), cmul_conj(g_v, d)


def chunk_side(score, loss, neg_weight, side_is_dst, s, r, d, negs, rounded=True, margin=1.0):
    """Loss and gradients of one chunk for one corrupted side.

    s, r, d: [C, dim] float64 rows of the chunk's positive edges (r ignored for Dot).
    negs:    [N, dim] float64 rows of the shared negatives of this side.
    Returns dict(loss [C], f [C], S [C,N], W = dl/dS [C,N], a = dl/df [C], q [C,dim] (the composed
    operand that meets the negatives), g_s, g_r (or None), g_d [C,dim], g_neg [N,dim])."""
    if side_is_dst:
        q = compose_u(score, s, r, rounded) if score == TRANSE else compose_u(score, s, r)       # meets destination-like rows
        other = d
    else:
        q = compose_v(score, r, d, rounded) if score == TRANSE else compose_v(score, r, d)       # meets source-like rows
        other = s
    if score == TRANSE:
        return _chunk_side_translational(loss, neg_weight, side_is_dst, q, other, negs, margin)
    f = np.sum(q * other, axis=1)
    S = q @ negs.T
    l, a, W = side_loss(loss, f, S, neg_weight, margin)
    g_q = a[:, None] * other + W @ negs
    g_other = a[:, None] * q
    g_neg = W.T @ q
    if side_is_dst:
        g_s, g_r = chain_from_u(score, g_q, s, r)
        g_d = g_other
    else:
        g_d, g_r = chain_from_v(score, g_q, r, d)
        g_s = g_other
    return dict(loss=l, f=f, S=S, W=W, a=a, q=q, g_s=g_s, g_r=g_r, g_d=g_d, g_neg=g_neg)


def _chunk_side_translational(loss, neg_weight, side_is_dst, q, other, negs, margin=1.0):
    """chunk_side for the translational score: pair score -|q - row|_1,
    d(pair)/dq = -sign(q - row), d(pair)/drow = +sign(q - row)."""
    f = -np.abs(q - other).sum(axis=1)
    sg = np.sign(q[:, None, :] - negs[None, :, :])            # [C, N, dim]
    S = -np.abs(q[:, None, :] - negs[None, :, :]).sum(axis=-1)
    l, a, W = side_loss(loss, f, S, neg_weight, margin)
    sg_pos = np.sign(q - other)
    g_q = -a[:, None] * sg_pos - np.einsum("ck,ckj->cj", W, sg)
    g_other = a[:, None] * sg_pos
    g_neg = np.einsum("ck,ckj->kj", W, sg)
    if side_is_dst:                                            # q = s + r
        return dict(loss=l, f=f, S=S, W=W, a=a, q=q, g_s=g_q, g_r=g_q, g_d=g_other, g_neg=g_neg)
    return dict(loss=l, f=f, S=S, W=W, a=a, q=q, g_s=g_other, g_r=-g_q, g_d=g_q, g_neg=g_neg)    # q = d - r
