"""Forward-error model of an fp32 evaluation of one chunk's gradients (test infrastructure, not the oracle).

The oracle (oracle/) computes the method in float64 and knows nothing of this file.  The parity tests
compare an fp32 GPU result with it and need, per gradient element, a scale for what any fp32 evaluation
of that element may be off by: the sum M of the absolute values of the elementary products the element
is made of.  A forward error bound is a small multiple (KAPPA roundoffs, parity_util.py) of M.

Softmax weights W_ek and dl/df are functions of score differences, so they carry the ABSOLUTE rounding
error of the fp32 scores, which scales with A_ek = sum_j |q_ej| |theta_kj| rather than with |S_ek|: their
magnitudes are widened by (1 + max_k A_ek / 4) per row (about 8 roundoffs times the row's largest A --
twice a dot product's few-roundoff error, once for S_ek and once for the row's log-sum -- in the callers'
unit of 32 roundoffs).  For the translational score the same role is played by max|S| dim / 128: a score
is a sum of dim same-sign distances built by up to dim/4 sequential fp32 additions of partial sums.
"""

from __future__ import annotations

import numpy as np

DOT, DISTMULT, COMPLEX, TRANSE = 0, 1, 2, 3
MARGIN_LOSS = 3
# The margin loss decides per (positive, negative) pair whether the pair pays: margin - f + S > 0, a discrete decision
# on fp32 scores whose summation order the oracle cannot reproduce.  A pair whose float64 shortfall lies within
# BAND roundoffs times its magnitude A_ek + A_f + margin of zero may be decided either way: its whole gradient term
# (not a rounding-sized share of it) goes into a second, unscaled magnitude.  Everything else about this loss is
# exact (the weights are 0 or 1), so its ordinary magnitudes carry no widening.
BAND = 16 * 2.0 ** -24


def _halves(x):
    h = x.shape[-1] // 2
    return x[..., :h], x[..., h:]


def abs_compose(score, a, b):
    """Sum of the absolute values of the products that form a (x) b (either form, conjugated or not):
    the magnitude against which the rounding error of that product is measured."""
    if score == DOT:
        return np.abs(a)
    a, b = np.abs(a), np.abs(b)
    if score == DISTMULT:
        return a * b
    ar, ai = _halves(a)
    br, bi = _halves(b)
    return np.concatenate([ar * br + ai * bi, ar * bi + ai * br], axis=-1)


def chunk_magnitudes(score, side_is_dst, s, r, d, negs, out, loss=None, margin=1.0):
    """Magnitudes for one chunk and one corrupted side.

    s, r, d, negs: the float64 rows the oracle's chunk_side was given; out: its result (W, a, S, f, q).
    Returns dict(m_s, m_r (or None), m_d [C,dim], m_neg [N,dim], m_loss [C]); for the margin loss also
    b_s, b_r, b_d, b_neg: the magnitudes of the terms whose hinge decision may fall either way."""
    W, a, q = out["W"], out["a"], out["q"]
    other = d if side_is_dst else s
    if loss == MARGIN_LOSS and score != TRANSE:
        x = s if side_is_dst else d
        aq = abs_compose(score, x, r)
        A_neg = aq @ np.abs(negs).T
        A_f = np.sum(aq * np.abs(other), axis=1)
        short = margin - out["f"][:, None] + out["S"]
        flip = (np.abs(short) <= BAND * (A_neg + A_f[:, None] + margin)).astype(np.float64)
        am = np.abs(a)
        m_q = am[:, None] * np.abs(other) + W @ np.abs(negs)
        m_other = am[:, None] * aq
        b_q = flip.sum(axis=1)[:, None] * np.abs(other) + flip @ np.abs(negs)
        b_other = flip.sum(axis=1)[:, None] * aq
        def chain(v):
            return (v if score == DOT else abs_compose(score, r, v)), (None if score == DOT else abs_compose(score, x, v))
        m_x, m_r = chain(m_q)
        b_x, b_r = chain(b_q)
        return dict(m_neg=W.T @ aq, m_r=m_r, m_loss=(W * (A_neg + A_f[:, None])).sum(axis=1) + flip.sum(axis=1) * margin,
                    m_s=m_x if side_is_dst else m_other, m_d=m_other if side_is_dst else m_x,
                    b_neg=flip.T @ aq, b_r=b_r, b_s=b_x if side_is_dst else b_other, b_d=b_other if side_is_dst else b_x)
    if score == TRANSE and loss == MARGIN_LOSS:
        # scores are minus sums of absolute differences: their magnitude is their own absolute value; the weights
        # are 0 or 1 and every gradient term is a sign
        sg = np.abs(np.sign(q[:, None, :] - negs[None, :, :]))
        sg_pos = np.abs(np.sign(q - other))
        A_neg, A_f = np.abs(out["S"]), np.abs(out["f"])
        short = margin - out["f"][:, None] + out["S"]
        flip = (np.abs(short) <= BAND * (A_neg + A_f[:, None] + margin)).astype(np.float64)
        # a gradient element is a sum of a few thousand terms +1, -1 or 0: exact in fp32 and in float64 alike, no
        # rounding to allow for (the ordinary magnitudes are zero); only the either-way pairs can differ
        m_q = np.zeros_like(q)
        m_other = np.zeros_like(q)
        b_q = flip.sum(axis=1)[:, None] * sg_pos + np.einsum("ck,ckj->cj", flip, sg)
        b_other = flip.sum(axis=1)[:, None] * sg_pos
        return dict(m_neg=np.zeros_like(negs), m_r=m_q,
                    m_loss=(W * (A_neg + A_f[:, None])).sum(axis=1) + flip.sum(axis=1) * margin,
                    m_s=m_q if side_is_dst else m_other, m_d=m_other if side_is_dst else m_q,
                    b_neg=np.einsum("ck,ckj->kj", flip, sg), b_r=b_q,
                    b_s=b_q if side_is_dst else b_other, b_d=b_other if side_is_dst else b_q)
    if score == TRANSE:
        sg = np.abs(np.sign(q[:, None, :] - negs[None, :, :]))        # which terms exist: sign(0) = 0 contributes nothing
        sg_pos = np.abs(np.sign(q - other))
        spread = np.maximum(np.abs(out["S"]).max(axis=1), np.abs(out["f"])) * (q.shape[1] / 128.0)
        Wm = np.abs(W) * (1.0 + spread)[:, None]
        am = np.abs(a) * (1.0 + spread)
        m_q = am[:, None] * sg_pos + np.einsum("ck,ckj->cj", Wm, sg)
        m_other = am[:, None] * sg_pos
        return dict(m_neg=np.einsum("ck,ckj->kj", Wm, sg), m_r=m_q, m_loss=spread,
                    m_s=m_q if side_is_dst else m_other, m_d=m_other if side_is_dst else m_q)
    x = s if side_is_dst else d
    aq = abs_compose(score, x, r)
    spread = np.maximum((aq @ np.abs(negs).T).max(axis=1), np.sum(aq * np.abs(other), axis=1)) / 4.0
    Wm = np.abs(W) * (1.0 + spread)[:, None]
    am = np.abs(a) * (1.0 + spread)
    m_q = am[:, None] * np.abs(other) + Wm @ np.abs(negs)
    m_other = am[:, None] * aq
    m_x = m_q if score == DOT else abs_compose(score, r, m_q)
    m_r = None if score == DOT else abs_compose(score, x, m_q)
    return dict(m_neg=Wm.T @ aq, m_r=m_r, m_loss=spread,
                m_s=m_x if side_is_dst else m_other, m_d=m_other if side_is_dst else m_x)


class BatchMagnitudes:
    """Observer for oracle.bucket.batch_gradients: collects the magnitudes of a batch's chunks and
    coalesces them by table row the way the gradients themselves are coalesced."""

    def __init__(self, score, same_part, loss=None, margin=1.0):
        self.score, self.loss, self.margin = score, loss, margin
        self.tj = 0 if same_part else 1
        self.keys = {0: [], 1: [], 2: []}
        self.mags = {0: [], 1: [], 2: []}
        self.bands = {0: [], 1: [], 2: []}
        self.loss_magnitude = 0.0

    def __call__(self, si, side_is_dst, c, edge_rows, neg_ids, s, r, d, negs, out):
        m = chunk_magnitudes(self.score, side_is_dst, s, r, d, negs, out, self.loss, self.margin)
        self.loss_magnitude += float(m["m_loss"].sum())
        neg_slot = self.tj if side_is_dst else 0
        banded = "b_s" in m
        for slot, keys, mag, band in ((0, edge_rows[:, 0], m["m_s"], m.get("b_s")), (self.tj, edge_rows[:, 2], m["m_d"], m.get("b_d")),
                                      (neg_slot, neg_ids, m["m_neg"], m.get("b_neg"))):
            self.keys[slot].append(np.asarray(keys, np.int64))
            self.mags[slot].append(mag)
            if banded:
                self.bands[slot].append(band)
        if m["m_r"] is not None and self.score != DOT:
            self.keys[2].append(np.asarray(edge_rows[:, 1], np.int64))
            self.mags[2].append(m["m_r"])
            if banded:
                self.bands[2].append(m["b_r"])

    def coalesced(self):
        """{slot: (unique rows, summed magnitudes, summed either-way magnitudes or None)} for slots 0 (partition i),
        1 (partition j != i), 2 (relations)."""
        res = {}
        for slot in (0, 1, 2):
            if not self.keys[slot]:
                continue
            k = np.concatenate(self.keys[slot])
            uniq, inv = np.unique(k, return_inverse=True)

            def summed(parts):
                g = np.concatenate(parts, axis=0)
                acc = np.zeros((uniq.size, g.shape[1]))
                np.add.at(acc, inv, g)
                return acc
            res[slot] = (uniq, summed(self.mags[slot]), summed(self.bands[slot]) if self.bands[slot] else None)
        return res
