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


def chunk_magnitudes(score, side_is_dst, s, r, d, negs, out):
    """Magnitudes for one chunk and one corrupted side.

    s, r, d, negs: the float64 rows the oracle's chunk_side was given; out: its result (W, a, S, f, q).
    Returns dict(m_s, m_r (or None), m_d [C,dim], m_neg [N,dim], m_loss [C])."""
    W, a, q = out["W"], out["a"], out["q"]
    other = d if side_is_dst else s
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

    def __init__(self, score, same_part):
        self.score = score
        self.tj = 0 if same_part else 1
        self.keys = {0: [], 1: [], 2: []}
        self.mags = {0: [], 1: [], 2: []}
        self.loss_magnitude = 0.0

    def __call__(self, si, side_is_dst, c, edge_rows, neg_ids, s, r, d, negs, out):
        m = chunk_magnitudes(self.score, side_is_dst, s, r, d, negs, out)
        self.loss_magnitude += float(m["m_loss"].sum())
        neg_slot = self.tj if side_is_dst else 0
        for slot, keys, mag in ((0, edge_rows[:, 0], m["m_s"]), (self.tj, edge_rows[:, 2], m["m_d"]), (neg_slot, neg_ids, m["m_neg"])):
            self.keys[slot].append(np.asarray(keys, np.int64))
            self.mags[slot].append(mag)
        if m["m_r"] is not None and self.score != DOT:
            self.keys[2].append(np.asarray(edge_rows[:, 1], np.int64))
            self.mags[2].append(m["m_r"])

    def coalesced(self):
        """{slot: (unique rows, summed magnitudes)} for slots 0 (partition i), 1 (partition j != i), 2 (relations)."""
        res = {}
        for slot in (0, 1, 2):
            if not self.keys[slot]:
                continue
            k = np.concatenate(self.keys[slot])
            g = np.concatenate(self.mags[slot], axis=0)
            uniq, inv = np.unique(k, return_inverse=True)
            acc = np.zeros((uniq.size, g.shape[1]))
            np.add.at(acc, inv, g)
            res[slot] = (uniq, acc)
        return res
