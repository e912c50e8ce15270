"""The forward-error model of the parity tests (tests/error_model.py) against a plain float32 program."""

import numpy as np
import pytest
import torch

from oracle import model
from tests import error_model


@pytest.mark.parametrize("std", [0.1, 1.0, 3.0])
@pytest.mark.parametrize("score,loss", [(model.DOT, model.SOFTMAX), (model.DISTMULT, model.SOFTMAX_POS),
                                        (model.COMPLEX, model.LOGISTIC), (model.DISTMULT, model.SOFTMAX)])
def test_gradient_magnitudes_bound_a_plain_float32_evaluation(score, loss, std):
    """The magnitudes computed next to the oracle's gradients are an error model: any fp32 evaluation of a gradient
    element must lie within a few dozen roundoffs times its magnitude.  Checked against the same formulas
    run in float32 by torch (its own matmul and reduction order), from small scores to scores in the hundreds."""
    rng = np.random.default_rng(17)
    C, N, d = 50, 300, 100
    s, r, dd, negs = (rng.standard_normal(sh) * std for sh in ((C, d), (C, d), (C, d), (N, d)))
    s, r, dd, negs = (a.astype(np.float32) for a in (s, r, dd, negs))
    out = model.chunk_side(score, loss, 1.0 / N, True, s.astype(np.float64), r.astype(np.float64),
                           dd.astype(np.float64), negs.astype(np.float64))
    out.update(error_model.chunk_magnitudes(score, True, s.astype(np.float64), r.astype(np.float64), dd.astype(np.float64),
                                            negs.astype(np.float64), out))
    ts, tr, td, tn = (torch.tensor(a, requires_grad=True) for a in (s, r, dd, negs))
    if score == model.DOT:
        q = ts
    elif score == model.DISTMULT:
        q = ts * tr
    else:
        h = d // 2
        q = torch.cat([ts[:, :h] * tr[:, :h] - ts[:, h:] * tr[:, h:], ts[:, :h] * tr[:, h:] + ts[:, h:] * tr[:, :h]], 1)
    f = (q * td).sum(1)
    S = q @ tn.T
    if loss == model.SOFTMAX:
        l = torch.logsumexp(S, 1) - f
    elif loss == model.SOFTMAX_POS:
        l = torch.logsumexp(torch.cat([f[:, None], S], 1), 1) - f
    else:
        l = torch.nn.functional.softplus(-f) + torch.nn.functional.softplus(S).sum(1) / N
    l.sum().backward()
    kappa = 32 * 2.0 ** -24
    # weights below fp32's normal range (2^-126) are lost altogether: each of up to N terms, times an operand
    big = max(float(np.abs(a).max()) for a in (s, r, dd, negs))
    floor = 2.0 ** -126 * N * max(big, big * big)
    for name, got, mag in (("g_s", ts.grad, out["m_s"]), ("g_d", td.grad, out["m_d"]), ("g_neg", tn.grad, out["m_neg"])):
        err = np.abs(got.numpy().astype(np.float64) - out[name])
        assert np.all(err <= kappa * mag + floor), (name, float((err / (kappa * mag + floor)).max()))
    if score != model.DOT:
        err = np.abs(tr.grad.numpy().astype(np.float64) - out["g_r"])
        assert np.all(err <= kappa * out["m_r"] + floor)
    assert abs(float(l.sum()) - out["loss"].sum()) <= 1e-5 * abs(out["loss"].sum()) + kappa * out["m_loss"].sum()


@pytest.mark.parametrize("score", [model.DOT, model.DISTMULT, model.TRANSE])
def test_margin_loss_bands_cover_a_plain_float32_evaluation(score):
    """Margin loss: the weights are 0 or 1, decided on fp32 scores.  A float32 evaluation (torch, its own
    summation order) may decide a pair within a few roundoffs of its hinge the other way; the error model carries
    the whole gradient term of such a pair in a second magnitude (b_*).  Everything else is within the ordinary
    magnitudes - which are zero for the translational score, whose gradient elements are exact sums of signs."""
    rng = np.random.default_rng(23)
    C, N, d, margin = 50, 300, 100, 1.0
    std = 0.3
    s, r, dd, negs = (rng.standard_normal(sh) * std for sh in ((C, d), (C, d), (C, d), (N, d)))
    s, r, dd, negs = (a.astype(np.float32) for a in (s, r, dd, negs))
    if score == model.TRANSE:
        # put some pairs exactly on their hinge: a negative equal to the positive's row scores f, so margin 0 ...
        margin = 0.0
        negs[:C:5] = dd[::5]
    args64 = [a.astype(np.float64) for a in (s, r, dd, negs)]
    out = model.chunk_side(score, model.MARGIN, 1.0 / N, True, *args64, margin=margin)
    mags = error_model.chunk_magnitudes(score, True, *args64, out, loss=model.MARGIN, margin=margin)
    ts, tr, td, tn = (torch.tensor(a, requires_grad=True) for a in (s, r, dd, negs))
    if score == model.DOT:
        q = ts
    elif score == model.DISTMULT:
        q = ts * tr
    else:
        q = ts + tr
    if score == model.TRANSE:
        f = -(q - td).abs().sum(1)
        S = -(q[:, None, :] - tn[None, :, :]).abs().sum(2)
    else:
        f = (q * td).sum(1)
        S = q @ tn.T
    l = torch.clamp(margin - f[:, None] + S, min=0.0).sum(1)
    l.sum().backward()
    kappa = 32 * 2.0 ** -24
    flips = 0.0
    for name, got, mag, band in (("g_s", ts.grad, mags["m_s"], mags["b_s"]), ("g_d", td.grad, mags["m_d"], mags["b_d"]),
                                 ("g_neg", tn.grad, mags["m_neg"], mags["b_neg"])):
        err = np.abs(got.numpy().astype(np.float64) - out[name])
        assert np.all(err <= kappa * mag + band), (name, float(err.max()))
        flips += float(band.sum())
    if score == model.TRANSE:
        assert not mags["m_s"].any() and not mags["m_neg"].any() and flips > 0      # exact but for the pairs on the hinge
    assert abs(float(l.sum()) - out["loss"].sum()) <= 1e-5 * abs(out["loss"].sum()) + kappa * mags["m_loss"].sum()
