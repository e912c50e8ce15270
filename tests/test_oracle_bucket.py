"""Pins for the oracle's update stage and bucket-level semantics."""

import numpy as np
import pytest
import torch

from oracle import model, negatives
from oracle.bucket import (OracleConfig, Tables, adagrad_rows, batch_gradients, score_edges,
                           train_batch, train_bucket)


def test_adagrad_first_step_closed_form():
    theta = np.array([[1.0, -2.0, 0.5]], np.float32)
    state = np.zeros_like(theta)
    g = np.array([[0.25, -4.0, 1e-3]], np.float64)
    adagrad_rows(theta, state, np.array([0]), g, lr=0.1, eps=1e-10)
    # zero accumulator: delta = -lr * G / (|G| + eps), i.e. -lr * sign(G) to 1e-7
    np.testing.assert_allclose(theta, [[1.0 - 0.1, -2.0 + 0.1, 0.5 - 0.1]], rtol=2e-7)
    np.testing.assert_allclose(state, g ** 2, rtol=2e-7)


def test_adagrad_second_step_uses_accumulated_squares():
    theta = np.zeros((1, 1), np.float32)
    state = np.zeros((1, 1), np.float32)
    adagrad_rows(theta, state, np.array([0]), np.array([[3.0]]), 0.5, 1e-10)
    adagrad_rows(theta, state, np.array([0]), np.array([[4.0]]), 0.5, 1e-10)
    assert state[0, 0] == 25.0
    np.testing.assert_allclose(theta[0, 0], -0.5 - 0.5 * 4.0 / 5.0, rtol=1e-7)


def _setup(score=model.DISTMULT, corrupt=2, n_part=2, nodes=40, dim=8, seed=0, loss=model.SOFTMAX,
           batch=12, chunk=5, negs=7, deg=2, m=30):
    cfg = OracleConfig(num_nodes=nodes, num_relations=4 if score else 0, dim=dim, num_partitions=n_part,
                       batch_size=batch, chunk_size=chunk, num_negs=negs, num_degree_negs=deg,
                       score=score, loss=loss, corrupt=corrupt, seed=seed)
    rng = np.random.default_rng(seed)
    node = (0.5 * rng.standard_normal((nodes, dim))).astype(np.float32)
    rel = (0.5 * rng.standard_normal((4, dim))).astype(np.float32)
    rp = cfg.rows_per_partition
    edges = np.stack([rng.integers(0, rp, m), rng.integers(0, 4, m), rng.integers(0, rp, m)], 1).astype(np.int32)
    return cfg, node, rel, edges


@pytest.mark.parametrize("bucket", [(0, 0), (0, 1)])
def test_sparse_update_equals_dense_torch_adagrad(bucket):
    # Two consecutive batches: the dense optimiser applied to the scattered batch
    # gradient must move touched rows exactly like the sparse rule and must not
    # move anything else.
    i, j = bucket
    cfg, node, rel, edges = _setup()
    tab = Tables(cfg, node, rel)
    rp = cfg.rows_per_partition
    dense_node = torch.tensor(node.copy())
    dense_rel = torch.tensor(rel.copy())
    opt = torch.optim.Adagrad([dense_node, dense_rel], lr=cfg.lr, eps=cfg.eps, initial_accumulator_value=0.0)
    for b in range(2):
        ref = Tables(cfg, dense_node.numpy().copy(), dense_rel.numpy().copy())
        _, gnode, grel = batch_gradients(ref, i, j, edges, b, 0)
        gn = np.zeros_like(node, dtype=np.float64)
        for slot, part in ((0, i), (1, j)):
            if slot in gnode:
                rows, g = gnode[slot]
                gn[part * rp + rows] += g
        gr = np.zeros_like(rel, dtype=np.float64)
        gr[grel[0]] = grel[1]
        dense_node.grad = torch.tensor(gn.astype(np.float32))
        dense_rel.grad = torch.tensor(gr.astype(np.float32))
        opt.step()
        train_batch(tab, i, j, edges, b, 0)
        np.testing.assert_allclose(tab.node_table(0), dense_node.numpy(), rtol=3e-6, atol=1e-7)
        np.testing.assert_allclose(tab.RE, dense_rel.numpy(), rtol=3e-6, atol=1e-7)
    acc = opt.state[dense_node]["sum"].numpy()
    np.testing.assert_allclose(tab.node_table(1), acc, rtol=3e-6, atol=1e-12)


@pytest.mark.parametrize("score", [model.DOT, model.COMPLEX])
def test_untouched_and_padding_rows_stay_bit_identical(score):
    cfg, node, rel, edges = _setup(score=score, nodes=41, n_part=2, corrupt=0, m=12)
    assert cfg.rows_per_partition == 21            # partition 1 has one padding row
    tab = Tables(cfg, node, rel)
    before_E = [e.copy() for e in tab.E]
    before_S = [s.copy() for s in tab.S]
    before_R = tab.RE.copy()
    rec = {}
    train_batch(tab, 0, 1, edges, 0, 0, record=rec)
    touched = rec["touched"]
    rows = {t: set() for t in (0, 1, 2)}
    for k in touched:
        rows[int(k) >> 32].add(int(k) & 0xFFFFFFFF)
    for slot, part in ((0, 0), (1, 1)):
        for r in range(21):
            same = (tab.E[part][r].tobytes() == before_E[part][r].tobytes()
                    and tab.S[part][r].tobytes() == before_S[part][r].tobytes())
            if r not in rows[slot]:
                assert same, (slot, r)
    assert 20 not in rows[1]                       # the padding row is never sampled
    if score == model.DOT:
        assert tab.RE.tobytes() == before_R.tobytes()
    # a touched row with a non-zero gradient moved
    moved = sum(tab.E[0][r].tobytes() != before_E[0][r].tobytes() for r in rows[0])
    assert moved == len(rows[0])


def test_next_batch_sees_previous_update_and_reads_are_snapshots():
    cfg, node, rel, edges = _setup(score=model.DOT, corrupt=0, n_part=1, nodes=20, m=24)
    tab = Tables(cfg, node, rel)
    train_batch(tab, 0, 0, edges, 0, 0)
    after_one = tab.E[0].copy()
    l1 = train_batch(tab, 0, 0, edges, 1, 0)
    # loss of batch 1 equals the loss computed from the tables after batch 0, not the initial ones
    fresh = Tables(cfg, after_one, rel)
    assert batch_gradients(fresh, 0, 0, edges, 1, 0)[0] == l1
    init = Tables(cfg, node, rel)
    assert batch_gradients(init, 0, 0, edges, 1, 0)[0] != l1


def test_partial_last_batch_and_bucket_totals():
    cfg, node, rel, edges = _setup(m=30, batch=12)
    tab = Tables(cfg, node, rel)
    out = train_bucket(tab, 1, 0, edges, epoch=2)
    assert out["batches"] == 3 and out["edges"] == 30
    tab2 = Tables(cfg, node, rel)
    total = sum(train_batch(tab2, 1, 0, edges, b, 2) for b in range(3))
    assert total == out["loss_sum"]


def test_score_edges_uses_global_ids_across_partitions():
    cfg, node, rel, _ = _setup(score=model.COMPLEX, nodes=41)
    tab = Tables(cfg, node, rel)
    src = np.array([0, 40, 21, 20])
    dst = np.array([39, 1, 22, 0])
    r = np.array([0, 1, 2, 3])
    got = score_edges(tab, src, r, dst)
    want = model.positive_scores(model.COMPLEX, node[src].astype(np.float64), rel[r].astype(np.float64),
                                 node[dst].astype(np.float64))
    np.testing.assert_array_equal(got, want)


def test_training_reduces_eq1_loss_on_a_learnable_toy_graph():
    # ring graph: training must pull the loss of the same edges down
    n = 30
    cfg = OracleConfig(num_nodes=n, num_relations=0, dim=8, num_partitions=1, batch_size=n, chunk_size=10,
                       num_negs=10, score=model.DOT, seed=3, lr=0.1)
    rng = np.random.default_rng(0)
    node = (0.1 * rng.standard_normal((n, 8))).astype(np.float32)
    edges = np.stack([np.arange(n), np.zeros(n, int), (np.arange(n) + 1) % n], 1).astype(np.int32)
    tab = Tables(cfg, node, None)
    losses = [train_bucket(tab, 0, 0, edges, epoch=ep)["loss_sum"] for ep in range(30)]
    assert losses[-1] < 0.5 * losses[0]
