"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times.

One batch step from identical tables, compared element by element on every row the batch touches
(the oracle finishes a full-size batch in seconds), plus bit-exact negative ids / touched-row sets
and bit-identical untouched rows.  c1: the whole epoch; c2 (the benchmark workload): first batches
of an off-diagonal and a diagonal bucket; c3: first, second and the partial last batch.  c4 shares
c2's per-batch shape (d = 100, B = 50 000, C = 50, N = 1 000) and differs in table size only.  c5
adds ComplEx, 14 824 relations and corruption of both sides to that shape: its full batch runs
here on a graph with 1/64 of the nodes (the tables of the full one do not fit the test's time
budget); smaller ComplEx cases are in test_gpu_parity.py.
"""

import numpy as np
import pytest

from oracle import negatives
from oracle.bucket import OracleConfig
from tests.parity_util import EMB_RTOL, STATE_RTOL, OracleRun, compare_table
from workloads import graphs

pytestmark = pytest.mark.gpu


class _Setup:
    def __init__(self, name, seed=5):
        from paper_2505_09258_amd import binding as L
        self.L = L
        self.w = w = graphs.WORKLOADS[name] if isinstance(name, str) else name
        src, rel_ids, dst = graphs.generate_edges(w, seed)
        self.buckets = graphs.bucket_edges(w, src, rel_ids, dst)
        del src, rel_ids, dst
        node, rel = graphs.init_tables(w, seed)
        self.uses_rel = w.score != graphs.SCORE_DOT
        n = w.num_partitions
        cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=n,
                            num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                            batch_size=w.batch_size, chunk_size=w.chunk_size, num_negs=w.num_negs,
                            num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=seed)
        self.ctx = L.legend_init_partitions(cfg, node, rel if self.uses_rel else None)
        for p in range(n):
            L.legend_swap_partition(self.ctx, -1, p)
        self.ocfg = OracleConfig.from_workload(w, seed=seed)
        self.run = OracleRun(self.ocfg, node, rel if self.uses_rel else None)
        self.rp = self.ocfg.rows_per_partition
        self.rng = np.random.default_rng(seed)

    def close(self):
        self.L.legend_destroy(self.ctx)

    def check_batch(self, i, j, b, epoch=0, check_indices=True):
        """Trains batch b of bucket (i, j) on both sides from tables that are equal, compares,
        then copies the GPU's rows into the oracle so that the next call starts equal again."""
        L, ctx, w, run, rp, d = self.L, self.ctx, self.w, self.run, self.rp, self.w.dim
        edges = self.buckets[(i, j)]
        e = edges[b * w.batch_size:(b + 1) * w.batch_size]
        tag = f"{w.name} bucket ({i},{j}) batch {b}"

        if check_indices:
            want_neg = negatives.batch_negatives(self.ocfg, epoch, i, j, b, e, edges)
            want_touched = negatives.touched_rows(self.ocfg, i, j, e, want_neg)
            neg, touched = L.legend_debug_batch_indices(ctx, i, j, edges, epoch, b, want_neg.size, want_touched.size + 8)
            np.testing.assert_array_equal(neg.reshape(want_neg.shape), want_neg)
            np.testing.assert_array_equal(touched, want_touched)

        # rows the batch will not touch, sampled before the step
        parts = sorted({i, j})
        quiet = {}
        for p in parts:
            valid = min(rp, w.num_nodes - p * rp)
            rows = self.rng.integers(0, valid, size=min(valid, 100_000))
            quiet[p] = (rows, run.tab.E[p][rows].copy(), run.tab.S[p][rows].copy())

        stats = L.legend_train_bucket_range(ctx, i, j, edges, epoch=epoch, batch_begin=b, batch_end=b + 1)
        want_loss = run.train_bucket(i, j, edges, epoch=epoch, batch_begin=b, max_batches=1)
        assert stats["batches"] == 1 and stats["edges"] == e.shape[0]
        assert abs(stats["loss_sum"] - want_loss) <= 1e-5 * abs(want_loss) + run.last_loss_allowance, (tag, stats["loss_sum"], want_loss)

        for p in parts:
            rows = np.flatnonzero(run.touched_node[p])
            assert rows.size
            ids = p * rp + rows
            got_E = L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, ids, ids.size, d)
            got_S = L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, ids, ids.size, d)
            compare_table(f"{tag} partition {p} embeddings", got_E, run.tab.E[p][rows], run.fe_node[p][rows], EMB_RTOL, 0.1)
            compare_table(f"{tag} partition {p} state", got_S, run.tab.S[p][rows], run.fs_node[p][rows], STATE_RTOL, 0.0)
            qrows, qE, qS = quiet[p]
            still = ~run.touched_node[p][qrows]
            qids = p * rp + qrows[still]
            assert np.array_equal(L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, qids, qids.size, d), qE[still])
            assert np.array_equal(L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, qids, qids.size, d), qS[still])
            # next call starts from the GPU's values
            run.tab.E[p][rows] = got_E
            run.tab.S[p][rows] = got_S
            run.fe_node[p][rows] = 0
            run.fs_node[p][rows] = 0
            run.touched_node[p][rows] = False
        if self.uses_rel:
            nrel = run.tab.RE.shape[0]
            got_E = L.legend_read_embeddings(ctx, L.TABLE_REL_EMB, None, nrel, d)
            got_S = L.legend_read_embeddings(ctx, L.TABLE_REL_STATE, None, nrel, d)
            compare_table(f"{tag} relation embeddings", got_E, run.tab.RE, run.fe_rel, EMB_RTOL, 0.1)
            compare_table(f"{tag} relation state", got_S, run.tab.RS, run.fs_rel, STATE_RTOL, 0.0)
            run.tab.RE[:] = got_E
            run.tab.RS[:] = got_S
            run.fe_rel[:] = 0
            run.fs_rel[:] = 0
            run.touched_rel[:] = False


def test_c1_whole_epoch_batch_by_batch():
    s = _Setup("c1")
    try:
        nb = -(-s.buckets[(0, 0)].shape[0] // s.w.batch_size)
        assert nb == 100
        for b in range(nb):
            s.check_batch(0, 0, b, check_indices=b in (0, nb - 1))
    finally:
        s.close()


def test_c2_full_size_batches():
    """The workload bench.py times: 50 000 edges, 1 000 chunks of 50 with 1 000 negatives each."""
    s = _Setup("c2")
    try:
        s.check_batch(0, 1, 0)
        s.check_batch(2, 2, 0)
        s.check_batch(0, 1, 1, check_indices=False)
    finally:
        s.close()


def test_c3_full_size_batches():
    """d = 400, both sides corrupted, 1 345 relations; the last batch is partial."""
    s = _Setup("c3")
    try:
        nb = -(-s.buckets[(0, 0)].shape[0] // s.w.batch_size)
        for b in (0, 1, nb - 1):
            s.check_batch(0, 0, b, check_indices=b != 1)
    finally:
        s.close()


def test_c5_shape_full_batch():
    """c5's batch (ComplEx, d = 100, 50 000 edges, both sides corrupted, 2 000 chunk launches of
    50 x 1 000) on 1/64 of its nodes in 4 partitions."""
    w = graphs.scaled(graphs.WORKLOADS["c5"], 64, 32, num_partitions=4)
    s = _Setup(w)
    try:
        assert s.buckets[(1, 2)].shape[0] >= 2 * w.batch_size
        s.check_batch(1, 2, 0)
        s.check_batch(3, 3, 0, check_indices=False)
    finally:
        s.close()
