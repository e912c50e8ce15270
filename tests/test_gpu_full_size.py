"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times.

One batch step from identical tables, compared element by element on every row the batch touches
(the oracle finishes a full-size batch in seconds), plus bit-exact negative ids / touched-row sets
and bit-identical untouched rows.  c1: the whole epoch; c2: first batches of an off-diagonal and a diagonal bucket; c3: first, second
and the partial last batch.  c4 and c5 at their table geometry: two of their sixteen partitions at
full size (2.6 M and 5.375 M rows; a c5 slot holds byte offsets past 2^31), one full batch of an
off-diagonal and of a diagonal bucket each.  c5's batch also runs on a graph with 1/64 of the nodes
in four partitions.  Every case reports, and the full-size ones assert, how much of the comparison
ran at the plain 1e-5 bound.
"""

import numpy as np
import pytest

from oracle import negatives
from oracle.bucket import OracleConfig
from tests.parity_util import EMB_RTOL, STATE_RTOL, OracleRun, check_loss, compare_table
from workloads import graphs

pytestmark = pytest.mark.gpu

# Floors asserted on the full-size cases (see _Setup.assert_shares): the share of the embedding elements that
# agree with the oracle at the plain bound 1e-5 * max(|theta|, lr), with no allowance at all, and the cap on the
# share of elements whose allowance exceeds a whole Adagrad step (ill-conditioned: the terms of the gradient cancel
# to below 1e-6 of their size, so the sign-like first step is decided by rounding; such an element is not tested).
# Measured: c1 0.99999, c2 0.99969, c3 0.99942, c4 geometry 0.99998, c5 geometry 0.99995 at the plain bound;
# at most 9.1e-6 of the elements untested.
_MIN_SHARE_AT_PLAIN_BOUND = 0.999
_MAX_SHARE_UNTESTED = 1e-4


class _Setup:
    """seeded_fill: the tables come from the library's own seeded fill (init pointers NULL, standard deviation
    init_std) and are read back for the oracle -- for geometries whose tables take too long to draw on the host."""

    def __init__(self, name, seed=5, seeded_fill=False, init_std=None):
        from paper_2505_09258_amd import binding as L
        self.L = L
        self.w = w = graphs.WORKLOADS[name] if isinstance(name, str) else name
        src, rel_ids, dst = graphs.generate_edges(w, seed)
        self.buckets = graphs.bucket_edges(w, src, rel_ids, dst)
        del src, rel_ids, dst
        self.uses_rel = w.score != graphs.SCORE_DOT
        n = w.num_partitions
        nrel = max(w.num_relations, 1)
        cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=n,
                            num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                            batch_size=w.batch_size, chunk_size=w.chunk_size, num_negs=w.num_negs,
                            num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=seed,
                            init_std=init_std if init_std is not None else w.init_std)
        if seeded_fill:
            self.ctx = L.legend_init_partitions(cfg, None, None)
            node = L.legend_read_embeddings(self.ctx, L.TABLE_NODE_EMB, None, w.num_nodes, w.dim)
            rel = L.legend_read_embeddings(self.ctx, L.TABLE_REL_EMB, None, nrel, w.dim)
            if self.uses_rel:
                assert rel.any()
        else:
            node, rel = graphs.init_tables(w, seed)
            self.ctx = L.legend_init_partitions(cfg, node, rel if self.uses_rel else None)
        for p in range(n):
            L.legend_swap_partition(self.ctx, -1, p)
        self.ocfg = OracleConfig.from_workload(w, seed=seed)
        self.run = OracleRun(self.ocfg, node, rel if self.uses_rel else None, sparse=True)
        del node
        self.rp = self.ocfg.rows_per_partition
        self.rng = np.random.default_rng(seed)
        self.stats = []          # (table kind, statistics) of every comparison

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
            if valid > 1000:
                rows[:3] = [0, valid - 1, valid // 2]           # the ends of the partition among them
            quiet[p] = (rows, run.tab.E[p][rows].copy(), run.tab.S[p][rows].copy())

        stats = L.legend_train_bucket_range(ctx, i, j, edges, epoch=epoch, batch_begin=b, batch_end=b + 1)
        want_loss = run.train_bucket(i, j, edges, epoch=epoch, batch_begin=b, max_batches=1)
        assert stats["batches"] == 1 and stats["edges"] == e.shape[0]
        check_loss(f"{tag} loss", stats["loss_sum"], want_loss, run.last_loss_allowance)

        for p in parts:
            rows, fe, fs = run.last[p]
            assert rows.size
            ids = p * rp + rows
            got_E = L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, ids, ids.size, d)
            got_S = L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, ids, ids.size, d)
            self.stats.append(compare_table(f"{tag} partition {p} embeddings", got_E, run.tab.E[p][rows], fe, EMB_RTOL, 0.1,
                                            untested_above=w.lr))
            self.stats.append(compare_table(f"{tag} partition {p} state", got_S, run.tab.S[p][rows], fs, STATE_RTOL, 0.0))
            qrows, qE, qS = quiet[p]
            still = ~np.isin(qrows, rows)
            qids = p * rp + qrows[still]
            assert np.array_equal(L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, qids, qids.size, d), qE[still])
            assert np.array_equal(L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, qids, qids.size, d), qS[still])
            # next call starts from the GPU's values
            run.tab.E[p][rows] = got_E
            run.tab.S[p][rows] = got_S
        if self.uses_rel:
            nrel = run.tab.RE.shape[0]
            got_E = L.legend_read_embeddings(ctx, L.TABLE_REL_EMB, None, nrel, d)
            got_S = L.legend_read_embeddings(ctx, L.TABLE_REL_STATE, None, nrel, d)
            compare_table(f"{tag} relation embeddings", got_E, run.tab.RE, run.fe_rel, EMB_RTOL, 0.1, untested_above=w.lr)
            compare_table(f"{tag} relation state", got_S, run.tab.RS, run.fs_rel, STATE_RTOL, 0.0)
            run.tab.RE[:] = got_E
            run.tab.RS[:] = got_S
            run.fe_rel[:] = 0
            run.fs_rel[:] = 0
            run.touched_rel[:] = False
        return run.last

    def assert_shares(self, min_plain_emb, max_untested):
        """Over all node-table comparisons of this setup: the share of embedding elements that agree at the
        plain 1e-5 * max(|theta|, lr) bound (no allowance) is at least min_plain_emb, and the share whose
        allowance exceeds a whole Adagrad step (so that the comparison says nothing) is at most max_untested."""
        emb = [s for s in self.stats if s["kind"] == "emb"]
        n = sum(s["n"] for s in emb)
        plain = sum(s["share_plain"] * s["n"] for s in emb) / n
        untested = sum(s["share_untested"] * s["n"] for s in emb) / n
        assert plain >= min_plain_emb, (plain, min_plain_emb)
        assert untested <= max_untested, (untested, max_untested)


def test_c1_whole_epoch_batch_by_batch():
    s = _Setup("c1")
    try:
        nb = -(-s.buckets[(0, 0)].shape[0] // s.w.batch_size)
        assert nb == 100
        for b in range(nb):
            s.check_batch(0, 0, b, check_indices=b in (0, nb - 1))
        s.assert_shares(_MIN_SHARE_AT_PLAIN_BOUND, _MAX_SHARE_UNTESTED)
    finally:
        s.close()


def test_c2_full_size_batches():
    """The workload bench.py times: 50 000 edges, 1 000 chunks of 50 with 1 000 negatives each."""
    s = _Setup("c2")
    try:
        s.check_batch(0, 1, 0)
        s.check_batch(2, 2, 0)
        s.check_batch(0, 1, 1, check_indices=False)
        s.assert_shares(_MIN_SHARE_AT_PLAIN_BOUND, _MAX_SHARE_UNTESTED)
    finally:
        s.close()


def test_c3_full_size_batches():
    """d = 400, both sides corrupted, 1 345 relations; the last batch is partial."""
    s = _Setup("c3")
    try:
        nb = -(-s.buckets[(0, 0)].shape[0] // s.w.batch_size)
        for b in (0, 1, nb - 1):
            s.check_batch(0, 0, b, check_indices=b != 1)
        s.assert_shares(_MIN_SHARE_AT_PLAIN_BOUND, _MAX_SHARE_UNTESTED)
    finally:
        s.close()


def test_c5_geometry_two_partitions_past_2_gib():
    """c5's table geometry: partitions of R_p = 5 375 000 rows (the E half of a slot is 2.15 GB, so byte offsets
    of rows, and of the whole state half, lie past 2^31), d = 100, ComplEx, both sides, 14 824 relations; two of
    c5's sixteen partitions, with c5's degree skew over their 10.75 M nodes.  One full batch of an off-diagonal and
    one of a diagonal bucket: about 1 M touched rows per partition compared element by element, 100 000 quiet rows
    bit-identical.  Tables: the library's seeded fill at standard deviation 0.1, read back for the oracle."""
    w = graphs.scaled(graphs.WORKLOADS["c5"], 8, 800, num_partitions=2)
    assert w.rows_per_partition == 5_375_000 and 4 * w.rows_per_partition * w.dim > 2 ** 31
    s = _Setup(w, seeded_fill=True, init_std=0.1)
    try:
        assert min(s.buckets[(0, 1)].shape[0], s.buckets[(1, 1)].shape[0]) >= w.batch_size
        last = s.check_batch(0, 1, 0)
        assert last[1][0].size > 900_000 and last[1][0].max() * w.dim * 4 > 2 ** 31       # rows past 2 GiB were compared
        last = s.check_batch(1, 1, 0, check_indices=False)
        assert last[1][0].size > 1_500_000
        s.assert_shares(_MIN_SHARE_AT_PLAIN_BOUND, _MAX_SHARE_UNTESTED)
    finally:
        s.close()


def test_c4_geometry_two_partitions_a_million_unique_rows():
    """c4's table geometry: partitions of 2.6 M rows, Dot, 1 000 uniform negatives per chunk of 50: about 0.8 M
    unique rows of the destination partition (1.0 M of both in the diagonal bucket) get a gradient per batch."""
    w = graphs.scaled(graphs.WORKLOADS["c4"], 8, 4000, num_partitions=2)
    assert w.rows_per_partition == 2_600_000
    s = _Setup(w, seeded_fill=True, init_std=0.1)
    try:
        assert min(s.buckets[(1, 0)].shape[0], s.buckets[(0, 0)].shape[0]) >= w.batch_size
        last = s.check_batch(1, 0, 0)
        assert last[0][0].size > 750_000
        last = s.check_batch(0, 0, 0, check_indices=False)
        assert last[0][0].size > 750_000
        s.assert_shares(_MIN_SHARE_AT_PLAIN_BOUND, _MAX_SHARE_UNTESTED)
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
