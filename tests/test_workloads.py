"""Input generators: the per-bucket edge generator draws from the law of the whole-graph generator."""

import numpy as np

from workloads import graphs


def test_bucket_generator_follows_the_law_of_the_whole_graph_generator():
    w = graphs.scaled(graphs.WORKLOADS["c5"], 2000, 200)          # 43 000 nodes, 1.69 M edges, 16 partitions, relations
    src, rel, dst = graphs.generate_edges(w, 3)
    full = graphs.bucket_edges(w, src, rel, dst)
    wanted = [(0, 1), (2, 2), (5, 0)]
    sub, share = graphs.generate_bucket_edges(w, 3, wanted)
    rp = w.rows_per_partition
    assert abs(sum(share.values()) - 3 / 256) < 0.01
    for key in wanted:
        e, f = sub[key], full[key]
        assert e.dtype == np.int32 and e.shape[1] == 3
        assert e[:, [0, 2]].min() >= 0 and e[:, [0, 2]].max() < rp and e[:, 1].min() >= 0 and e[:, 1].max() < w.num_relations
        expected = share[key] * w.num_edges
        # bucket sizes: both are Binomial(E, share) draws
        assert abs(e.shape[0] - expected) < 6 * np.sqrt(expected) and abs(f.shape[0] - expected) < 6 * np.sqrt(expected)
        # endpoint and relation frequencies: two-sample chi-square over the 40 most frequent values (+ the rest)
        for col, size in ((0, rp), (2, rp), (1, w.num_relations)):
            a = np.bincount(e[:, col], minlength=size).astype(np.float64)
            b = np.bincount(f[:, col], minlength=size).astype(np.float64)
            top = np.argsort(-(a + b))[:40]
            a = np.append(a[top], a.sum() - a[top].sum())
            b = np.append(b[top], b.sum() - b[top].sum())
            k1, k2 = np.sqrt(b.sum() / a.sum()), np.sqrt(a.sum() / b.sum())
            chi2 = (((k1 * a - k2 * b) ** 2) / (a + b)).sum()
            assert chi2 < 90.0, (key, col, chi2)                 # 40 degrees of freedom: 90 is beyond the 1e-5 tail
    # deterministic in the seed
    again, _ = graphs.generate_bucket_edges(w, 3, wanted[:1])
    assert np.array_equal(again[(0, 1)], sub[(0, 1)])
