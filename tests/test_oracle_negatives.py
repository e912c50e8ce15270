"""Pins for the oracle's integer side: hash, range reduction, negative ids, touched rows."""

import numpy as np
import pytest

from oracle import negatives
from oracle.bucket import OracleConfig

M64 = (1 << 64) - 1


def test_mix64_matches_published_splitmix64_stream():
    # First outputs of the splitmix64 generator seeded with 0 (Vigna's reference
    # stream): state advances by the golden-ratio constant, output = mix64(state).
    expect = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state = 0
    for want in expect:
        state = (state + negatives.GOLDEN) & M64
        assert int(negatives.mix64(np.uint64(state))) == want


def test_fold_first_step_is_splitmix_output():
    assert int(negatives.fold(np.uint64(0), 0)) == 0xE220A8397B1DCDAF


def test_mulhi64_against_big_integers():
    rng = np.random.default_rng(1)
    a = rng.integers(0, 1 << 64, size=2000, dtype=np.uint64)
    a[:4] = [0, 1, M64, 1 << 63]
    for b in (1, 2, 3, 64, 10_000, 1_200_000, 5_375_000, (1 << 32) - 1, 1 << 32, (1 << 40) + 12345, M64):
        got = negatives.mulhi64(a, b)
        want = [(int(x) * b) >> 64 for x in a]
        assert [int(g) for g in got] == want


def _py_fold(h, f):
    z = (h + negatives.GOLDEN + f) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_chunk_hash_field_order_bruteforce():
    # scalar big-integer walk over the tuple (seed, epoch, i, j, b, c, side, k)
    seed, epoch, i, j, b, c, side = 0xDEADBEEFCAFEF00D, 3, 2, 1, 17, 5, 1
    h = negatives.chunk_hash(seed, epoch, i, j, b, c, side, 9)
    for k in range(9):
        x = seed
        for f in (epoch, i, j, b, c, side, k):
            x = _py_fold(x, f)
        assert int(h[k]) == x
    # every field matters
    base = [int(v) for v in h]
    for alt in [(seed + 1, epoch, i, j, b, c, side), (seed, epoch + 1, i, j, b, c, side),
                (seed, epoch, j, i, b, c, side), (seed, epoch, i, j, b + 1, c, side),
                (seed, epoch, i, j, b, c + 1, side), (seed, epoch, i, j, b, c, 0)]:
        assert [int(v) for v in negatives.chunk_hash(*alt, 9)] != base


def _cfg(**kw):
    d = dict(num_nodes=1000, num_relations=0, dim=4, num_partitions=3, batch_size=40, chunk_size=8,
             num_negs=16, num_degree_negs=0, seed=7)
    d.update(kw)
    return OracleConfig(**d)


def test_rows_valid_and_range_of_uniform_ids():
    cfg = _cfg()
    rp = cfg.rows_per_partition
    assert rp == 334
    assert [negatives.rows_valid(1000, 3, p) for p in range(3)] == [334, 334, 332]
    edges = np.zeros((10, 3), np.int32)
    for part in range(3):
        ids = np.concatenate([negatives.chunk_negatives(cfg, 0, 0, part, b, 0, negatives.SIDE_DST, edges)
                              for b in range(200)])
        assert ids.min() >= 0 and ids.max() < negatives.rows_valid(1000, 3, part)
    # source-side corruption draws from the source partition
    ids = np.concatenate([negatives.chunk_negatives(cfg, 0, 2, 0, b, 0, negatives.SIDE_SRC, edges)
                          for b in range(200)])
    assert ids.max() < 332 and ids.max() > 300


def test_uniform_ids_chi_square():
    cfg = _cfg(num_nodes=64, num_partitions=1, num_negs=4096)
    edges = np.zeros((1, 3), np.int32)
    ids = np.concatenate([negatives.chunk_negatives(cfg, 0, 0, 0, b, 0, 0, edges) for b in range(32)])
    counts = np.bincount(ids, minlength=64)
    expected = ids.size / 64
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    # 63 degrees of freedom: mean 63, sd ~11.2; a broken reducer is off by orders of magnitude
    assert 20 < chi2 < 130


def test_degree_weighted_ids_follow_in_bucket_degree():
    cfg = _cfg(num_nodes=50, num_partitions=1, num_negs=2000, num_degree_negs=1000)
    # bucket in which destination 7 has 60 % of the edges, destination 9 the rest
    edges = np.zeros((1000, 3), np.int32)
    edges[:, 0] = np.arange(1000) % 50
    edges[:600, 2] = 7
    edges[600:, 2] = 9
    ids = negatives.chunk_negatives(cfg, 1, 0, 0, 0, 0, negatives.SIDE_DST, edges)
    uni, deg = ids[:1000], ids[1000:]
    assert set(np.unique(deg)) == {7, 9}
    assert abs((deg == 7).mean() - 0.6) < 0.06
    assert len(np.unique(uni)) > 40               # the uniform half covers the table
    # source side takes the source column
    ids_s = negatives.chunk_negatives(cfg, 1, 0, 0, 0, 0, negatives.SIDE_SRC, edges)
    assert len(np.unique(ids_s[1000:])) > 40


def test_touched_rows_bruteforce_diagonal_and_offdiagonal():
    for (i, j) in ((0, 0), (0, 1)):
        for score in (0, 1):
            cfg = _cfg(num_nodes=60, num_partitions=2, num_negs=5, chunk_size=4, batch_size=10,
                       corrupt=2, score=score, num_relations=3 if score else 0)
            rng = np.random.default_rng(3)
            edges = rng.integers(0, 30, size=(10, 3)).astype(np.int32)
            edges[:, 1] = rng.integers(0, 3, size=10)
            neg = negatives.batch_negatives(cfg, 0, i, j, 0, edges, edges)
            assert neg.shape == (2, 3, 5)
            want = set()
            for e in edges:
                want.add((0, int(e[0])))
                want.add((0 if i == j else 1, int(e[2])))
                if score:
                    want.add((2, int(e[1])))
            for x in neg[0].ravel():            # dst-side negatives live in partition j
                want.add((0 if i == j else 1, int(x)))
            for x in neg[1].ravel():            # src-side negatives live in partition i
                want.add((0, int(x)))
            got = negatives.touched_rows(cfg, i, j, edges, neg)
            assert [(int(k) >> 32, int(k) & 0xFFFFFFFF) for k in got] == sorted(want)


def test_partial_last_chunk_still_draws_all_negatives():
    cfg = _cfg(batch_size=10, chunk_size=4, num_negs=6)
    edges = np.zeros((10, 3), np.int32)
    neg = negatives.batch_negatives(cfg, 0, 0, 0, 0, edges[:10], edges)
    assert neg.shape == (1, 3, 6)
