"""Seeded initial embeddings of legend_init_partitions (both init pointers NULL): the values the
header documents, bit for bit, and their first two moments."""

import numpy as np
import pytest

from oracle import negatives as oneg

pytestmark = pytest.mark.gpu

TAG_NODE, TAG_REL = 0x6E6F6465, 0x72656C73


def _documented_fill(seed, tag, rows, dim, init_std):
    """value(g, k) = float(u - 131070) * float(init_std * sqrt(3) / 65536), u the sum of the four
    16-bit fields of fold(fold(fold(seed, tag), g), k) -- written out from the header's text."""
    h = oneg.fold(np.uint64(seed), tag)
    h = oneg.fold(np.full(rows, h, np.uint64), np.arange(rows, dtype=np.uint64))
    h = oneg.fold(np.repeat(h, dim), np.tile(np.arange(dim, dtype=np.uint64), rows))
    m = np.uint64(0xFFFF)
    u = (h & m) + ((h >> np.uint64(16)) & m) + ((h >> np.uint64(32)) & m) + (h >> np.uint64(48))
    scale = np.float32(np.float64(np.float32(init_std)) * 1.7320508075688772 / 65536.0)
    return ((u.astype(np.int64) - 131070).astype(np.float32) * scale).reshape(rows, dim)


@pytest.mark.parametrize("score,nrel", [(0, 0), (1, 37)], ids=["dot", "distmult"])
def test_seeded_fill_is_the_documented_function_of_the_seed(score, nrel):
    from paper_2505_09258_amd import binding as L
    V, d, n, std, seed = 10_003, 36, 3, 0.02, 0xC0FFEE12345
    cfg = L.make_config(num_nodes=V, dim=d, num_partitions=n, num_relations=nrel, score=score, batch_size=64,
                        chunk_size=8, num_negs=8, init_std=std, seed=seed)
    ctx = L.legend_init_partitions(cfg, None, None)
    try:
        host = L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, None, V, d)        # from the host tier
        for p in range(n):
            L.legend_swap_partition(ctx, -1, p)
        dev = L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, None, V, d)         # from the buffer slots
        want = _documented_fill(seed, TAG_NODE, V, d, std)
        assert np.array_equal(host, want) and np.array_equal(dev, want)
        assert abs(float(want.mean())) < 4 * std / np.sqrt(want.size)
        assert abs(float(want.std()) / std - 1.0) < 0.01
        assert not L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, None, V, d).any()
        rel = L.legend_read_embeddings(ctx, L.TABLE_REL_EMB, None, max(nrel, 1), d)
        if score == 0:
            assert not rel.any()
        else:
            assert np.array_equal(rel, _documented_fill(seed, TAG_REL, nrel, d, std))
    finally:
        L.legend_destroy(ctx)


def test_seeded_fill_needs_a_positive_init_std():
    from paper_2505_09258_amd import binding as L
    cfg = L.make_config(num_nodes=100, dim=8, batch_size=8, chunk_size=4, num_negs=4, init_std=0.0)
    with pytest.raises(L.LegendError) as ei:
        L.legend_init_partitions(cfg, None, None)
    assert ei.value.code == L.LEGEND_E_INVAL
