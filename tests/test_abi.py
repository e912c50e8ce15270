"""Host-side checks of the C ABI: the library loads, exports what the header declares,
and its host-only planner agrees with the oracle's reading of Alg. 1 / Alg. 2."""

import ctypes
import os
import re

import numpy as np
import pytest

from oracle import order

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "legend.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(legend_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2505_09258_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = _declared()
    assert {"legend_init_partitions", "legend_train_bucket", "legend_score_edges",
            "legend_read_embeddings"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_config_struct_layout_matches_header_field_order():
    from paper_2505_09258_amd import binding
    text = open(HEADER).read()
    body = text[text.index("typedef struct legend_config {"):text.index("} legend_config;")]
    fields = re.findall(r"^\s+(?:uint32_t|int32_t|int64_t|uint64_t|float|void\*)\s+(\w+);", body, flags=re.M)
    assert fields == [f[0] for f in binding.legend_config._fields_]
    assert ctypes.sizeof(binding.legend_config) == 112


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 8, 12, 16, 23])
def test_plan_order_equals_oracle_reading(n):
    from paper_2505_09258_amd import binding as L
    states, buckets, begin, overlap = L.legend_plan_order(n)
    want_states = order.loading_order(n)
    assert [tuple(int(x) for x in s) for s in states] == [tuple(s) for s in want_states]
    plan = order.iteration_order(want_states, n)
    assert len(plan) == len(states)
    seq = []
    for k, (ev, ld, before, during) in enumerate(plan):
        got_before = [tuple(map(int, b)) for b in buckets[begin[k]:overlap[k]]]
        got_during = [tuple(map(int, b)) for b in buckets[overlap[k]:begin[k + 1]]]
        assert got_before == before and got_during == during
        seq += before + during
    assert len(seq) == n * n == begin[-1]


def test_plan_order_rejects_bad_arguments():
    from paper_2505_09258_amd import binding as L
    with pytest.raises(L.LegendError):
        L.legend_plan_order(0)
    small = np.zeros((2, 3), np.int32)
    out = np.zeros((36, 2), np.int32)
    b = np.zeros(64, np.int32)
    ns = ctypes.c_int32(0)
    rc = L._lib.legend_plan_order(6, small.ctypes.data_as(ctypes.c_void_p), 2, ctypes.byref(ns),
                                  out.ctypes.data_as(ctypes.c_void_p), b.ctypes.data_as(ctypes.c_void_p),
                                  b.ctypes.data_as(ctypes.c_void_p))
    assert rc == L.LEGEND_E_INVAL and ns.value == 8


def test_profile_names():
    from paper_2505_09258_amd import binding as L
    names = []
    k = 0
    while L.legend_profile_name(k) is not None:
        names.append(L.legend_profile_name(k))
        k += 1
    assert names == ["prepare", "sort", "chunk", "update", "chunk_redo", "misc", "update_long"]
