"""The seeded input generator: reproducible, bf16-exact where it says so, shaped as documented, and free
of the method's arithmetic (it is shared by the oracle's tests and the HIP path's tests)."""
import ast
import os

import numpy as np

from paper_2603_14303_amd import workloads as wl


def test_inputs_are_reproducible_and_bf16_exact():
    w = wl.get_workload("layer32k")
    m1, m2 = wl.delimiter_mask(w, 0), wl.delimiter_mask(w, 0)
    assert np.array_equal(m1, m2) and m1.dtype == np.uint8 and m1.shape == (w.n_max,)
    gaps = np.diff(np.concatenate([[-1], np.nonzero(m1)[0]]))
    assert gaps.min() >= 1 and gaps.max() <= w.gap_cap and 20 < gaps.mean() < 28      # min(Geom(1/24), 128)
    K1, V1 = wl.keys_values(w, 0, 0, 3, m1, 4096)
    K2, V2 = wl.keys_values(w, 0, 0, 3, m1, 4096)
    assert np.array_equal(K1, K2) and np.array_equal(V1, V2)
    assert np.array_equal(wl.round_to_bf16(K1), K1) and np.array_equal(wl.round_to_bf16(V1), V1)
    K3, _ = wl.keys_values(w, 1, 0, 3, m1, 4096)                                      # another layer: other keys
    assert not np.array_equal(K1, K3)
    q = wl.queries(w, 0, 5)
    assert q.shape == (w.batch, w.q_heads, w.head_dim) and np.array_equal(wl.round_to_bf16(q), q)


def test_ragged_lengths_and_workload_table():
    names = [w.name for w in wl.WORKLOADS] if not isinstance(wl.WORKLOADS, dict) else list(wl.WORKLOADS)
    assert {"tiny", "layer32k", "stack32k", "long128k", "batch_gqa7"} <= set(names)
    w = wl.get_workload("batch_gqa7")
    lens = wl.seq_lens(w)
    lo, hi = w.ragged
    assert lens.shape == (w.batch,) and lens.min() >= lo and lens.max() <= hi and len(set(lens.tolist())) > 16
    assert w.q_heads // w.kv_heads == 7 == w.group


def test_chunking_variants():
    w = wl.get_workload("layer32k")
    m = wl.delimiter_mask(w, 0)
    n = 1000
    assert np.array_equal(wl.variant_mask("delimiters", m, n), m)
    f = wl.variant_mask("fixed", m, n)
    assert np.array_equal(np.nonzero(f)[0], np.arange(63, n, 64))
    assert not wl.variant_mask("global", m, n).any()
    try:
        wl.variant_mask("other", m, n)
        assert False
    except ValueError:
        pass


def test_generator_holds_none_of_the_methods_arithmetic():
    # no similarity, clustering, merging or attention in the module that both sides draw inputs from
    src = open(os.path.join(os.path.dirname(wl.__file__), "workloads.py")).read()
    tree = ast.parse(src)
    names = {n.id for n in ast.walk(tree) if isinstance(n, ast.Name)} | {n.attr for n in ast.walk(tree) if isinstance(n, ast.Attribute)}
    assert not names & {"oracle", "binding", "softmax", "exp", "log", "dot", "matmul", "norm", "einsum"}
    imported = {a.name for n in ast.walk(tree) if isinstance(n, ast.Import) for a in n.names} | \
               {n.module for n in ast.walk(tree) if isinstance(n, ast.ImportFrom)}
    assert imported <= {"__future__", "dataclasses", "typing", "numpy"}
