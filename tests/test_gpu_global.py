"""GPU parity of sc_gsc_merge_global (Alg. 1 over the whole sequence as one chunk: the "no chunking"
variant of the paper's ablation, Sec. 3.4) against the oracle run on one-chunk offsets: cluster ids,
sizes and lengths bit for bit, merged rows and decode within the bounds of gpu_common."""
import dataclasses

import numpy as np
import pytest
import torch

import gpu_common as g
from helpers import build_case
from paper_2603_14303_amd import binding as sc
from paper_2603_14303_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _global_case(w, tau, **kw):
    case = build_case(w, tau, chunking="global", **kw)
    assert case["num_chunks"].tolist() == [1] * len(case["num_chunks"]) and not case["mask"].any()
    case["global_call"] = True
    return case


@pytest.mark.parametrize("n,heads,tau", [(63, 2, 0.7), (64, 1, 0.7), (1000, 2, 0.7), (8192 + 11, 2, 0.7),
                                         (3000, 2, 0.9745), (2000, 1, 1.0), (2000, 1, -1.01)])
def test_dedicated_path(n, heads, tau):
    # blocks of 64 rows: less than one, exactly one, many with a ragged tail; a threshold inside the band of
    # the similarities (pairs decided in fp64, many clusters); no merging at all; everything in one cluster
    w = wl.get_workload("layer32k")
    case = _global_case(w, tau, n_max=n, heads=heads, exclude_near=(tau == 0.7))
    out = g.check_compress(case)
    errs = g.check_decode(case, out, range(2), q_heads=heads * w.group)
    print("global n=%d tau=%g: rows %s merge_err %.2e decode %s" % (n, tau, out["comp_lens"].tolist(), out["worst_merge_err"], errs))


def test_full_length_one_head_checked():
    # 32768 tokens, all 8 heads computed, the oracle recomputes one of them (thousands of clusters in one chunk)
    w = wl.get_workload("layer32k")
    case = _global_case(w, 0.7, sample=[(0, 3)])
    out = g.check_compress(case)
    errs = g.check_decode_sampled(case, out, [0])
    print("global full: rows", out["comp_lens"].tolist(), "merge_err %.2e" % out["worst_merge_err"], "decode", errs)


def test_ragged_batch_and_capacity():
    w = dataclasses.replace(wl.get_workload("batch_gqa7"), batch=3, kv_heads=2, q_heads=14)
    case = _global_case(w, 0.7, n_max=1500, batch=3)
    assert len(set(case["seq_lens"].tolist())) > 1
    out = g.check_compress(case)
    rows = out["comp_lens"].cpu().numpy()
    cap = int(rows.max()) - 1
    small = g.run_compress(case, torch.float32, cap=cap)
    got = small["comp_lens"].cpu().numpy()
    assert ((got == -1) == (rows > cap)).all() and (got[rows <= cap] == rows[rows <= cap]).all()
    for b in range(rows.shape[0]):
        for h in range(rows.shape[1]):
            r = min(int(rows[b, h]), cap)      # a head that does not fit still gets its first cap rows
            assert torch.equal(small["counts"][b, h, :r], out["counts"][b, h, :r])
            assert torch.equal(small["Kc"][b, h, :r], out["Kc"][b, h, :r]) and torch.equal(small["Vc"][b, h, :r], out["Vc"][b, h, :r])


@pytest.mark.parametrize("base,knob", [("tiny", None), ("layer32k", "gsc_fast_path")])
def test_other_shapes_go_through_the_ordinary_kernels(base, knob):
    # fp32 / d = 64, and bf16 / d = 128 with the dedicated path switched off: same call, same comparisons
    w = wl.get_workload(base)
    old = sc.tune_get(knob) if knob else None
    try:
        if knob:
            sc.tune_set(knob, 0)
        case = _global_case(w, 0.7, n_max=700, heads=2)
        out = g.check_compress(case)
    finally:
        if knob:
            sc.tune_set(knob, old)
    print(base, "rows", out["comp_lens"].tolist(), "merge_err %.2e" % out["worst_merge_err"])
