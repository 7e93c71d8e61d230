"""GPU parity at the full sizes of the benchmark configurations, in the default launch configuration.

The kernels run on the complete shape of one layer; the oracle recomputes the listed (sequence, head)
problems in full (every cluster index, size and merged row) and, for decode, every query head of those
problems.  Inputs are generated for the whole layer either way.
"""
import numpy as np
import pytest
import torch

import gpu_common as g
from helpers import build_case
from paper_2603_14303_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _report(tag, case, out, errs):
    lens = out["comp_lens"].cpu().numpy()
    tokens = int(case["seq_lens"].sum()) * lens.shape[1]
    print("%s: checked %d of %d (b,h); redraws %d; ratio %.2fx; merge_err %.2e; decode %s"
          % (tag, len(case["ref"]), lens.size, case["redraws"], tokens / max(1, int(lens.sum())),
             out["worst_merge_err"], errs))


@pytest.mark.parametrize("tau_index,layer,sample", [
    (0, 0, None),                                                       # whole layer
    (1, 16, [(0, h) for h in range(8)] + [(1, 1), (2, 6), (3, 3)]),     # sequence 0 in full + one head each
    (2, 31, [(0, h) for h in range(8)] + [(1, 7), (2, 0), (3, 4)]),
])
def test_stack32k_layer(tau_index, layer, sample):
    w = wl.get_workload("stack32k")
    tau = w.taus[tau_index]
    case = build_case(w, tau, layer=layer, sample=sample)
    out = g.check_compress(case)
    errs = g.check_decode_sampled(case, out, [0, w.decode_steps - 1])
    _report("stack32k tau=%g layer=%d" % (tau, layer), case, out, errs)


def test_long128k_full():
    w = wl.get_workload("long128k")
    case = build_case(w, w.taus[0])
    out = g.check_compress(case)
    errs = g.check_decode_sampled(case, out, [0, w.decode_steps - 1])
    _report("long128k", case, out, errs)


@pytest.mark.parametrize("tau_index,layer", [(0, 0), (1, 27)])
def test_batch_gqa7_full(tau_index, layer):
    w = wl.get_workload("batch_gqa7")
    tau = w.taus[tau_index]
    lens = wl.seq_lens(w)
    order = np.argsort(lens)
    # shortest, longest and a spread of sequences in between, heads rotating
    picks = [int(order[0]), int(order[-1])] + [int(b) for b in order[3:-1:4]]
    sample = [(b, i % w.kv_heads) for i, b in enumerate(picks)]
    case = build_case(w, tau, layer=layer, sample=sample)
    assert len(set(case["seq_lens"].tolist())) > 16
    out = g.check_compress(case)
    got = out["comp_lens"].cpu().numpy()
    assert (got > 0).all() and len(set(got.ravel().tolist())) > 32
    errs = g.check_decode_sampled(case, out, [0, w.decode_steps - 1])
    _report("batch_gqa7 tau=%g layer=%d" % (tau, layer), case, out, errs)
