"""GPU parity on the chunking variants of the paper's ablation (Sec. 3.4, Table 4): the same keys and
values, but chunk boundaries every 64 tokens, or none at all (the whole sequence is one chunk).
Same comparisons and tolerances as for the delimiter-bounded chunks."""
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
    print("%s: checked %d of %d (b,h); chunks %s; ratio %.2fx; merge_err %.2e; decode %s"
          % (tag, len(case["ref"]), lens.size, case["num_chunks"].tolist(), tokens / max(1, int(lens.sum())),
             out["worst_merge_err"], errs))


@pytest.mark.parametrize("n,sample", [(4096 + 37, None), (None, [(0, 0), (0, 5)])])
def test_fixed_blocks_of_64(n, sample):
    # every task is two chunks of 63 + 1 tokens that never share a window; blocks cut across the
    # semantic structure of the keys, so a block holds pieces of several mixtures
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7, n_max=n, heads=3 if n else None, sample=sample, chunking="fixed")
    assert (case["mask"][0, 63::64] == 1).all() and int(case["mask"][0].sum()) == case["mask"].shape[1] // 64
    out = g.check_compress(case)
    if sample is None:
        errs = g.check_decode(case, out, range(2), q_heads=3 * w.group)
    else:
        errs = g.check_decode_sampled(case, out, [0, w.decode_steps - 1])
    _report("fixed-64 n=%s" % n, case, out, errs)


@pytest.mark.parametrize("n,heads,sample", [(1000, 2, None), (8192 + 11, 2, None), (None, None, [(0, 3)])])
def test_one_chunk_for_the_whole_sequence(n, heads, sample):
    # no boundary: Alg. 1 runs over all tokens of a head, thousands of clusters in one chunk
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7, n_max=n, heads=heads, sample=sample, chunking="global")
    assert case["num_chunks"].tolist() == [1] and not case["mask"].any()
    out = g.check_compress(case)
    if sample is None:
        errs = g.check_decode(case, out, range(2), q_heads=heads * w.group)
    else:
        errs = g.check_decode_sampled(case, out, [0])
    _report("global n=%s" % n, case, out, errs)
