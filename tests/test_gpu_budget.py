"""GPU parity for sc_gsc_merge_budget: the bisection on the device must probe the thresholds the oracle's
bisection probes (every probe's row count is an integer the two sides agree on exactly), end on the
same fp32 threshold, and leave the merged cache of that threshold in the outputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_14303_amd import binding as sc
from paper_2603_14303_amd import workloads as wl
from helpers import build_case

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_common as g


def _oracle_rows(case, heads):
    cache = {}

    def rows_at(tau):
        if tau not in cache:
            tot = 0
            for b in range(case["K"].shape[0]):
                n = int(case["seq_lens"][b])
                for h in range(heads):
                    tot += oracle.compress_head(case["K"][b, h, :n], case["V"][b, h, :n], case["offsets"][b], tau)["n_rows"]
            cache[tau] = tot
        return cache[tau]
    return rows_at


@pytest.mark.parametrize("name,n,heads,fracs,iters", [
    ("tiny", None, 2, (0.2, 0.5, 0.95), 12),                 # fp32, d = 64: generic kernels
    ("layer32k", 4096 + 37, 2, (0.2, 0.35), 10),             # bf16 fast path; budgets of the paper
    ("batch_gqa7", 1536, 2, (0.35,), 8),                     # ragged batch
])
def test_budget_search_matches_oracle(name, n, heads, fracs, iters):
    w = wl.get_workload(name)
    batch = 3 if name == "batch_gqa7" else None
    case = build_case(w, 0.7, n_max=n, heads=heads, batch=batch, exclude_near=False)
    bf16 = w.dtype == "bf16"
    K, V = g.to_device(case["K"], bf16), g.to_device(case["V"], bf16)
    off, nch, sl = g.run_segment(case["mask"], case["seq_lens"])
    rows_at = _oracle_rows(case, heads)
    total = int(case["seq_lens"].sum()) * heads
    for frac in fracs:
        budget = int(round(frac * total))
        want_tau, probed = oracle.tau_for_budget(rows_at, budget, -1.01, 1.0, iters)
        Kc, Vc, counts, lens, cid, tau, rows = sc.sc_gsc_merge_budget(K, V, off, nch, budget, -1.01, 1.0, iters, seq_lens=sl,
                                                                      out_dtype=torch.float32, want_cluster_id=True)
        torch.cuda.synchronize()
        got_tau = tau.cpu().numpy()[0]
        assert got_tau == want_tau, (frac, got_tau, want_tau, probed)
        assert int(rows.item()) == rows_at(float(want_tau)) == int(lens.sum().item())
        if rows_at(-1.01) <= budget:
            assert int(rows.item()) <= budget
        # the outputs are those of a plain call at that threshold
        Kc2, Vc2, counts2, lens2, cid2 = sc.sc_gsc_merge(K, V, off, nch, float(got_tau), seq_lens=sl,
                                                         out_dtype=torch.float32, want_cluster_id=True)
        torch.cuda.synchronize()
        assert torch.equal(lens, lens2) and torch.equal(cid, cid2)
        for b in range(K.shape[0]):
            for h in range(heads):
                r = int(lens[b, h])
                assert torch.equal(counts[b, h, :r], counts2[b, h, :r])
                assert torch.equal(Kc[b, h, :r], Kc2[b, h, :r]) and torch.equal(Vc[b, h, :r], Vc2[b, h, :r])
        print(name, "budget %.2f -> tau %.6f rows %d of %d (%.1f %%)" % (frac, got_tau, int(rows.item()), total,
                                                                      100.0 * int(rows.item()) / total))
    # no iterations: the call is sc_gsc_merge at tau_lo
    _, _, _, lens0, _, tau0, rows0 = sc.sc_gsc_merge_budget(K, V, off, nch, total, 0.7, 0.9, 0, seq_lens=sl)
    torch.cuda.synchronize()
    assert tau0.item() == np.float32(0.7) and int(rows0.item()) == rows_at(0.7) == int(lens0.sum().item())
    # a capacity that the probes overflow counts as "over budget" and the search still ends below it
    small_cap = max(8, int(lens0.max().item()) + 4)
    out = sc.sc_gsc_merge_budget(K, V, off, nch, total, -1.01, 1.0, iters, seq_lens=sl, cap=small_cap)
    torch.cuda.synchronize()
    assert (out[3] >= 0).all() and (out[3] <= small_cap).all()


def test_budget_search_replays_from_a_graph():
    # the whole search is a fixed sequence of launches: capture it once, replay it with other work and
    # synchronisations in between, and get the eager result every time
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7, n_max=2048 + 5, heads=2, exclude_near=False)
    K, V = g.to_device(case["K"], True), g.to_device(case["V"], True)
    off, nch, sl = g.run_segment(case["mask"], case["seq_lens"])
    budget = int(0.3 * 2 * int(case["seq_lens"][0]))
    eager = sc.sc_gsc_merge_budget(K, V, off, nch, budget, -1.01, 1.0, 9, seq_lens=sl)
    torch.cuda.synchronize()
    ws = sc.Workspace(sc.load_library().sc_gsc_merge_budget_workspace_bytes(1, 2, K.shape[2], 128), g.DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        warm = sc.sc_gsc_merge_budget(K, V, off, nch, budget, -1.01, 1.0, 9, seq_lens=sl, workspace=ws)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            out = sc.sc_gsc_merge_budget(K, V, off, nch, budget, -1.01, 1.0, 9, seq_lens=sl, workspace=ws)
    torch.cuda.synchronize()
    for replay in range(3):
        out[5].zero_(); out[3].zero_(); out[0].zero_()
        scratch = torch.randn(1 << 20, device=g.DEV).sum()          # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert out[5].item() == eager[5].item() and out[6].item() == eager[6].item(), replay
        assert torch.equal(out[3], eager[3])
        for h in range(2):
            r = int(eager[3][0, h])
            assert torch.equal(out[0][0, h, :r], eager[0][0, h, :r]) and torch.equal(out[2][0, h, :r], eager[2][0, h, :r])
        del scratch
