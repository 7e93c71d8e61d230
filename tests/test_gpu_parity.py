"""GPU parity: the HIP path (through the C ABI binding) against the CPU oracle, element by element."""
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


# ------------------------------------------------------------------ sc_segment
def test_segment_edge_cases():
    N = 40
    rows = [
        np.zeros(N, np.uint8),                                   # no delimiter: one chunk
        np.ones(N, np.uint8),                                    # all delimiters: N+1 empty chunks
        np.array([1] + [0] * (N - 2) + [1], np.uint8),           # leading and trailing delimiter
        np.array(([1, 1, 0, 0, 0] * 8), np.uint8),               # adjacent delimiters
    ]
    mask = np.stack(rows)
    g.check_segment(mask, None)
    g.check_segment(mask, np.array([0, 1, 17, 39], np.int32))    # ragged, including an empty sequence


@pytest.mark.parametrize("name", ["tiny", "layer32k", "long128k"])
def test_segment_workloads(name):
    w = wl.get_workload(name)
    mask = np.stack([wl.delimiter_mask(w, b) for b in range(w.batch)])
    g.check_segment(mask, None)


def test_segment_ragged_batch_and_unaligned_rows():
    w = wl.get_workload("batch_gqa7")
    lens = wl.seq_lens(w)[:6]
    mask = np.zeros((6, w.n_max + 3), np.uint8)
    for b in range(6):
        mask[b, : w.n_max] = wl.delimiter_mask(w, b)
    g.check_segment(mask, lens)                                   # row stride 16387: rows are not 16-byte aligned
    rng = np.random.default_rng(0)
    dense = (rng.random((3, 70001)) < 0.5).astype(np.uint8)      # several tiles, ragged tail, half delimiters
    g.check_segment(dense, np.array([70001, 33333, 16384], np.int32))


def test_segment_capacity_overflow_is_flagged():
    mask = torch.ones((2, 64), dtype=torch.uint8, device=g.DEV)
    mask[1, 5:] = 0
    off = torch.full((2, 10), -5, dtype=torch.int32, device=g.DEV)
    _, nch = sc.sc_segment(mask, None, offsets=off)
    torch.cuda.synchronize()
    assert nch.tolist() == [-1, 6]
    assert off[1, :7].tolist() == [0, 1, 2, 3, 4, 5, 65]
    # several tiles of mask per sequence, each filed by a workgroup of its own: none writes beyond the capacity
    mask = torch.ones((2, 70000), dtype=torch.uint8, device=g.DEV)
    mask[1, 40:69990] = 0
    wide = torch.full((2, 200), -5, dtype=torch.int32, device=g.DEV)
    _, nch = sc.sc_segment(mask, None, offsets=wide[:, :100])
    torch.cuda.synchronize()
    assert nch.tolist() == [-1, 51]
    assert wide[0, :100].tolist() == list(range(100)) and (wide[:, 100:] == -5).all()
    assert wide[1, :52].tolist() == list(range(41)) + list(range(69991, 70001)) + [70001]


# ------------------------------------------------------------------ sc_gsc_merge + sc_decode_attn
@pytest.mark.parametrize("tau", [0.7, 1.0, -1.01, 0.9745])
def test_tiny_full(tau):
    w = wl.get_workload("tiny")
    case = build_case(w, tau)
    out = g.check_compress(case)
    errs = g.check_decode(case, out, range(w.decode_steps))
    print("tiny tau=%g redraws=%d merge_err=%.2e decode_err=%s" % (tau, case["redraws"], out["worst_merge_err"], errs))


@pytest.mark.parametrize("name,n,tau", [("layer32k", 4096 + 37, 0.7), ("layer32k", 3000, 0.9745),
                                        ("long128k", 8192 + 5, 0.7), ("long128k", 6000, 0.03)])
def test_truncated_workloads(name, n, tau):
    # a few thousand tokens: several work items per head, chunks longer than one 64-row block, ragged tail
    w = wl.get_workload(name)
    case = build_case(w, tau, n_max=n, heads=3)
    out = g.check_compress(case)
    errs = g.check_decode(case, out, range(3), q_heads=3 * w.group)
    print(name, n, tau, "redraws", case["redraws"], "merge_err %.2e" % out["worst_merge_err"], "decode", errs)


@pytest.mark.parametrize("base,dtype,d", [("layer32k", "bf16", 64), ("tiny", "f32", 128), ("tiny", "bf16", 128)])
def test_other_dtype_and_head_dim_combinations(base, dtype, d):
    # the combinations the header promises beyond the two the workloads use (bf16 / 128 and fp32 / 64):
    # bf16 with d = 64 and fp32 with d = 128 through sc_gsc_merge (generic kernels) and sc_decode_attn
    import dataclasses
    w = dataclasses.replace(wl.get_workload(base), dtype=dtype, head_dim=d, kv_heads=2, q_heads=8)
    case = build_case(w, 0.7, n_max=1500 + 3)
    out = g.check_compress(case)
    errs = g.check_decode(case, out, range(3))
    print(base, dtype, d, "redraws", case["redraws"], "merge_err %.2e" % out["worst_merge_err"], "decode", errs)


def test_layer32k_full_size():
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7)
    out = g.check_compress(case)
    errs = g.check_decode(case, out, [0, 1, 31, 63])
    print("layer32k full: redraws", case["redraws"], "pairs/token %.2f" % (case["n_pairs"] / (8 * 32768)),
          "rows", out["comp_lens"].tolist(), "merge_err %.2e" % out["worst_merge_err"], "decode", errs)


def test_batch_ragged_gqa7():
    w = wl.get_workload("batch_gqa7")
    case = build_case(w, 0.975, n_max=2048, batch=5)
    assert len(set(case["seq_lens"].tolist())) > 1
    out = g.check_compress(case)
    lens = out["comp_lens"].cpu().numpy()
    assert len(set(lens.ravel().tolist())) > 4                     # per-sequence, per-head lengths differ
    errs = g.check_decode(case, out, range(2))
    print("gqa7 ragged: lens", lens.tolist(), "decode", errs)


def test_capacity_overflow_and_empty_sequences():
    w = wl.get_workload("tiny")
    case = build_case(w, 0.7)
    full = g.run_compress(case, torch.float32)
    rows = full["comp_lens"].cpu().numpy()
    cap = int(rows.min()) - 3
    small = g.run_compress(case, torch.float32, cap=cap)
    assert small["comp_lens"].tolist() == [[-1, -1]]
    assert sc.check_lengths(small["comp_lens"]) == 0 and sc.check_lengths(full["comp_lens"]) == -1
    assert torch.equal(small["Kc"][:, :, :cap], full["Kc"][:, :, :cap])
    assert torch.equal(small["counts"][:, :, :cap], full["counts"][:, :, :cap])
    # a sequence of length 0 gives an empty merged cache, and decode over it returns zeros
    case0 = build_case(w, 0.7)
    case0["seq_lens"] = np.array([0], np.int32)
    out0 = g.run_compress(case0, torch.float32)
    assert out0["comp_lens"].tolist() == [[0, 0]]
    Q = g.to_device(wl.queries(w, 0, 0), False)
    O, lse = sc.sc_decode_attn(Q, out0["Kc"], out0["Vc"], out0["counts"], out0["comp_lens"], want_lse=True)
    torch.cuda.synchronize()
    assert (O == 0).all() and torch.isinf(lse).all() and (lse < 0).all()


def test_zero_norm_and_duplicate_keys():
    # degenerate keys: zero rows never merge, exact duplicates merge at any tau < 1
    d = 64
    rng = np.random.default_rng(7)
    n = 200
    K = rng.standard_normal((n, d)).astype(np.float32)
    K[10] = 0; K[11] = 0; K[50] = K[40]; K[51] = K[40] * 3.0
    V = rng.standard_normal((n, d)).astype(np.float32)
    mask = np.zeros((1, n), np.uint8)
    mask[0, [30, 90, 91, 150]] = 1
    off = oracle.segment(mask[0], n)
    ref = oracle.compress_head(K, V, off, 0.999)
    Kd = torch.from_numpy(K).to(g.DEV).view(1, 1, n, d)
    Vd = torch.from_numpy(V).to(g.DEV).view(1, 1, n, d)
    offs, nch, _ = g.run_segment(mask, None)
    Kc, Vc, counts, lens, cid = sc.sc_gsc_merge(Kd, Vd, offs, nch, 0.999, want_cluster_id=True)
    torch.cuda.synchronize()
    assert lens.item() == ref["n_rows"]
    assert np.array_equal(cid[0, 0].cpu().numpy(), ref["cid"])
    assert np.array_equal(counts[0, 0, : ref["n_rows"]].cpu().numpy(), ref["counts"][: ref["n_rows"]])


def test_strided_kv_views():
    # K/V handed over as strided views of a [B, N, H, d] allocation (a common cache layout)
    w = wl.get_workload("tiny")
    case = build_case(w, 0.7)
    base = g.run_compress(case, torch.float32)
    K = torch.from_numpy(case["K"]).to(g.DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    V = torch.from_numpy(case["V"]).to(g.DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not K.is_contiguous()
    Kc, Vc, counts, lens, _ = sc.sc_gsc_merge(K, V, base["offsets"], base["num_chunks"], 0.7)
    torch.cuda.synchronize()
    assert torch.equal(lens, base["comp_lens"])
    for h in range(2):
        r = int(lens[0, h])
        assert torch.equal(Kc[0, h, :r], base["Kc"][0, h, :r]) and torch.equal(Vc[0, h, :r], base["Vc"][0, h, :r])
        assert torch.equal(counts[0, h, :r], base["counts"][0, h, :r])


def test_repeatable_bit_for_bit():
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7, n_max=5000, heads=2, exclude_near=False)
    a = g.run_compress(case, torch.bfloat16)
    ws = sc.decode_attn_workspace(1, 8, 2, 5000, 128, g.DEV)
    Q = g.to_device(wl.queries(w, 0, 0)[:, :8], True)
    O0, _ = sc.sc_decode_attn(Q, a["Kc"], a["Vc"], a["counts"], a["comp_lens"], workspace=ws)
    O0 = O0.clone()
    for _ in range(5):
        b = g.run_compress(case, torch.bfloat16)
        assert torch.equal(a["comp_lens"], b["comp_lens"]) and torch.equal(a["cid"], b["cid"])
        for h in range(2):
            r = int(a["comp_lens"][0, h])
            assert torch.equal(a["Kc"][0, h, :r], b["Kc"][0, h, :r]) and torch.equal(a["Vc"][0, h, :r], b["Vc"][0, h, :r])
            assert torch.equal(a["counts"][0, h, :r], b["counts"][0, h, :r])
        O1, _ = sc.sc_decode_attn(Q, a["Kc"], a["Vc"], a["counts"], a["comp_lens"], workspace=ws)
        torch.cuda.synchronize()
        # split partials are combined in a fixed order, so the result does not depend on arrival order
        assert torch.equal(O0, O1)


@pytest.mark.parametrize("knobs", [
    dict(gsc_chunks_per_task=1), dict(gsc_chunks_per_task=3, gsc_grid_x=16), dict(gsc_chunks_per_task=5),
    dict(gsc_chunks_per_task=32, gsc_grid_x=4), dict(gsc_grid_x=7), dict(gsc_fast_path=0),
    dict(gsc_fast_path=0, gsc_chunks_per_item=3, gsc_grid_x=5),
    dict(decode_mfma_min_group=1), dict(decode_mfma_min_group=9), dict(decode_max_splits=3, decode_min_rows=64),
])
def test_launch_shape_knobs_do_not_change_results(knobs):
    # other task sizes, grids narrower than the task count (workgroups then walk several tasks), the
    # generic kernels on the fast path's inputs, and single-row decode on either attention kernel:
    # same integers, merged rows and attention outputs within the same bounds
    w = wl.get_workload("long128k")
    case = build_case(w, 0.7, n_max=5000 + 11, heads=2)
    old = {k: sc.tune_get(k) for k in knobs}
    try:
        for k, v in knobs.items():
            sc.tune_set(k, v)
        out = g.check_compress(case)
        errs = g.check_decode(case, out, range(2), q_heads=2 * w.group)
    finally:
        for k, v in old.items():
            sc.tune_set(k, v)
    print(knobs, "merge_err %.2e" % out["worst_merge_err"], "decode", errs)


def test_decode_capacity_beyond_32bit_row_offsets():
    # the fast decode kernel addresses the rows of a (sequence, head) with 32-bit byte offsets; a cache
    # whose capacity does not fit is served by the generic kernel: same result within the decode tolerance
    rows, d, G = 3000 + 7, 128, 4
    rng = np.random.default_rng(11)
    Ks = torch.from_numpy(rng.standard_normal((1, 1, rows, d)).astype(np.float32)).to(g.DEV).to(torch.bfloat16)
    Vs = torch.from_numpy(rng.standard_normal((1, 1, rows, d)).astype(np.float32)).to(g.DEV).to(torch.bfloat16)
    cs = torch.from_numpy(rng.integers(1, 9, (1, 1, rows)).astype(np.int32)).to(g.DEV)
    lens = torch.tensor([[rows]], dtype=torch.int32, device=g.DEV)
    Q = torch.from_numpy(rng.standard_normal((1, G, d)).astype(np.float32)).to(g.DEV).to(torch.bfloat16)
    O_small, lse_small = sc.sc_decode_attn(Q, Ks, Vs, cs, lens, want_lse=True)
    cap = (1 << 31) // (d * 2) + 5
    Kb = torch.empty((1, 1, cap, d), dtype=torch.bfloat16, device=g.DEV)
    Vb = torch.empty_like(Kb)
    cb = torch.empty((1, 1, cap), dtype=torch.int32, device=g.DEV)
    Kb[:, :, :rows], Vb[:, :, :rows], cb[:, :, :rows] = Ks, Vs, cs
    O_big, lse_big = sc.sc_decode_attn(Q, Kb, Vb, cb, lens, want_lse=True)
    torch.cuda.synchronize()
    want_O, want_l = oracle.decode_attn(Q.float().cpu().numpy().astype(np.float64), Ks.float().cpu().numpy().astype(np.float64),
                                        Vs.float().cpu().numpy().astype(np.float64), cs.cpu().numpy(), lens.cpu().numpy())
    for O, lse in ((O_small, lse_small), (O_big, lse_big)):
        assert np.abs(O.float().cpu().numpy() - want_O).max() <= 4e-3 * max(1.0, np.abs(want_O).max())
        assert np.abs(lse.cpu().numpy() - want_l).max() <= 1e-3
