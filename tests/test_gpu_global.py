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


def _run_rows(K, V, tau):
    """K, V [n, 128] float arrays (bf16-exact) as one (sequence, head): GPU call and oracle on one-chunk offsets."""
    import oracle
    n = K.shape[0]
    Kd = torch.from_numpy(K).to(g.DEV).to(torch.bfloat16).view(1, 1, n, 128)
    Vd = torch.from_numpy(V).to(g.DEV).to(torch.bfloat16).view(1, 1, n, 128)
    Kc, Vc, counts, lens, cid = sc.sc_gsc_merge_global(Kd, Vd, tau, out_dtype=torch.float32, want_cluster_id=True)
    torch.cuda.synchronize()
    ref = oracle.compress_head(K.astype(np.float64), V.astype(np.float64), np.array([0, n + 1], np.int32), tau)
    assert lens.item() == ref["n_rows"]
    assert np.array_equal(cid[0, 0].cpu().numpy(), ref["cid"])
    r = ref["n_rows"]
    assert np.array_equal(counts[0, 0, :r].cpu().numpy(), ref["counts"][:r])
    assert g.rowwise_err(Kc[0, 0, :r].cpu().numpy(), ref["Kc"][:r]) <= 1e-3
    assert g.rowwise_err(Vc[0, 0, :r].cpu().numpy(), ref["Vc"][:r]) <= 1e-3
    return ref


def _bf16_exact(x):
    return torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).float().numpy()


def test_more_candidates_than_a_list_holds_and_none_is_a_seed():
    # Row j resembles 40 rows b_k of an earlier block, all of which were absorbed by a seed that j does not
    # resemble; the seed that does take j comes after them.  j's candidate list (32 entries) then holds no
    # seed although j has one: the kernel must go back to the bit arrays.  Unit vectors in a plane:
    # a at 0, b_k at 18, j at 36, s at 50 degrees, tau = 0.9 (cos 18 = 0.951, cos 36 = 0.809, cos 14 = 0.970, cos 32 = 0.848).
    rng = np.random.default_rng(3)
    n, d = 200, 128
    e0, e1 = np.zeros(d), np.zeros(d)
    e0[5], e1[77] = 1.0, 1.0

    def at(deg, scale=1.0):
        return scale * (np.cos(np.radians(deg)) * e0 + np.sin(np.radians(deg)) * e1)
    K = np.zeros((n, d))
    filler = rng.standard_normal((n, d))
    filler[:, 5] = 0
    filler[:, 77] = 0                      # orthogonal to the plane: resembles nothing in it
    K[:] = filler
    K[0] = at(0)
    for k in range(40):
        K[3 + k] = at(18, 1.0 + 0.1 * k)    # block 0: absorbed by row 0
    K[70] = at(50)                          # block 1: a seed (resembles neither a nor the b_k)
    K[150] = at(36)                         # block 2: candidates = 40 b_k (no seeds) and then row 70
    K[151] = at(36.5, 3.0)
    K = _bf16_exact(K)
    V = _bf16_exact(rng.standard_normal((n, d)))
    ref = _run_rows(K, V, 0.9)
    assert ref["cid"][150] == ref["cid"][70] and ref["cid"][3] == ref["cid"][0] and ref["cid"][150] != ref["cid"][0]


def test_zero_rows_duplicates_and_scaled_rows():
    # zero rows resemble nothing (also inside a block and across blocks), exact duplicates and scaled copies merge
    rng = np.random.default_rng(5)
    n, d = 300, 128
    K = rng.standard_normal((n, d))
    K[10] = 0; K[11] = 0; K[200] = 0
    K[50] = K[40]; K[130] = K[40] * 3.0; K[270] = K[40] * 0.01; K[271] = K[41]
    K = _bf16_exact(K)
    K[130] = _bf16_exact(K[40] * 4.0)       # exact in bf16: a power of two
    K[270] = _bf16_exact(K[40] * 0.0078125)
    V = _bf16_exact(rng.standard_normal((n, d)))
    ref = _run_rows(K, V, 0.999)
    for j in (50, 130, 270):
        assert ref["cid"][j] == ref["cid"][40]
    assert ref["cid"][271] == ref["cid"][41] and len({ref["cid"][10], ref["cid"][11], ref["cid"][200]}) == 3


@pytest.mark.parametrize("seed", range(8))
def test_random_structures_as_one_chunk(seed):
    # the key mixtures of test_gpu_random.py (centres drawn per stretch, duplicates, zero rows, rows scaled by 0.01
    # and 30, thresholds inside the similarity bands) clustered as ONE chunk per sequence: ragged batch of three
    import oracle
    from test_gpu_random import _random_mask, _random_keys
    rng = np.random.default_rng(1000 + seed)
    B, H, d = 3, 2, 128
    N = int(rng.integers(100, 1200))
    lens = rng.integers(1, N + 1, size=B).astype(np.int32)
    lens[0] = N
    K = np.zeros((B, H, N, d), np.float32)
    V = np.zeros_like(K)
    for b in range(B):
        n = int(lens[b])
        shape_mask = _random_mask(rng, n)          # shapes the keys only; the clustering sees no boundary
        for h in range(H):
            K[b, h, :n], V[b, h, :n] = _random_keys(rng, shape_mask, n, d, True)
    tau = float(rng.choice([0.3, 0.7, 0.9, 0.97, 0.985, 0.995, 0.9999, -0.5]))
    dK, dV = g.to_device(K, True), g.to_device(V, True)
    sl = torch.from_numpy(lens).to(g.DEV)
    Kc, Vc, counts, clens, cid = sc.sc_gsc_merge_global(dK, dV, tau, seq_lens=sl, out_dtype=torch.float32, want_cluster_id=True)
    torch.cuda.synchronize()
    compared = 0
    for b in range(B):
        n = int(lens[b])
        for h in range(H):
            r = oracle.compress_head(K[b, h, :n], V[b, h, :n], np.array([0, n + 1], np.int32), tau)
            if r["chunk_margin"].min() <= 1e-9:
                continue                                             # a coin toss in fp64 itself: not a parity case
            compared += 1
            rows = r["n_rows"]
            assert int(clens[b, h]) == rows, (seed, b, h, int(clens[b, h]), rows)
            assert np.array_equal(cid[b, h, :n].cpu().numpy(), r["cid"]), (seed, b, h)
            assert np.array_equal(counts[b, h, :rows].cpu().numpy(), r["counts"][:rows]), (seed, b, h)
            assert g.rowwise_err(Kc[b, h, :rows].cpu().numpy(), r["Kc"][:rows]) <= 1e-3
            assert g.rowwise_err(Vc[b, h, :rows].cpu().numpy(), r["Vc"][:rows]) <= 1e-3
    assert compared >= (B * H + 1) // 2, (seed, compared)
    print("seed", seed, "compared", compared, "N", N, "tau", tau, "rows", clens.cpu().numpy().tolist())
