"""GPU parity for sc_multi_attn (Eq. 4 with a matrix of query rows, Sec. 2.4) against the CPU oracle.

Same bounds as for single-row decode on the same cache: <= 4e-3 * max(1, |O|) with bf16 output (the
matrix-core path also rounds the probabilities to bf16, relative 2^-9 per term), 2e-5 with fp32 output
through the row-by-row path; lse <= 1e-3."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_14303_amd import binding as sc
from paper_2603_14303_amd import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_common as g


def _round_like(x, bf16):
    return wl.round_to_bf16(x.astype(np.float32)) if bf16 else x.astype(np.float32)


@pytest.mark.parametrize("bf16,d,Hkv,G,B,cap,nq", [
    (True, 128, 8, 4, 1, 6000, 16),      # two row blocks per KV head, many splits
    (True, 128, 4, 7, 3, 1500, 5),       # 35 rows: a full block and a ragged one, G does not divide 32
    (True, 128, 2, 1, 2, 300, 1),        # a single query row (one lane of a tile in use)
    (True, 128, 2, 8, 1, 40, 9),         # cache shorter than one step
    (False, 64, 2, 2, 2, 300, 3),        # row by row through the decode kernels, fp32
])
def test_multi_attn_against_oracle(bf16, d, Hkv, G, B, cap, nq):
    rng = np.random.default_rng(500 + cap + nq)
    Hq = Hkv * G
    Q = _round_like(rng.standard_normal((nq, B, Hq, d)), bf16)
    Kc, Vc = _round_like(rng.standard_normal((B, Hkv, cap, d)), bf16), _round_like(rng.standard_normal((B, Hkv, cap, d)), bf16)
    counts = rng.integers(1, 40, (B, Hkv, cap)).astype(np.int32)
    lens = rng.integers(cap // 2, cap + 1, (B, Hkv)).astype(np.int32)
    lens[0, 0] = cap
    lens[-1, -1] = 0
    dQ, dKc, dVc = g.to_device(Q, bf16), g.to_device(Kc, bf16), g.to_device(Vc, bf16)
    dcounts, dlens = torch.from_numpy(counts).to(g.DEV), torch.from_numpy(lens).to(g.DEV)
    want_O, want_L = oracle.multi_attn(Q, Kc, Vc, counts, lens)
    tol = 4e-3 if bf16 else 2e-5
    for trial in range(2):       # twice on one workspace: it carries no state
        if trial == 0:
            ws = sc.Workspace(sc.load_library().sc_multi_attn_workspace_bytes(B, Hq, Hkv, nq, cap, d), g.DEV)
        O, lse = sc.sc_multi_attn(dQ, dKc, dVc, dcounts, dlens, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
        got = O.float().cpu().numpy().astype(np.float64)
        err = np.abs(got - want_O) / np.maximum(1.0, np.abs(want_O))
        assert err.max() <= tol, (trial, err.max(), np.unravel_index(err.argmax(), err.shape))
        got_l = lse.cpu().numpy().astype(np.float64)
        finite = np.isfinite(want_L)
        assert np.array_equal(np.isneginf(got_l), np.isneginf(want_L))
        assert np.abs(got_l[finite] - want_L[finite]).max() <= 1e-3
    # one query row of the call is what sc_decode_attn gives for that row (same cache, same tolerance)
    Od, _ = sc.sc_decode_attn(dQ[nq - 1].contiguous(), dKc, dVc, dcounts, dlens)
    torch.cuda.synchronize()
    diff = (Od.float() - O[nq - 1].float()).abs().max().item()
    assert diff <= 2 * tol * max(1.0, float(np.abs(want_O).max())), diff


def test_multi_attn_on_a_compressed_layer():
    # the real pipeline: compress a truncated layer, then 8 query rows over it; fp32 output to see the
    # kernel's own error against the oracle on the same cache
    from helpers import build_case
    w = wl.get_workload("layer32k")
    case = build_case(w, 0.7, n_max=4096 + 37, heads=3)
    out = g.run_compress(case, torch.bfloat16)
    nq, Hq = 8, 3 * w.group
    Q = np.stack([wl.queries(w, 0, s)[:1, :Hq] for s in range(nq)])
    dQ = g.to_device(Q, True)
    O32 = torch.empty((nq, 1, Hq, w.head_dim), dtype=torch.float32, device=g.DEV)
    O, lse = sc.sc_multi_attn(dQ, out["Kc"], out["Vc"], out["counts"], out["comp_lens"], O=O32, want_lse=True)
    torch.cuda.synchronize()
    gK, gV = out["Kc"].float().cpu().numpy(), out["Vc"].float().cpu().numpy()
    want_O, want_L = oracle.multi_attn(Q, gK, gV, out["counts"].cpu().numpy(), out["comp_lens"].cpu().numpy())
    err = np.abs(O.cpu().numpy() - want_O).max()
    assert err <= 4e-3 * max(1.0, np.abs(want_O).max()), err
    assert np.abs(lse.cpu().numpy() - want_L).max() <= 1e-3
    print("multi_attn on compressed layer: err %.2e" % err)


@pytest.mark.parametrize("Hkv,G,B,cap,tcap,nq,causal", [
    (8, 4, 1, 6000, 300, 16, True),      # two row blocks, tail spread over the last splits
    (4, 7, 3, 1500, 64, 5, True),        # ragged row blocks, per-sequence tails, one shorter than the query block
    (2, 2, 2, 300, 40, 3, False),        # no mask
    (2, 8, 1, 40, 100, 9, True),         # tail longer than the merged cache
])
def test_multi_attn_tail_against_oracle(Hkv, G, B, cap, tcap, nq, causal):
    rng = np.random.default_rng(900 + cap + nq)
    Hq, d = Hkv * G, 128
    Q = _round_like(rng.standard_normal((nq, B, Hq, d)), True)
    Kc, Vc = _round_like(rng.standard_normal((B, Hkv, cap, d)), True), _round_like(rng.standard_normal((B, Hkv, cap, d)), True)
    Kt, Vt = _round_like(rng.standard_normal((B, Hkv, tcap, d)), True), _round_like(rng.standard_normal((B, Hkv, tcap, d)), True)
    counts = rng.integers(1, 40, (B, Hkv, cap)).astype(np.int32)
    lens = rng.integers(cap // 2, cap + 1, (B, Hkv)).astype(np.int32)
    lens[-1, -1] = 0
    tails = rng.integers(nq, tcap + 1, (B,)).astype(np.int32)
    if B > 1:
        tails[1] = max(1, nq - 2)                                   # fewer tail rows than query rows
    dQ, dKc, dVc = g.to_device(Q, True), g.to_device(Kc, True), g.to_device(Vc, True)
    dKt, dVt = g.to_device(Kt, True), g.to_device(Vt, True)
    dcounts, dlens = torch.from_numpy(counts).to(g.DEV), torch.from_numpy(lens).to(g.DEV)
    dtails = torch.from_numpy(tails).to(g.DEV)
    O, lse = sc.sc_multi_attn(dQ, dKc, dVc, dcounts, dlens, want_lse=True, Kt=dKt, Vt=dVt, tail_lens=dtails, causal=causal)
    torch.cuda.synchronize()
    want_O, want_L = oracle.multi_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, tails, causal)
    got = O.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - want_O) / np.maximum(1.0, np.abs(want_O))
    assert err.max() <= 4e-3, (err.max(), np.unravel_index(err.argmax(), err.shape))
    got_l = lse.cpu().numpy().astype(np.float64)
    finite = np.isfinite(want_L)
    assert np.array_equal(np.isneginf(got_l), np.isneginf(want_L))
    assert np.abs(got_l[finite] - want_L[finite]).max() <= 1e-3
    # one query row, no mask: what sc_decode_attn with the same tail gives (either kernel, same tolerance)
    O1, _ = sc.sc_multi_attn(dQ[:1].contiguous(), dKc, dVc, dcounts, dlens, Kt=dKt, Vt=dVt, tail_lens=dtails)
    Od, _ = sc.sc_decode_attn(dQ[0].contiguous(), dKc, dVc, dcounts, dlens, Kt=dKt, Vt=dVt, tail_lens=dtails)
    torch.cuda.synchronize()
    assert (O1[0].float() - Od.float()).abs().max().item() <= 8e-3 * max(1.0, float(np.abs(want_O).max()))


def test_multi_attn_tail_mask_needs_the_matrix_core_path():
    B, Hkv, G, cap, tcap, nq, d = 1, 2, 1, 64, 16, 2, 64
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device=g.DEV)
    with pytest.raises(sc.SemantiCacheError, match="UNSUPPORTED"):
        sc.sc_multi_attn(z(nq, B, Hkv * G, d), z(B, Hkv, cap, d), z(B, Hkv, cap, d),
                         torch.ones((B, Hkv, cap), dtype=torch.int32, device=g.DEV),
                         torch.full((B, Hkv), cap, dtype=torch.int32, device=g.DEV), Kt=z(B, Hkv, tcap, d),
                         Vt=z(B, Hkv, tcap, d), tail_lens=torch.full((B,), tcap, dtype=torch.int32, device=g.DEV), causal=True)
    # without the mask the same shapes go row by row through the decode kernels
    O, _ = sc.sc_multi_attn(z(nq, B, Hkv * G, d), z(B, Hkv, cap, d), z(B, Hkv, cap, d) + 2.0,
                            torch.ones((B, Hkv, cap), dtype=torch.int32, device=g.DEV),
                            torch.full((B, Hkv), cap, dtype=torch.int32, device=g.DEV), Kt=z(B, Hkv, tcap, d),
                            Vt=z(B, Hkv, tcap, d) + 2.0, tail_lens=torch.full((B,), tcap, dtype=torch.int32, device=g.DEV))
    torch.cuda.synchronize()
    assert torch.allclose(O, torch.full_like(O, 2.0), atol=1e-5)


@pytest.mark.parametrize("knobs", [
    dict(multi_block_rows=16, multi_target_wgs=64), dict(multi_block_rows=32, multi_target_wgs=1024),
    dict(multi_block_rows=16, multi_target_wgs=1024), dict(multi_block_rows=32, multi_target_wgs=8),
])
def test_multi_attn_launch_shapes(knobs):
    # one or two tiles of query rows per workgroup, few and many splits: the workspace query and the launch
    # follow the same knobs, the result stays within the bound of the default shape
    rng = np.random.default_rng(641)
    B, Hkv, G, cap, nq, d = 2, 4, 4, 3000, 7, 128          # 28 query rows per KV head
    Hq = Hkv * G
    Q = _round_like(rng.standard_normal((nq, B, Hq, d)), True)
    Kc, Vc = _round_like(rng.standard_normal((B, Hkv, cap, d)), True), _round_like(rng.standard_normal((B, Hkv, cap, d)), True)
    counts = rng.integers(1, 40, (B, Hkv, cap)).astype(np.int32)
    lens = rng.integers(cap // 2, cap + 1, (B, Hkv)).astype(np.int32)
    lens[0, 0] = cap
    want_O, want_L = oracle.multi_attn(Q, Kc, Vc, counts, lens)
    dQ, dKc, dVc = g.to_device(Q, True), g.to_device(Kc, True), g.to_device(Vc, True)
    dcounts, dlens = torch.from_numpy(counts).to(g.DEV), torch.from_numpy(lens).to(g.DEV)
    old = {k: sc.tune_get(k) for k in knobs}
    try:
        for k, v in knobs.items():
            sc.tune_set(k, v)
        O, lse = sc.sc_multi_attn(dQ, dKc, dVc, dcounts, dlens, want_lse=True)
        torch.cuda.synchronize()
    finally:
        for k, v in old.items():
            sc.tune_set(k, v)
    err = np.abs(O.float().cpu().numpy().astype(np.float64) - want_O) / np.maximum(1.0, np.abs(want_O))
    assert err.max() <= 4e-3, (knobs, err.max())
    assert np.abs(lse.cpu().numpy().astype(np.float64) - want_L).max() <= 1e-3
