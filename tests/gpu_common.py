"""Helpers for the GPU parity tests: upload a seeded case, run the HIP path through the C ABI
binding, and compare with the oracle element by element.

Tolerances (from the benchmark definition):
  * chunk offsets, cluster indices, sizes, compressed lengths: bit-exact;
  * merged K/V: per-row normwise error max_e|x_gpu - x_ref| / max_e|x_ref| <= 1e-3 on the
    fp32-output mode (fp32 accumulation of at most a few hundred bf16/fp32 terms is ~1e-6; the bound
    leaves room for nothing else), the bf16-output mode must be the RNE rounding of the fp32 mode
    bit for bit, and rows of size 1 must carry the values of their input rows unchanged;
  * decode output: max abs error <= 2e-2 against the oracle run on its OWN fp64 merged cache
    (covers bf16 storage of the cores), and <= 4e-3 (bf16 out: half an ulp of bf16 is 2^-8 relative) / 2e-5 (fp32 out) against the oracle run
    on the GPU's merged cache (the attention kernel's own error).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2603_14303_amd import binding as sc
from paper_2603_14303_amd import workloads as wl

DEV = "cuda:0"


def to_device(x: np.ndarray, bf16: bool):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


def run_segment(mask: np.ndarray, seq_lens: np.ndarray | None):
    m = torch.from_numpy(mask).to(DEV)
    sl = None if seq_lens is None else torch.from_numpy(seq_lens.astype(np.int32)).to(DEV)
    off, nch = sc.sc_segment(m, sl)
    torch.cuda.synchronize()
    return off, nch, sl


def check_segment(mask: np.ndarray, seq_lens: np.ndarray | None):
    off, nch, sl = run_segment(mask, seq_lens)
    off_h, nch_h = off.cpu().numpy(), nch.cpu().numpy()
    B, N = mask.shape
    for b in range(B):
        n = N if seq_lens is None else int(seq_lens[b])
        want = oracle.segment(mask[b], n)
        assert nch_h[b] == want.shape[0] - 1, (b, nch_h[b], want.shape[0] - 1)
        assert np.array_equal(off_h[b, : want.shape[0]], want), b
    return off, nch, sl


def rowwise_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of max_e|got-ref| / max_e|ref|"""
    if ref.shape[0] == 0:
        return 0.0
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float((np.abs(got.astype(np.float64) - ref).max(axis=1) / den).max())


def run_compress(case, out_dtype, cap=None, want_cid=True, offsets=None, num_chunks=None, seq_lens_dev=None):
    """Upload case (from helpers.build_case) and run sc_segment (unless given) + sc_gsc_merge; a case
    marked "global_call" goes through sc_gsc_merge_global instead (it must have one chunk per sequence)."""
    w = case["workload"]
    bf16 = w.dtype == "bf16"
    K, V = to_device(case["K"], bf16), to_device(case["V"], bf16)
    if case.get("global_call"):
        assert not case["mask"].any()
        sl = torch.from_numpy(case["seq_lens"].astype(np.int32)).to(DEV)
        Kc, Vc, counts, lens, cid = sc.sc_gsc_merge_global(K, V, case["tau"], seq_lens=sl, cap=cap, out_dtype=out_dtype,
                                                           want_cluster_id=want_cid)
        torch.cuda.synchronize()
        return dict(K=K, V=V, offsets=None, num_chunks=None, seq_lens=sl, Kc=Kc, Vc=Vc, counts=counts, comp_lens=lens, cid=cid)
    if offsets is None:
        offsets, num_chunks, seq_lens_dev = run_segment(case["mask"], case["seq_lens"])
    Kc, Vc, counts, lens, cid = sc.sc_gsc_merge(K, V, offsets, num_chunks, case["tau"], seq_lens=seq_lens_dev, cap=cap,
                                                out_dtype=out_dtype, want_cluster_id=want_cid)
    torch.cuda.synchronize()
    return dict(K=K, V=V, offsets=offsets, num_chunks=num_chunks, seq_lens=seq_lens_dev, Kc=Kc, Vc=Vc, counts=counts,
                comp_lens=lens, cid=cid)


def check_compress(case, heads=None, check_bf16_mode=True):
    """Comparison of sc_gsc_merge with the oracle for every (b, h) the case holds an oracle result for
    (all of them unless the case was built with a sample); the kernels always run on the full shape."""
    w = case["workload"]
    B, H = case["K"].shape[:2]
    out = run_compress(case, torch.float32)
    lens = out["comp_lens"].cpu().numpy()
    worst = 0.0
    for (b, h) in sorted(case["ref"]):
        n = int(case["seq_lens"][b])
        r = case["ref"][(b, h)]
        rows = r["n_rows"]
        assert lens[b, h] == rows, (b, h, lens[b, h], rows)
        cid = out["cid"][b, h, :n].cpu().numpy()
        counts = out["counts"][b, h, :rows].cpu().numpy()
        Kc, Vc = out["Kc"][b, h, :rows].cpu().numpy(), out["Vc"][b, h, :rows].cpu().numpy()
        assert np.array_equal(cid, r["cid"]), (b, h, "cluster ids differ")
        assert np.array_equal(counts, r["counts"][:rows]), (b, h, "sizes differ")
        ek = rowwise_err(Kc, r["Kc"][:rows])
        ev = rowwise_err(Vc, r["Vc"][:rows])
        worst = max(worst, ek, ev)
        assert ek <= 1e-3 and ev <= 1e-3, (b, h, ek, ev)
        single = np.nonzero(r["counts"][:rows] == 1)[0]
        # rows of size 1 carry the values of an input row unchanged (the oracle's row IS the input row)
        assert np.array_equal(Kc[single].astype(np.float64), r["Kc"][single]), (b, h, "singleton K")
        assert np.array_equal(Vc[single].astype(np.float64), r["Vc"][single]), (b, h, "singleton V")
    if check_bf16_mode and w.dtype == "bf16":
        out16 = run_compress(case, torch.bfloat16, offsets=out["offsets"], num_chunks=out["num_chunks"],
                             seq_lens_dev=out["seq_lens"])
        assert torch.equal(out16["comp_lens"], out["comp_lens"]) and torch.equal(out16["cid"], out["cid"])
        for b in range(B):
            for h in range(H):
                rows = int(lens[b, h])
                assert torch.equal(out16["counts"][b, h, :rows], out["counts"][b, h, :rows])
                assert torch.equal(out16["Kc"][b, h, :rows], out["Kc"][b, h, :rows].to(torch.bfloat16)), (b, h)
                assert torch.equal(out16["Vc"][b, h, :rows], out["Vc"][b, h, :rows].to(torch.bfloat16)), (b, h)
        out["bf16"] = out16
    out["worst_merge_err"] = worst
    return out


def check_decode_sampled(case, gpu_out, steps, tol_vs_oracle=2e-2):
    """sc_decode_attn at the full shape of the case; the oracle recomputes, one query head at a time,
    the outputs of the (b, h) pairs the case holds an oracle result for."""
    w = case["workload"]
    bf16 = w.dtype == "bf16"
    B, H = case["K"].shape[:2]
    G = w.group
    cache = gpu_out.get("bf16", gpu_out) if bf16 else gpu_out
    Kc, Vc, counts, lens = cache["Kc"], cache["Vc"], cache["counts"], cache["comp_lens"]
    ws = sc.decode_attn_workspace(B, H * G, H, Kc.shape[2], w.head_dim, DEV)
    worst_a = worst_b = worst_l = 0.0
    gpu_cache = {}
    for (b, h), r in case["ref"].items():
        rows = r["n_rows"]
        gpu_cache[(b, h)] = (Kc[b, h, :rows].float().cpu().numpy(), Vc[b, h, :rows].float().cpu().numpy(),
                             counts[b, h, :rows].cpu().numpy())
    for step in steps:
        Q = wl.queries(w, case.get("layer", 0), step)[:B]
        O, lse = sc.sc_decode_attn(to_device(Q, bf16), Kc, Vc, counts, lens, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
        Og, Lg = O.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
        for (b, h), r in case["ref"].items():
            gK, gV, gC = gpu_cache[(b, h)]
            for hq in range(h * G, (h + 1) * G):
                oa, _ = oracle.decode_head(Q[b, hq], r["Kc"], r["Vc"], r["counts"], r["n_rows"])
                ob, lb = oracle.decode_head(Q[b, hq], gK, gV, gC, r["n_rows"])
                ea, eb = float(np.abs(Og[b, hq] - oa).max()), float(np.abs(Og[b, hq] - ob).max())
                el = abs(float(Lg[b, hq]) - lb)
                worst_a, worst_b, worst_l = max(worst_a, ea), max(worst_b, eb), max(worst_l, el)
                assert ea <= tol_vs_oracle, (step, b, hq, ea)
                assert eb <= (4e-3 if bf16 else 2e-5) * max(1.0, float(np.abs(ob).max())), (step, b, hq, eb)
                assert el <= 1e-3, (step, b, hq, el)
    return worst_a, worst_b, worst_l


def oracle_cache_arrays(case, cap):
    """Oracle merged cache of a case as dense [B, H, cap, d] fp64 arrays."""
    B, H, _, d = case["K"].shape
    Kc = np.zeros((B, H, cap, d))
    Vc = np.zeros((B, H, cap, d))
    counts = np.ones((B, H, cap), dtype=np.int32)
    lens = np.zeros((B, H), dtype=np.int32)
    for (b, h), r in case["ref"].items():
        rows = r["n_rows"]
        assert rows <= cap
        Kc[b, h, :rows], Vc[b, h, :rows] = r["Kc"][:rows], r["Vc"][:rows]
        counts[b, h, :rows] = r["counts"][:rows]
        lens[b, h] = rows
    return Kc, Vc, counts, lens


def check_decode(case, gpu_out, steps, layer=0, q_heads=None, tol_vs_oracle=2e-2):
    """Run sc_decode_attn on the GPU's merged cache for the given decode steps and compare."""
    w = case["workload"]
    bf16 = w.dtype == "bf16"
    B, H = case["K"].shape[:2]
    G = w.group
    Hq = H * G if q_heads is None else q_heads
    cache = gpu_out.get("bf16", gpu_out) if bf16 else gpu_out
    Kc, Vc, counts, lens = cache["Kc"], cache["Vc"], cache["counts"], cache["comp_lens"]
    cap = Kc.shape[2]
    ws = sc.decode_attn_workspace(B, Hq, H, cap, w.head_dim, DEV)
    oK, oV, oC, oL = oracle_cache_arrays(case, cap)
    gK, gV = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    gC, gL = counts.cpu().numpy(), lens.cpu().numpy()
    worst_a = worst_b = worst_l = 0.0
    for step in steps:
        Q = wl.queries(w, layer, step)[:B, :Hq]
        Qd = to_device(Q, bf16)
        O, lse = sc.sc_decode_attn(Qd, Kc, Vc, counts, lens, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
        Og, Lg = O.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
        Oa, La = oracle.decode_attn(Q, oK, oV, oC, oL)        # oracle end to end
        Ob, Lb = oracle.decode_attn(Q, gK, gV, gC, gL)        # oracle on the GPU's cache
        ea, eb = float(np.abs(Og - Oa).max()), float(np.abs(Og - Ob).max())
        el = float(np.abs(Lg - Lb).max())
        worst_a, worst_b, worst_l = max(worst_a, ea), max(worst_b, eb), max(worst_l, el)
        assert ea <= tol_vs_oracle, (step, ea)
        assert eb <= (4e-3 if bf16 else 2e-5) * max(1.0, float(np.abs(Ob).max())), (step, eb)
        assert el <= 1e-3, (step, el)
    return worst_a, worst_b, worst_l
