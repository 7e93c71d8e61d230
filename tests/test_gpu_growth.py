"""GPU parity for decode-time growth: attention over the merged cache plus an uncompressed tail
(sc_decode_attn_tail) and compression of a further stretch of tokens behind the rows already there
(sc_gsc_merge_append), both through the C ABI binding against the CPU oracle.

Tolerances as for the plain calls: sizes and lengths bit-exact, merged rows <= 1e-3 per-row normwise
(fp32 output mode), attention on the same cache <= 4e-3 * max(1, |O|) for bf16 output and 2e-5 for fp32.
"""
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


def _round_like(x, bf16):
    return wl.round_to_bf16(x.astype(np.float32)) if bf16 else x.astype(np.float32)


@pytest.mark.parametrize("bf16,q_bf16,d,Hkv,G,B,cap,tcap", [
    (True, True, 128, 8, 4, 1, 6000, 300),      # fast kernel, several splits, tail spread over the last ones
    (True, True, 128, 4, 7, 3, 1500, 64),       # padded head group, per-sequence tails
    (True, True, 128, 2, 1, 2, 200, 1000),      # tail longer than the merged cache
    (False, False, 64, 2, 1, 1, 300, 40),       # generic kernel, fp32
    (True, False, 128, 2, 2, 2, 700, 33),       # generic kernel: bf16 cache, fp32 queries
])
def test_decode_tail_against_oracle(bf16, q_bf16, d, Hkv, G, B, cap, tcap):
    rng = np.random.default_rng(1000 + cap + tcap)
    Hq = Hkv * G
    Q = _round_like(rng.standard_normal((B, Hq, d)), q_bf16)
    Kc, Vc = _round_like(rng.standard_normal((B, Hkv, cap, d)), bf16), _round_like(rng.standard_normal((B, Hkv, cap, d)), bf16)
    Kt, Vt = _round_like(rng.standard_normal((B, Hkv, tcap, d)), bf16), _round_like(rng.standard_normal((B, Hkv, tcap, d)), bf16)
    counts = rng.integers(1, 40, (B, Hkv, cap)).astype(np.int32)
    lens = rng.integers(cap // 2, cap + 1, (B, Hkv)).astype(np.int32)
    lens[0, 0] = cap
    lens[-1, -1] = 0                                             # one head group with nothing merged yet
    tails = rng.integers(1, tcap + 1, (B,)).astype(np.int32)
    dQ, dKc, dVc = g.to_device(Q, q_bf16), g.to_device(Kc, bf16), g.to_device(Vc, bf16)
    dKt, dVt = g.to_device(Kt, bf16), g.to_device(Vt, bf16)
    dcounts, dlens = torch.from_numpy(counts).to(g.DEV), torch.from_numpy(lens).to(g.DEV)
    ws = sc.decode_attn_workspace(B, Hq, Hkv, cap, d, g.DEV)
    tol = 4e-3 if q_bf16 else 2e-5
    for trial, tl in enumerate([tails, np.zeros(B, np.int32), np.full(B, tcap, np.int32)]):
        dtails = torch.from_numpy(tl.astype(np.int32)).to(g.DEV)
        O, lse = sc.sc_decode_attn(dQ, dKc, dVc, dcounts, dlens, want_lse=True, workspace=ws, Kt=dKt, Vt=dVt,
                                   tail_lens=dtails)
        torch.cuda.synchronize()
        want_O, want_L = oracle.decode_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, tl)
        got = O.float().cpu().numpy().astype(np.float64)
        err = np.abs(got - want_O) / np.maximum(1.0, np.abs(want_O))
        assert err.max() <= tol, (trial, err.max())
        got_l = lse.cpu().numpy().astype(np.float64)
        finite = np.isfinite(want_L)
        assert np.array_equal(np.isneginf(got_l), np.isneginf(want_L))
        assert np.abs(got_l[finite] - want_L[finite]).max() <= 1e-3, trial
        if trial == 1:
            # an empty tail is the plain call: bit for bit where both run the same kernel (wide head
            # groups take the matrix-core kernel for the plain call), within the tolerance otherwise
            O0, lse0 = sc.sc_decode_attn(dQ, dKc, dVc, dcounts, dlens, want_lse=True, workspace=ws)
            torch.cuda.synchronize()
            if not (bf16 and q_bf16 and d == 128 and G >= sc.tune_get("decode_mfma_min_group")):
                assert torch.equal(O0, O) and torch.equal(lse0, lse)
            else:
                got0 = O0.float().cpu().numpy().astype(np.float64)
                assert (np.abs(got0 - want_O) / np.maximum(1.0, np.abs(want_O))).max() <= tol
    # nothing merged anywhere: attention over the new tokens alone
    dzero = torch.zeros_like(dlens)
    O, _ = sc.sc_decode_attn(dQ, dKc, dVc, dcounts, dzero, workspace=ws, Kt=dKt, Vt=dVt,
                             tail_lens=torch.from_numpy(tails).to(g.DEV))
    torch.cuda.synchronize()
    want_O, _ = oracle.decode_attn_tail(Q, Kc, Vc, counts, np.zeros_like(lens), Kt, Vt, tails)
    assert (np.abs(O.float().cpu().numpy() - want_O) / np.maximum(1.0, np.abs(want_O))).max() <= tol


def _cut_after_delimiter(mask_row, n, frac):
    delims = np.nonzero(mask_row[:n])[0]
    return int(delims[int(len(delims) * frac)]) + 1


@pytest.mark.parametrize("name,n,tau,frac", [
    ("tiny", 1024, 0.7, 0.5),              # fp32, d = 64: generic kernels (their scan adds the old length)
    ("layer32k", 4096 + 37, 0.7, 0.4),     # bf16 fast path, relocation adds the old length itself
    ("layer32k", 3000, 0.9745, 0.9),       # short stretch behind a long prefix
    ("long128k", 70000, 0.7, 0.3),         # stretch beyond 32k tokens: fast path with the scan kernel
])
def test_append_gives_the_rows_of_one_call_over_the_whole_sequence(name, n, tau, frac):
    w = wl.get_workload(name)
    heads = 2
    case = build_case(w, tau, n_max=n, heads=heads)
    bf16 = w.dtype == "bf16"
    n = int(case["seq_lens"][0])
    cut = _cut_after_delimiter(case["mask"][0], n, frac)
    assert 0 < cut < n
    K, V = g.to_device(case["K"], bf16), g.to_device(case["V"], bf16)
    cap = n
    # prefix [0, cut): ends with a delimiter
    off0, nch0, _ = g.run_segment(case["mask"][:, :cut].copy(), None)
    Kc, Vc, counts, lens0, _ = sc.sc_gsc_merge(K[:, :, :cut], V[:, :, :cut], off0, nch0, tau, cap=cap,
                                               out_dtype=torch.float32)
    # the rest, positions counted from `cut`
    off1, nch1, _ = g.run_segment(case["mask"][:, cut:n].copy(), None)
    lens1 = torch.full_like(lens0, -5)
    sc.sc_gsc_merge(K[:, :, cut:n], V[:, :, cut:n], off1, nch1, tau, cap=cap, out_dtype=torch.float32,
                    Kc=Kc, Vc=Vc, counts=counts, comp_lens=lens1, base_lens=lens0)
    torch.cuda.synchronize()
    got_lens = lens1.cpu().numpy()
    worst = 0.0
    for h in range(heads):
        r = case["ref"][(0, h)]
        rows = r["n_rows"]
        assert got_lens[0, h] == rows, (h, got_lens[0, h], rows)
        assert np.array_equal(counts[0, h, :rows].cpu().numpy(), r["counts"][:rows]), h
        ek = g.rowwise_err(Kc[0, h, :rows].cpu().numpy(), r["Kc"][:rows])
        ev = g.rowwise_err(Vc[0, h, :rows].cpu().numpy(), r["Vc"][:rows])
        worst = max(worst, ek, ev)
        assert ek <= 1e-3 and ev <= 1e-3, (h, ek, ev)
    print(name, n, tau, "cut", cut, "rows", got_lens.tolist(), "merge_err %.2e" % worst)

    # capacity: one row too few for the total -> -1, and the rows that fit are still the right ones
    rows_min = int(got_lens.min())
    small_cap = rows_min - 1
    Kc2, Vc2, counts2, lens0b, _ = sc.sc_gsc_merge(K[:, :, :cut], V[:, :, :cut], off0, nch0, tau, cap=small_cap,
                                                   out_dtype=torch.float32)
    lens2 = torch.full_like(lens0b, -5)
    sc.sc_gsc_merge(K[:, :, cut:n], V[:, :, cut:n], off1, nch1, tau, cap=small_cap, out_dtype=torch.float32,
                    Kc=Kc2, Vc=Vc2, counts=counts2, comp_lens=lens2, base_lens=lens0b)
    torch.cuda.synchronize()
    assert (lens2 == -1).all()
    ok_prefix = (lens0b >= 0).cpu().numpy()
    for h in range(heads):
        if ok_prefix[0, h]:
            assert torch.equal(counts2[0, h, :small_cap], counts[0, h, :small_cap])
            assert torch.equal(Kc2[0, h, :small_cap], Kc[0, h, :small_cap])
    # a state that has already overflowed stays overflowed and nothing is written
    before = Kc2.clone()
    lens3 = torch.full_like(lens2, -5)
    sc.sc_gsc_merge(K[:, :, cut:n], V[:, :, cut:n], off1, nch1, tau, cap=small_cap, out_dtype=torch.float32,
                    Kc=Kc2, Vc=Vc2, counts=counts2, comp_lens=lens3, base_lens=lens2)
    torch.cuda.synchronize()
    assert (lens3 == -1).all() and torch.equal(before, Kc2)


def test_generation_loop_on_a_ragged_batch():
    """Prefill, then tokens arrive one stretch at a time: attend over cache + tail, and every time the
    stretch ends with a delimiter compress it and append.  Checked against the oracle doing the same."""
    w = wl.get_workload("batch_gqa7")
    B, n_max = 3, 1536
    case = build_case(w, 0.7, n_max=n_max, batch=B)
    lens = case["seq_lens"].astype(np.int64)
    G, Hkv, d = w.group, w.kv_heads, w.head_dim
    # per sequence: prefill up to a delimiter at about 60 %, the rest arrives as the tail in two stretches
    cut0 = np.array([_cut_after_delimiter(case["mask"][b], int(lens[b]), 0.6) for b in range(B)])
    cut1 = np.array([_cut_after_delimiter(case["mask"][b], int(lens[b]), 0.8) for b in range(B)])
    K, V = g.to_device(case["K"], True), g.to_device(case["V"], True)
    cap = n_max
    mask0 = case["mask"].copy()
    for b in range(B):
        mask0[b, cut0[b]:] = 0
    off0, nch0, sl0 = g.run_segment(mask0, cut0.astype(np.int32))
    Kc, Vc, counts, lens_a, _ = sc.sc_gsc_merge(K, V, off0, nch0, 0.7, seq_lens=sl0, cap=cap)
    # tail buffers hold the tokens after the prefill, per sequence from position 0
    tcap = int((lens - cut0).max())
    Kt = torch.zeros((B, Hkv, tcap, d), dtype=torch.bfloat16, device=g.DEV)
    Vt = torch.zeros_like(Kt)
    tmask = np.zeros((B, tcap), np.uint8)
    for b in range(B):
        t = int(lens[b] - cut0[b])
        Kt[b, :, :t] = K[b, :, cut0[b]:lens[b]]
        Vt[b, :, :t] = V[b, :, cut0[b]:lens[b]]
        tmask[b, :t] = case["mask"][b, cut0[b]:lens[b]]
    Q = wl.queries(w, 0, 0)[:B]
    dQ = g.to_device(Q, True)
    ws = sc.decode_attn_workspace(B, Hkv * G, Hkv, cap, d, g.DEV)

    def attend(lens_dev, Kt_view, Vt_view, tails):
        O, _ = sc.sc_decode_attn(dQ, Kc, Vc, counts, lens_dev, workspace=ws, Kt=Kt_view.contiguous(),
                                 Vt=Vt_view.contiguous(), tail_lens=torch.from_numpy(tails.astype(np.int32)).to(g.DEV))
        torch.cuda.synchronize()
        return O.float().cpu().numpy()

    def oracle_attend(rows_fn, tail_from, tails):
        # the oracle attends over ITS merged rows of the compressed part plus the raw tail tokens
        Kh = case["K"]; Vh = case["V"]
        out = np.zeros((B, Hkv * G, d))
        for b in range(B):
            for h in range(Hkv):
                st = rows_fn(b, h)
                t = int(tails[b])
                k_all = np.concatenate([st["Kc"][:st["n_rows"]], Kh[b, h, tail_from[b]:tail_from[b] + t].astype(np.float64)])
                v_all = np.concatenate([st["Vc"][:st["n_rows"]], Vh[b, h, tail_from[b]:tail_from[b] + t].astype(np.float64)])
                s_all = np.concatenate([st["counts"][:st["n_rows"]], np.ones(t, np.int32)])
                for q in range(G):
                    out[b, h * G + q], _ = oracle.decode_head(Q[b, h * G + q], k_all, v_all, s_all, st["n_rows"] + t)
        return out

    def oracle_prefix(upto):
        return lambda b, h: oracle.compress_head(case["K"][b, h, :upto[b]], case["V"][b, h, :upto[b]],
                                                 oracle.segment(case["mask"][b, :upto[b]]), 0.7)

    # step 1: the whole remainder is still uncompressed
    tails1 = (lens - cut0)
    got = attend(lens_a, Kt, Vt, tails1)
    want = oracle_attend(oracle_prefix(cut0), cut0, tails1)
    assert np.abs(got - want).max() <= 2e-2, np.abs(got - want).max()
    # step 2: the first stretch [cut0, cut1) ends with a delimiter: compress it and append
    st_len = (cut1 - cut0).astype(np.int32)
    off1, nch1, sl1 = g.run_segment(tmask, st_len)
    lens_b = torch.full_like(lens_a, -5)
    sc.sc_gsc_merge(Kt, Vt, off1, nch1, 0.7, seq_lens=sl1, cap=cap, Kc=Kc, Vc=Vc, counts=counts, comp_lens=lens_b,
                    base_lens=lens_a)
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(Hkv):
            whole = oracle_prefix(cut1)(b, h)
            assert int(lens_b[b, h]) == whole["n_rows"], (b, h)
            assert np.array_equal(counts[b, h, :whole["n_rows"]].cpu().numpy(), whole["counts"][:whole["n_rows"]])
    # the tail now starts at cut1; the kernel takes a tail buffer per sequence from row 0, so shift it
    tails2 = (lens - cut1)
    Kt2, Vt2 = torch.zeros_like(Kt), torch.zeros_like(Vt)
    for b in range(B):
        Kt2[b, :, :tails2[b]] = K[b, :, cut1[b]:lens[b]]
        Vt2[b, :, :tails2[b]] = V[b, :, cut1[b]:lens[b]]
    got = attend(lens_b, Kt2, Vt2, tails2)
    want = oracle_attend(oracle_prefix(cut1), cut1, tails2)
    assert np.abs(got - want).max() <= 2e-2, np.abs(got - want).max()
