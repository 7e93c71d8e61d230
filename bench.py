#!/usr/bin/env python3
"""Benchmark of the SemantiCache compress-then-attend path on one MI355X.

One "step" = one pass of the whole hot path over one Llama-3-8B-shaped layer at 32k context
(workload "layer32k": 8 KV heads x 32768 tokens x d=128, bf16, tau=0.7, 32 query heads):
    sc_segment  ->  sc_gsc_merge  ->  64 x sc_decode_attn
All inputs are resident in HBM before the timed region.  To keep the 256 MB Infinity Cache from
serving re-reads that a real multi-layer model would not get, the K/V inputs rotate over 4 copies
(4 x 134 MB) and the merged caches over 16 buffers (each decode call reads a cache written several
calls earlier); the contents of the copies are identical, only the addresses differ.

Prints ONE JSON line.  `value` is the GSC+merge input throughput (tokens entering sc_segment +
sc_gsc_merge per second); the decode-attention figures and both rooflines ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
N_KV_COPIES = 4
N_CACHE_BUFS = 16


def _build_inputs(w, torch, dev):
    import numpy as np
    from paper_2603_14303_amd import workloads as wl
    mask = np.stack([wl.delimiter_mask(w, b) for b in range(w.batch)])
    lens = wl.seq_lens(w)
    K = np.zeros((w.batch, w.kv_heads, w.n_max, w.head_dim), dtype=np.float32)
    V = np.zeros_like(K)
    for b in range(w.batch):
        for h in range(w.kv_heads):
            K[b, h, : lens[b]], V[b, h, : lens[b]] = wl.keys_values(w, 0, b, h, mask[b], int(lens[b]))
    Q = np.stack([wl.queries(w, 0, s) for s in range(w.decode_steps)])
    host = dict(mask=mask, lens=lens, K=K, V=V, Q=Q)
    Kd = torch.from_numpy(K).to(dev).to(torch.bfloat16)
    Vd = torch.from_numpy(V).to(dev).to(torch.bfloat16)
    devt = dict(mask=torch.from_numpy(mask).to(dev), lens=torch.from_numpy(lens).to(dev),
                K=[Kd] + [Kd.clone() for _ in range(N_KV_COPIES - 1)],
                V=[Vd] + [Vd.clone() for _ in range(N_KV_COPIES - 1)],
                Q=torch.from_numpy(Q).to(dev).to(torch.bfloat16))
    return host, devt


def _cpu_baseline(w, host, tau):
    """The fp64 oracle, as it stands, on one host core: one whole step of the workload
    (segment, GSC + merge of every KV head, then every decode step on the oracle's own merged cache)."""
    import oracle
    t0 = time.perf_counter()
    tokens = 0
    caches = []
    for b in range(w.batch):
        n = int(host["lens"][b])
        off = oracle.segment(host["mask"][b], n)
        for h in range(w.kv_heads):
            caches.append(oracle.compress_head(host["K"][b, h, :n], host["V"][b, h, :n], off, tau))
        tokens += n
    t_comp = time.perf_counter() - t0
    t0 = time.perf_counter()
    steps = w.decode_steps
    G = w.group
    for s in range(steps):
        for b in range(w.batch):
            for h in range(w.kv_heads):
                r = caches[b * w.kv_heads + h]
                for g in range(G):
                    oracle.decode_head(host["Q"][s, b, h * G + g], r["Kc"], r["Vc"], r["counts"], r["n_rows"])
    t_dec = (time.perf_counter() - t0) / steps
    return {
        "value": tokens / t_comp / 1e6, "unit": "Mtok/s", "cores": 1, "kind": "oracle",
        "sample": "one whole step, once: segment + GSC + merge of all %d KV heads (%.2f s), then all %d decode "
                  "steps x %d query heads (%.2f s)" % (w.kv_heads, t_comp, steps, w.q_heads, t_dec * steps),
        "decode_us_per_step": t_dec * 1e6,
    }


def _measured_traffic(workload, tau, rows):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if it covers this workload
    (same compressed row count), else None.  Lines of the file: `<key> <value>`; '#' starts a comment."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    kv = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].split()
            if len(line) == 2:
                kv[line[0]] = float(line[1])
    if kv.get("tau") != float(tau) or int(kv.get("compressed_rows", -1)) != rows:
        return None
    return kv


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="layer32k")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="also time the calls that widen the path (tail attention, append, several query rows); "
                         "off by default so that a profile of the default command holds the main kernels only")
    ap.add_argument("--eager", action="store_true", help="launch every call from Python instead of replaying HIP graphs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; every box of this build has exactly one (got --gpus %d)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_14303_amd import binding as sc
    from paper_2603_14303_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sc.load_library()
    dev = "cuda:0"
    w = wl.get_workload(args.workload)
    tau = args.tau if args.tau is not None else w.taus[0]
    B, H, N, d, Hq = w.batch, w.kv_heads, w.n_max, w.head_dim, w.q_heads
    host, t = _build_inputs(w, torch, dev)
    n_tokens = int(host["lens"].sum())

    # merged-cache capacity: generous but not N_max, so 16 rotating buffers stay small
    cap = max(1024, N // 4)
    offsets = torch.empty((B, N + 2), dtype=torch.int32, device=dev)
    num_chunks = torch.empty((B,), dtype=torch.int32, device=dev)
    bufs = [dict(Kc=torch.empty((B, H, cap, d), dtype=torch.bfloat16, device=dev),
                 Vc=torch.empty((B, H, cap, d), dtype=torch.bfloat16, device=dev),
                 counts=torch.empty((B, H, cap), dtype=torch.int32, device=dev),
                 lens=torch.empty((B, H), dtype=torch.int32, device=dev)) for _ in range(N_CACHE_BUFS)]
    ws_g = sc.gsc_merge_workspace(B, H, N, d, dev)
    ws_d = sc.decode_attn_workspace(B, Hq, H, cap, d, dev)
    O = torch.empty((B, Hq, d), dtype=torch.bfloat16, device=dev)

    def compress(i):
        sc.sc_segment(t["mask"], t["lens"], offsets=offsets, num_chunks=num_chunks)
        c = bufs[i % N_CACHE_BUFS]
        sc.sc_gsc_merge(t["K"][i % N_KV_COPIES], t["V"][i % N_KV_COPIES], offsets, num_chunks, tau,
                        seq_lens=t["lens"], cap=cap, Kc=c["Kc"], Vc=c["Vc"], counts=c["counts"],
                        comp_lens=c["lens"], workspace=ws_g)

    def decode(i, s):
        c = bufs[(i + 1 + s) % N_CACHE_BUFS]
        sc.sc_decode_attn(t["Q"][s], c["Kc"], c["Vc"], c["counts"], c["lens"], O=O, workspace=ws_d)

    # fill every cache buffer once (untimed set-up), then warm up
    for i in range(N_CACHE_BUFS):
        compress(i)
    torch.cuda.synchronize()
    comp_lens = bufs[0]["lens"].cpu().numpy()
    assert (comp_lens > 0).all() and (comp_lens <= cap).all(), comp_lens
    rows = int(comp_lens.sum())
    M = int(num_chunks.sum().item())

    def step(i):
        compress(i)
        for s in range(w.decode_steps):
            decode(i, s)

    # The launch-bound loop (1 + 1 + 64 launches per step) is replayed from HIP graphs, one graph per
    # rotation phase, so the host's launch rate does not sit on the measurement.
    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    if args.eager:
        run_step = lambda i: step(i)
    else:
        step(0)
        torch.cuda.synchronize()
        graphs = [capture(lambda i=i: step(i)) for i in range(N_CACHE_BUFS)]
        run_step = lambda i: graphs[i % N_CACHE_BUFS].replay()

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        run_step(args.warmup + i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_ms = ev0.elapsed_time(ev1) / args.steps

    # device time of the individual calls: graphs holding only that call, replayed between two events
    def timed(graph_list, reps, calls_per_graph):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for g in graph_list:
            g.replay()
        torch.cuda.synchronize()
        a.record()
        for r in range(reps):
            graph_list[r % len(graph_list)].replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (reps * calls_per_graph)

    def gsc_only(i):
        c = bufs[i % N_CACHE_BUFS]
        sc.sc_gsc_merge(t["K"][i % N_KV_COPIES], t["V"][i % N_KV_COPIES], offsets, num_chunks, tau,
                        seq_lens=t["lens"], cap=cap, Kc=c["Kc"], Vc=c["Vc"], counts=c["counts"],
                        comp_lens=c["lens"], workspace=ws_g)

    def seg_only():
        sc.sc_segment(t["mask"], t["lens"], offsets=offsets, num_chunks=num_chunks)

    def dec_only(i):
        for s in range(w.decode_steps):
            decode(i, s)

    def copy_only(i):
        t["K"][(i + 1) % N_KV_COPIES].copy_(t["K"][i % N_KV_COPIES])

    # several calls per graph, so that the fixed cost of starting a graph does not sit on a short kernel
    def gsc_round():
        for i in range(N_KV_COPIES):
            gsc_only(i)

    def seg_round():
        for _ in range(8):
            seg_only()

    gsc_ms = timed([capture(gsc_round)], 10, N_KV_COPIES)
    stage_us = {}
    seg_ms = timed([capture(seg_round)], 10, 8)
    dec_call_ms = timed([capture(lambda i=i: dec_only(i)) for i in range(4)], 16, w.decode_steps)
    # plain device-to-device copy of one K copy (read 67 MB + write 67 MB) as an attainable-bandwidth reference
    copy_ms = timed([capture(lambda i=i: copy_only(i)) for i in range(N_KV_COPIES)], 40, 1)
    copy_gbps = 2 * t["K"][0].numel() * 2 / (copy_ms * 1e-3) / 1e9

    if args.extras:
        # decode-time growth: T new tokens per sequence sit uncompressed behind the merged cache (attended
        # with size 1), then get compressed and appended
        T = 256
        Kt, Vt = t["K"][0][:, :, :T].contiguous(), t["V"][0][:, :, :T].contiguous()
        tail_lens = torch.full((B,), T, dtype=torch.int32, device=dev)
        tmask = t["mask"][:, :T].contiguous()
        toff = torch.empty((B, T + 2), dtype=torch.int32, device=dev)
        tnch = torch.empty((B,), dtype=torch.int32, device=dev)
        ws_t = sc.gsc_merge_workspace(B, H, T, d, dev)
        lens_new = [torch.empty_like(c["lens"]) for c in bufs]

        def dec_tail_only(i):
            for s in range(w.decode_steps):
                c = bufs[(i + 1 + s) % N_CACHE_BUFS]
                sc.sc_decode_attn(t["Q"][s], c["Kc"], c["Vc"], c["counts"], c["lens"], O=O, workspace=ws_d,
                                  Kt=Kt, Vt=Vt, tail_lens=tail_lens)

        def append_round():
            # rows go behind the existing ones; the old lengths stay in place, so every replay does the same work
            for i, c in enumerate(bufs):
                sc.sc_segment(tmask, tail_lens, offsets=toff, num_chunks=tnch)
                sc.sc_gsc_merge(Kt, Vt, toff, tnch, tau, seq_lens=tail_lens, cap=cap, Kc=c["Kc"], Vc=c["Vc"],
                                counts=c["counts"], comp_lens=lens_new[i], base_lens=c["lens"], workspace=ws_t)

        dec_tail_ms = timed([capture(lambda i=i: dec_tail_only(i)) for i in range(4)], 16, w.decode_steps)
        append_ms = timed([capture(append_round)], 10, N_CACHE_BUFS)
        added = (lens_new[0] - bufs[0]["lens"]).cpu().numpy()
        assert (added > 0).all() and (lens_new[0] <= cap).all().item(), added

        # several query rows at once over the merged cache (Eq. 4 with a matrix Q), e.g. speculative tokens
        NQ = 8
        Qm = torch.stack([t["Q"][s] for s in range(NQ)]).contiguous()
        Om = torch.empty_like(Qm)
        ws_m = sc.Workspace(sc.load_library().sc_multi_attn_workspace_bytes(B, Hq, H, NQ, cap, d), dev)

        def multi_only(i):
            for s in range(8):
                c = bufs[(i + 1 + s) % N_CACHE_BUFS]
                sc.sc_multi_attn(Qm, c["Kc"], c["Vc"], c["counts"], c["lens"], O=Om, workspace=ws_m)

        multi_ms = timed([capture(lambda i=i: multi_only(i)) for i in range(2)], 8, 8)

    e = 2
    gsc_bytes = 2 * n_tokens * H * d * e + rows * (2 * d * e + 4) + n_tokens + 4 * (M + B)
    dec_bytes = rows * (2 * d * e + 4) + 2 * B * Hq * d * e
    comp_call_ms = seg_ms + gsc_ms
    value = n_tokens / (comp_call_ms * 1e-3) / 1e6

    tr = _measured_traffic(w.name, tau, rows)
    out = {
        "metric": "GSC+merge input Mtok/s and decode-attn HBM GB/s (frac of peak) at 32k ctx",
        "value": value, "unit": "Mtok/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_ms, "wall_ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: B=%d Hkv=%d Hq=%d d=%d N=%d bf16, tau=%g, %d decode steps per step"
                               % (w.name, B, H, Hq, d, N, tau, w.decode_steps),
                   "compressed_rows_per_head": comp_lens.ravel().tolist(), "chunks": M,
                   "compression_ratio": n_tokens * H / rows},
        "segment_plus_gsc_merge_ms": comp_call_ms, "sc_segment_ms": seg_ms, "sc_gsc_merge_ms": gsc_ms,
        "decode_us_per_step": dec_call_ms * 1e3,
        "decode_GBps": dec_bytes / (dec_call_ms * 1e-3) / 1e9,
        "decode_frac_of_peak": dec_bytes / (dec_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "d2d_copy_GBps": copy_gbps,
        # The call's algorithmic bytes over the duration of ALL kernels of the call (cluster + merge,
        # scan, relocation, back to back on one stream); the first of them dominates.
        "roofline": {"kernel": "sc_gsc_merge = " + " + ".join(stage_us) if stage_us else "sc_gsc_merge",
                     "bound": "hbm",
                     "achieved": gsc_bytes / (gsc_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gsc_bytes / (gsc_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": tr["gsc_merge_bytes"] if tr else None,
                     "algorithmic_bytes": gsc_bytes, "us": gsc_ms * 1e3, "per_kernel_us": stage_us},
        "roofline_decode": {"kernel": "decode_bf16_kernel<128,%d> (sc_decode_attn)" % w.group, "bound": "hbm",
                            "achieved": dec_bytes / (dec_call_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": dec_bytes / (dec_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                            "traffic": tr["decode_bytes"] if tr else None,
                            "algorithmic_bytes": dec_bytes, "us": dec_call_ms * 1e3},
    }
    if args.extras:
        tail_bytes = dec_bytes + B * H * T * 2 * d * e
        out["growth"] = {"tail_tokens": T, "decode_tail_us": dec_tail_ms * 1e3,
                         "decode_tail_GBps": tail_bytes / (dec_tail_ms * 1e-3) / 1e9,
                         "segment_plus_append_us": append_ms * 1e3, "rows_appended_per_head": added.ravel().tolist()}
        multi_bytes = rows * (2 * d * e + 4) + 2 * NQ * B * Hq * d * e
        out["multi_query"] = {"query_rows": NQ, "sc_multi_attn_us": multi_ms * 1e3,
                              "GBps": multi_bytes / (multi_ms * 1e-3) / 1e9,
                              "vs_row_by_row_decode": NQ * dec_call_ms / multi_ms}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(w, host, tau)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
