#!/usr/bin/env python3
"""Benchmark of the SemantiCache compress-then-attend path on one MI355X.

One "step" = one pass of the whole hot path over one Llama-3-8B-shaped layer at 32k context
(workload "layer32k": 8 KV heads x 32768 tokens x d=128, bf16, tau=0.7, 32 query heads):
    sc_segment  ->  sc_gsc_merge  ->  64 x sc_decode_attn
All inputs are resident in HBM before the timed region.  To keep the 256 MB Infinity Cache from
serving re-reads that a real multi-layer model would not get, the K/V inputs rotate over 4 copies
(4 x 134 MB) and the merged caches over 16 buffers (each decode call reads a cache written several
calls earlier); the contents of the copies are identical, only the addresses differ.

With --layers L (> 1; meant for the stacked workloads "stack32k" and "batch_gqa7") every layer has its
own seeded K/V and its own merged cache, as in a model: a step is sc_segment once, sc_gsc_merge for
every layer, then `decode steps` x L sc_decode_attn calls walking the layers in order, and the
throughput is the tokens of all sequences over the summed time of the layers.

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


def _layer_kv(w, layer, mask, lens):
    import numpy as np
    from paper_2603_14303_amd import workloads as wl
    K = np.zeros((w.batch, w.kv_heads, w.n_max, w.head_dim), dtype=np.float32)
    V = np.zeros_like(K)
    for b in range(w.batch):
        for h in range(w.kv_heads):
            K[b, h, : lens[b]], V[b, h, : lens[b]] = wl.keys_values(w, layer, b, h, mask[b], int(lens[b]))
    return K, V


def _host_inputs(w, decode_steps=None):
    """Seeded host-side inputs of layer 0 (numpy only: nothing here touches the GPU)."""
    import numpy as np
    from paper_2603_14303_amd import workloads as wl
    mask = np.stack([wl.delimiter_mask(w, b) for b in range(w.batch)])
    lens = wl.seq_lens(w)
    steps = w.decode_steps if decode_steps is None else decode_steps
    Q = np.stack([wl.queries(w, 0, s) for s in range(steps)])
    K, V = _layer_kv(w, 0, mask, lens)
    return dict(mask=mask, lens=lens, Q=Q, K=K, V=V)


def _build_inputs(w, torch, dev, layers=1, decode_steps=None, host=None):
    """Seeded inputs of the workload on the device: with layers == 1 the K/V of layer 0 in N_KV_COPIES
    copies, otherwise one K/V pair per layer."""
    if host is None:
        host = _host_inputs(w, decode_steps)
    mask, lens = host["mask"], host["lens"]
    devt = dict(mask=torch.from_numpy(mask).to(dev), lens=torch.from_numpy(lens).to(dev),
                Q=torch.from_numpy(host["Q"]).to(dev).to(torch.bfloat16), K=[], V=[])
    for layer in range(layers):
        K, V = (host["K"], host["V"]) if layer == 0 else _layer_kv(w, layer, mask, lens)
        devt["K"].append(torch.from_numpy(K).to(dev).to(torch.bfloat16))
        devt["V"].append(torch.from_numpy(V).to(dev).to(torch.bfloat16))
        del K, V
    if layers == 1:
        devt["K"] += [devt["K"][0].clone() for _ in range(N_KV_COPIES - 1)]
        devt["V"] += [devt["V"][0].clone() for _ in range(N_KV_COPIES - 1)]
    return host, devt


_UNITS = []   # (K, V, offsets, tau) per (sequence, head); filled before the workers are forked, so they inherit it


def _oracle_unit(i):
    """One (sequence, head) of the oracle's compression, in a worker process."""
    import oracle
    K, V, off, tau = _UNITS[i]
    r = oracle.compress_head(K, V, off, tau)
    return r["n_rows"]


def _cpu_baseline(w, host, tau):
    """The fp64 oracle, as it stands, on the host: segment + GSC + merge of every (sequence, KV head) of
    layer 0, repeated a few times on one core and then fanned out with one process per core over the
    independent (sequence, head) units; then the decode steps on the oracle's own merged cache, one core."""
    import multiprocessing as mp
    import oracle
    units = []
    t0 = time.perf_counter()
    tokens = 0
    caches = []
    reps, rep = 1, 0
    while rep < reps:
        caches = []
        for b in range(w.batch):
            n = int(host["lens"][b])
            off = oracle.segment(host["mask"][b], n)
            for h in range(w.kv_heads):
                caches.append(oracle.compress_head(host["K"][b, h, :n], host["V"][b, h, :n], off, tau))
                if rep == 0:
                    units.append((host["K"][b, h, :n], host["V"][b, h, :n], off, tau))
            tokens += n
        if rep == 0:      # about eight seconds of one core for the compression sample, whatever the workload
            reps = max(1, min(64, int(round(8.0 / max(time.perf_counter() - t0, 1e-3)))))
        rep += 1
    t_comp = time.perf_counter() - t0
    # all host cores: the same single-thread code, one process per core over the independent units
    cores = len(os.sched_getaffinity(0))
    workers = max(1, min(cores, len(units)))
    try:
        _UNITS[:] = units
        with mp.get_context("fork").Pool(workers) as pool:
            pool.map(_oracle_unit, range(workers))           # start-up and page-in, untimed
            t0 = time.perf_counter()
            for _ in range(reps):
                pool.map(_oracle_unit, range(len(units)), chunksize=1)
            t_all = time.perf_counter() - t0
        all_cores = {"value": tokens / t_all / 1e6, "unit": "Mtok/s", "cores": workers,
                     "sample": "the same %d (sequence, head) units x %d, one process per core" % (len(units), reps)}
    except Exception as e:   # no fork, no /dev/shm: the one-core figure stands alone
        all_cores = {"error": repr(e)}
    t0 = time.perf_counter()
    steps, s, G = min(host["Q"].shape[0], 4), 0, w.group
    while s < steps:
        for b in range(w.batch):
            for h in range(w.kv_heads):
                r = caches[b * w.kv_heads + h]
                for g in range(G):
                    oracle.decode_head(host["Q"][s, b, h * G + g], r["Kc"], r["Vc"], r["counts"], r["n_rows"])
        s += 1
        if s == steps and steps == min(host["Q"].shape[0], 4):      # about three seconds of decode steps
            steps = max(steps, min(host["Q"].shape[0], int(3.0 / max((time.perf_counter() - t0) / s, 1e-4))))
    t_dec = (time.perf_counter() - t0) / steps
    return {
        "value": tokens / t_comp / 1e6, "unit": "Mtok/s", "cores": 1, "kind": "oracle",
        "sample": "layer 0, %d x (segment + GSC + merge of all %d (sequence, KV head) pairs) in %.2f s; then %d decode "
                  "steps x %d query heads in %.2f s" % (reps, len(units), t_comp, steps, w.batch * w.q_heads, t_dec * steps),
        "decode_us_per_step": t_dec * 1e6,
        "all_cores": all_cores,
    }


def _measured_traffic(workload, tau, rows):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if it covers this workload
    (same compressed row count), else None.  Lines of the file: `<key> <value>`; '#' starts a comment."""
    rel = os.path.join("profiles", "hbm_traffic_%s.txt" % workload)
    if not os.path.exists(os.path.join(ROOT, rel)):
        rel = os.path.join("profiles", "hbm_traffic_%s_tau%g.txt" % (workload, tau))
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    kv = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].split()
            if len(line) == 2:
                kv[line[0]] = float(line[1])
    if kv.get("tau") != float(tau) or int(kv.get("compressed_rows", -1)) != rows:
        return None, None
    return kv, rel


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="layer32k")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--layers", type=int, default=1,
                    help="layers with their own K/V and merged cache (stacked workloads); 1 = one layer with rotating copies")
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per step (default: the workload's)")
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
    from paper_2603_14303_amd import workloads as wl

    w = wl.get_workload(args.workload)
    tau = args.tau if args.tau is not None else w.taus[0]
    B, H, N, d, Hq = w.batch, w.kv_heads, w.n_max, w.head_dim, w.q_heads
    L = max(1, args.layers)
    dsteps = w.decode_steps if args.decode_steps is None else max(1, args.decode_steps)
    host = _host_inputs(w, dsteps)
    # the CPU leg runs first, before this process has touched the GPU: it forks one worker per core
    cpu = None if args.no_cpu_baseline else _cpu_baseline(w, host, tau)

    import torch
    from paper_2603_14303_amd import binding as sc
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sc.load_library()
    dev = "cuda:0"
    host, t = _build_inputs(w, torch, dev, layers=L, decode_steps=dsteps, host=host)
    n_tokens = int(host["lens"].sum())
    n_kv = len(t["K"])                      # K/V sets to walk: the layers, or the rotating copies of layer 0
    n_bufs = L if L > 1 else N_CACHE_BUFS   # merged caches: one per layer, or the rotating buffers

    # merged-cache capacity: generous but not N_max, so the cache buffers stay small
    cap = max(1024, N // 4) if tau < 0.9 else (max(1024, 5 * N // 8) if tau < 0.985 else N + 1)
    offsets = torch.empty((B, N + 2), dtype=torch.int32, device=dev)
    num_chunks = torch.empty((B,), dtype=torch.int32, device=dev)
    bufs = [dict(Kc=torch.empty((B, H, cap, d), dtype=torch.bfloat16, device=dev),
                 Vc=torch.empty((B, H, cap, d), dtype=torch.bfloat16, device=dev),
                 counts=torch.empty((B, H, cap), dtype=torch.int32, device=dev),
                 lens=torch.empty((B, H), dtype=torch.int32, device=dev)) for _ in range(n_bufs)]
    ws_g = sc.gsc_merge_workspace(B, H, N, d, dev, torch.bfloat16)
    ws_d = sc.decode_attn_workspace(B, Hq, H, cap, d, dev)
    O = torch.empty((B, Hq, d), dtype=torch.bfloat16, device=dev)

    def segment():
        sc.sc_segment(t["mask"], t["lens"], offsets=offsets, num_chunks=num_chunks)

    def gsc(i):
        c = bufs[i % n_bufs]
        sc.sc_gsc_merge(t["K"][i % n_kv], t["V"][i % n_kv], offsets, num_chunks, tau,
                        seq_lens=t["lens"], cap=cap, Kc=c["Kc"], Vc=c["Vc"], counts=c["counts"],
                        comp_lens=c["lens"], workspace=ws_g)

    def decode(i, s):
        c = bufs[i % n_bufs]
        sc.sc_decode_attn(t["Q"][s], c["Kc"], c["Vc"], c["counts"], c["lens"], O=O, workspace=ws_d)

    # fill every cache buffer once (untimed set-up)
    segment()
    for i in range(n_bufs):
        gsc(i)
    torch.cuda.synchronize()
    all_lens = torch.stack([c["lens"] for c in bufs]).cpu().numpy()          # [n_bufs, B, H]
    assert (all_lens > 0).all() and (all_lens <= cap).all(), all_lens
    comp_lens = all_lens[0]
    rows = int(comp_lens.sum())
    rows_all = all_lens.reshape(n_bufs, -1).sum(axis=1)                      # rows per layer / buffer
    M = int(num_chunks.sum().item())

    if L > 1:
        def step(i):
            # a model: the prompt's layers are compressed, then every decode step walks the layers
            segment()
            for l in range(L):
                gsc(l)
            for s in range(dsteps):
                for l in range(L):
                    decode(l, s)
    else:
        def step(i):
            segment()
            gsc(i)
            for s in range(dsteps):
                decode(i + 1 + s, s)

    # The launch-bound loop is replayed from HIP graphs (one graph per rotation phase), so the host's launch
    # rate does not sit on the measurement.
    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    n_phase = 1 if L > 1 else N_CACHE_BUFS
    if args.eager:
        run_step = lambda i: step(i)
    else:
        step(0)
        torch.cuda.synchronize()
        graphs = [capture(lambda i=i: step(i)) for i in range(n_phase)]
        run_step = lambda i: graphs[i % n_phase].replay()

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
    # recorded on the stream the kernels are launched on
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

    # several calls per graph, so that the fixed cost of starting a graph does not sit on a short kernel
    n_round = L if L > 1 else N_KV_COPIES

    def gsc_round():
        for i in range(n_round):
            gsc(i)

    def seg_round():
        for _ in range(8):
            segment()

    def dec_round(i):
        if L > 1:
            for l in range(L):
                decode(l, i % dsteps)
        else:
            for s in range(dsteps):
                decode(i + 1 + s, s)

    dec_calls = L if L > 1 else dsteps
    gsc_ms = timed([capture(gsc_round)], 10, n_round)
    seg_ms = timed([capture(seg_round)], 10, 8)
    dec_call_ms = timed([capture(lambda i=i: dec_round(i)) for i in range(4)], 16, dec_calls)
    # attainable-bandwidth references on a buffer far larger than the caches: the library's streaming-read
    # probe (16 bytes per lane like the kernels here) and a plain device-to-device copy
    big = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).zero_()
    sink = torch.empty((4096,), dtype=torch.uint8, device=dev)
    halves = [big[: 1 << 29], big[1 << 29:]]
    read_ms = timed([capture(lambda: sc.stream_read_probe(big, sink))], 10, 1)
    read_gbps = big.numel() / (read_ms * 1e-3) / 1e9
    copy_ms = timed([capture(lambda: halves[1].copy_(halves[0]))], 10, 1)
    copy_gbps = 2 * halves[0].numel() / (copy_ms * 1e-3) / 1e9
    del big, halves

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
            for s in range(dsteps):
                c = bufs[(i + 1 + s) % n_bufs]
                sc.sc_decode_attn(t["Q"][s], c["Kc"], c["Vc"], c["counts"], c["lens"], O=O, workspace=ws_d,
                                  Kt=Kt, Vt=Vt, tail_lens=tail_lens)

        def append_round():
            # rows go behind the existing ones; the old lengths stay in place, so every replay does the same work
            for i, c in enumerate(bufs):
                sc.sc_segment(tmask, tail_lens, offsets=toff, num_chunks=tnch)
                sc.sc_gsc_merge(Kt, Vt, toff, tnch, tau, seq_lens=tail_lens, cap=cap, Kc=c["Kc"], Vc=c["Vc"],
                                counts=c["counts"], comp_lens=lens_new[i], base_lens=c["lens"], workspace=ws_t)

        dec_tail_ms = timed([capture(lambda i=i: dec_tail_only(i)) for i in range(4)], 16, dsteps)
        append_ms = timed([capture(append_round)], 10, n_bufs)
        added = (lens_new[0] - bufs[0]["lens"]).cpu().numpy()
        assert (added > 0).all() and (lens_new[0] <= cap).all().item(), added

        # several query rows at once over the merged cache (Eq. 4 with a matrix Q), e.g. speculative tokens
        NQ = min(8, dsteps)
        Qm = torch.stack([t["Q"][s] for s in range(NQ)]).contiguous()
        Om = torch.empty_like(Qm)
        ws_m = sc.Workspace(sc.load_library().sc_multi_attn_workspace_bytes(B, Hq, H, NQ, cap, d), dev)

        def multi_only(i):
            for s in range(8):
                c = bufs[(i + 1 + s) % n_bufs]
                sc.sc_multi_attn(Qm, c["Kc"], c["Vc"], c["counts"], c["lens"], O=Om, workspace=ws_m)

        multi_ms = timed([capture(lambda i=i: multi_only(i)) for i in range(2)], 8, 8)

        # the whole sequence as one chunk (the "no chunking" variant of the ablation): the call of its own
        ws_g = sc.Workspace(sc.load_library().sc_gsc_merge_global_workspace_bytes(B, H, N, d), dev)
        glob_out = [None]

        def global_round():
            for i in range(2):
                glob_out[0] = sc.sc_gsc_merge_global(t["K"][i % len(t["K"])], t["V"][i % len(t["V"])], tau, seq_lens=t["lens"],
                                                     cap=N, workspace=ws_g)
        global_round()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(3):
            global_round()
        ev1.record()
        torch.cuda.synchronize()
        global_ms = ev0.elapsed_time(ev1) / 6
        global_rows = int(glob_out[0][3].sum().item())

    e = 2
    rows_mean = float(rows_all.mean())
    # algorithmic bytes of one call (one layer): inputs read once, merged rows written once / read once
    gsc_bytes = 2 * n_tokens * H * d * e + rows_mean * (2 * d * e + 4) + n_tokens + 4 * (M + B)
    dec_bytes = rows_mean * (2 * d * e + 4) + 2 * B * Hq * d * e
    comp_call_ms = seg_ms / L + gsc_ms                       # per layer; the segmentation is shared by the layers
    value = n_tokens / (comp_call_ms * 1e-3) / 1e6

    tr, tr_src = _measured_traffic(w.name, tau, rows) if L == 1 else (None, None)
    out = {
        "metric": "GSC+merge input Mtok/s and decode-attn HBM GB/s (frac of peak) at 32k ctx",
        "value": value, "unit": "Mtok/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_ms, "wall_ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: B=%d Hkv=%d Hq=%d d=%d N=%d bf16, tau=%g, %d layer(s), %d decode steps per step"
                               % (w.name, B, H, Hq, d, N, tau, L, dsteps),
                   "tokens": n_tokens, "layers": L, "compressed_rows": rows,
                   "compressed_rows_per_head": comp_lens.ravel().tolist() if comp_lens.size <= 64 else None,
                   "compressed_rows_per_layer": rows_all.tolist() if L > 1 else None,
                   "chunks": M, "compression_ratio": n_tokens * H / rows_mean},
        "segment_plus_gsc_merge_ms": comp_call_ms, "sc_segment_ms": seg_ms, "sc_gsc_merge_ms": gsc_ms,
        "stack_Mtok_per_s": n_tokens / ((seg_ms + L * gsc_ms) * 1e-3) / 1e6,   # tokens over the summed time of all layers
        "decode_us_per_step": dec_call_ms * 1e3,
        "decode_GBps": dec_bytes / (dec_call_ms * 1e-3) / 1e9,
        "decode_frac_of_peak": dec_bytes / (dec_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "attainable": {"stream_read_GBps": read_gbps, "d2d_copy_GBps": copy_gbps,
                       "note": "1 GiB streamed by sc_stream_read_probe (16 B per lane); 512 MiB copied device to device "
                               "(read + write counted)"},
        # The call's algorithmic bytes over the duration of ALL kernels of the call (cluster + merge,
        # relocation, back to back on one stream); the first of them dominates.
        "roofline": {"kernel": "sc_gsc_merge = gsc_compress_kernel + gsc_relocate_kernel", "bound": "hbm",
                     "achieved": gsc_bytes / (gsc_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gsc_bytes / (gsc_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": tr["gsc_merge_bytes"] if tr else None, "traffic_source": tr_src,
                     "algorithmic_bytes": gsc_bytes, "us": gsc_ms * 1e3},
        "roofline_decode": {"kernel": "sc_decode_attn", "bound": "hbm",
                            "achieved": dec_bytes / (dec_call_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": dec_bytes / (dec_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                            "traffic": tr["decode_bytes"] if tr else None, "traffic_source": tr_src,
                            "algorithmic_bytes": dec_bytes, "us": dec_call_ms * 1e3},
    }
    if args.extras:
        tail_bytes = dec_bytes + B * H * T * 2 * d * e
        out["growth"] = {"tail_tokens": T, "decode_tail_us": dec_tail_ms * 1e3,
                         "decode_tail_GBps": tail_bytes / (dec_tail_ms * 1e-3) / 1e9,
                         "segment_plus_append_us": append_ms * 1e3, "rows_appended_per_head": added.ravel().tolist()[:64]}
        multi_bytes = rows_mean * (2 * d * e + 4) + 2 * NQ * B * Hq * d * e
        pair_flops = 2.0 * d * sum(int(x) * (int(x) + 1) / 2 for x in host["lens"]) * H      # all pairs i < j of every (sequence, head)
        out["one_chunk"] = {"sc_gsc_merge_global_ms": global_ms, "rows": global_rows, "workspace_GB": ws_g.nbytes / 1e9,
                            "Mtok_per_s": n_tokens / (global_ms * 1e-3) / 1e6,
                            "pair_TFLOPs": pair_flops / (global_ms * 1e-3) / 1e12,
                            "note": "eager launches; pair_TFLOPs counts the n^2/2 * d MACs of all pairwise comparisons over the whole call"}
        out["multi_query"] = {"query_rows": NQ, "sc_multi_attn_us": multi_ms * 1e3,
                              "GBps": multi_bytes / (multi_ms * 1e-3) / 1e9,
                              "vs_row_by_row_decode": NQ * dec_call_ms / multi_ms}
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
