"""Shared test plumbing: builds seeded cases from the workload generator and the oracle.

Near-threshold exclusion: Alg. 1 takes discrete decisions from a floating-point
comparison "Sim > tau".  A pair whose similarity lies within 1e-6 of tau could
legitimately flip between fp64 and fp32 arithmetic, so cases handed to the
parity tests contain no such evaluated pair: a chunk that has one gets its keys
redrawn (new sub-seed) until it has none; the number of redraws is reported.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2603_14303_amd import workloads as wl

NEAR_TAU = 1e-6


def build_case(w: wl.Workload, tau: float, layer: int = 0, n_max: int | None = None,
               batch: int | None = None, exclude_near: bool = True, heads: int | None = None,
               sample=None, workers: int = 8, chunking: str = "delimiters"):
    """Generate one layer of workload w (optionally truncated) and its oracle compression.

    sample: None = the oracle runs on every (sequence, head); else a list of (b, h) pairs: all
    inputs are still generated (the kernels run on the full shape) but the oracle, and the
    re-draw of near-threshold chunks, only cover the listed pairs.

    chunking: "delimiters" (the workload's mask), "fixed" (a boundary every 64 tokens) or "global" (one
    chunk): the keys and values keep the structure of the real delimiters, the boundaries change.

    Returns a dict with numpy arrays:
      mask u8 [B, N], seq_lens i32 [B], K, V f32 [B, Hkv, N, d] (bf16-exact for bf16 workloads),
      offsets (list of int32 arrays), num_chunks i32 [B],
      ref: per sampled (b, h) oracle result dicts (fp64), redraws (int), n_pairs (int)
    """
    from concurrent.futures import ThreadPoolExecutor
    B = batch if batch is not None else w.batch
    N = n_max if n_max is not None else w.n_max
    H = heads if heads is not None else w.kv_heads
    d = w.head_dim
    lens = np.minimum(wl.seq_lens(w)[:B], N).astype(np.int32)
    if w.ragged is not None and n_max is not None:
        # keep raggedness when truncating: scale the drawn lengths into [N/2, N]
        lo, hi = w.ragged
        lens = (N // 2 + (wl.seq_lens(w)[:B].astype(np.int64) - lo) * (N - N // 2) // max(1, hi - lo)).astype(np.int32)
    mask = np.zeros((B, N), dtype=np.uint8)
    K = np.zeros((B, H, N, d), dtype=np.float32)
    V = np.zeros((B, H, N, d), dtype=np.float32)
    key_mask = np.zeros((B, N), dtype=np.uint8)     # the delimiters that shape the keys and values
    offsets = []
    for b in range(B):
        n = int(lens[b])
        full = wl.delimiter_mask(w, b, n=min(n, w.n_max))
        key_mask[b, :n] = full[:n]
        mask[b] = wl.variant_mask(chunking, key_mask[b], n)
        offsets.append(oracle.segment(mask[b], n))
    wanted = None if sample is None else set((int(b), int(h)) for b, h in sample)

    def one(bh):
        b, h = bh
        n = int(lens[b])
        off = offsets[b]
        k, v = wl.keys_values(w, layer, b, h, key_mask[b], n)
        K[b, h, :n], V[b, h, :n] = k, v
        if wanted is not None and bh not in wanted:
            return bh, None, 0
        r = oracle.compress_head(k, v, off, tau)
        redraws = 0
        if exclude_near:
            attempt = 0
            while True:
                bad = np.nonzero(r["chunk_margin"] <= NEAR_TAU)[0]
                if bad.size == 0:
                    break
                attempt += 1
                assert attempt < 50, "could not move similarities away from tau"
                for m in bad:
                    s, e = int(off[m]), int(off[m + 1]) - 1
                    k[s:e] = wl.redraw_chunk_keys(w, layer, b, h, int(m), attempt, e - s)
                    redraws += 1
                r = oracle.compress_head(k, v, off, tau)
            K[b, h, :n] = k
        rows = r["n_rows"]
        for key in ("Kc", "Vc", "counts"):          # keep the produced rows only (memory at full sizes)
            r[key] = r[key][:rows].copy()
        return bh, r, redraws

    ref, redraws, pairs = {}, 0, 0
    todo = [(b, h) for b in range(B) for h in range(H)]
    with ThreadPoolExecutor(max(1, workers)) as pool:
        for bh, r, nr in pool.map(one, todo):
            if r is not None:
                ref[bh] = r
                pairs += r["n_pairs"]
            redraws += nr
    return dict(workload=w, tau=float(tau), mask=mask, seq_lens=lens, K=K, V=V, offsets=offsets,
                num_chunks=np.array([o.shape[0] - 1 for o in offsets], dtype=np.int32),
                ref=ref, redraws=redraws, n_pairs=pairs, layer=layer)


def reference_attention(q, K, V, scale):
    """Textbook softmax attention for one query, written with library routines (pin for Eq. 4)."""
    from scipy.special import softmax
    z = (np.asarray(K, dtype=np.float64) @ np.asarray(q, dtype=np.float64)) * scale
    return softmax(z) @ np.asarray(V, dtype=np.float64)
