"""Seeded synthetic inputs for the compress-then-attend path.

This module only draws random inputs (delimiter masks, sequence lengths, keys,
values, queries).  It holds none of the method's arithmetic: no similarity, no
clustering, no merging, no attention.  Both the CPU oracle's tests and the HIP
path's tests/bench draw their inputs from here so they see identical bits.

The five workloads mirror the shapes the paper evaluates on (Sec. 3.1:
Llama-3-8B / Mistral-7B style GQA layers, contexts up to 32k and beyond) with
delimiter-bounded chunks (Sec. 2.2, Eq. 1).  The paper's datasets are not
available; delimiter gaps and key/value mixtures are stand-ins:

* delimiter positions: consecutive delimiter-to-delimiter gaps are i.i.d.
  (geometric or truncated power law), capped; a gap of 1 gives two adjacent
  delimiters, i.e. an empty chunk.
* keys/values of a chunk: 1..C Gaussian centres N(0,1)^d (keys and values get
  independent centres), every token picks a centre uniformly and adds
  N(0, sigma^2) noise.  Delimiter tokens get their own N(0,1)^d rows.

All values of a bf16 workload are rounded to bf16 (round-to-nearest-even) on
the host and handed out as float32 arrays holding exactly those bf16 values,
so a float64 widening on the oracle side and a bf16 upload on the GPU side
describe the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "get_workload", "round_to_bf16", "bf16_bits",
    "seq_lens", "delimiter_mask", "variant_mask", "keys_values", "redraw_chunk_keys", "queries",
]


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # 1..5, position in the benchmark's config list
    layers: int
    batch: int
    kv_heads: int
    q_heads: int
    head_dim: int
    n_max: int
    dtype: str                 # "f32" or "bf16"
    gap_kind: str              # "geom" or "zipf"
    gap_param: float           # geometric mean gap, or power-law exponent
    gap_cap: int
    max_centers: int
    noise_std: float
    taus: Tuple[float, ...]
    decode_steps: int
    ragged: Optional[Tuple[int, int]] = None   # inclusive range of sequence lengths
    root_seed: int = field(default=0)

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 1, 2, 2, 64, 1024, "f32", "geom", 16.0, 64, 4, 0.10,
                     (0.7, 1.0, -1.01), 8, None, 0x5C0001),
    "layer32k": Workload("layer32k", 2, 1, 1, 8, 32, 128, 32768, "bf16", "geom", 24.0, 128, 6, 0.15,
                         (0.7,), 64, None, 0x5C0002),
    "stack32k": Workload("stack32k", 3, 32, 4, 8, 32, 128, 32768, "bf16", "geom", 24.0, 128, 6, 0.15,
                         (0.979, 0.9745, 0.03), 128, None, 0x5C0003),
    "long128k": Workload("long128k", 4, 1, 1, 8, 32, 128, 131072, "bf16", "zipf", 1.2, 256, 6, 0.15,
                         (0.7,), 256, None, 0x5C0004),
    "batch_gqa7": Workload("batch_gqa7", 5, 28, 32, 4, 28, 128, 16384, "bf16", "geom", 24.0, 128, 6, 0.15,
                           (0.7, 0.975), 64, (8192, 16384), 0x5C0005),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only)
# ----------------------------------------------------------------------------

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array whose values are exactly bf16 (RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array holding bf16-exact values -> uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _rng(w: Workload, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.root_seed, *[int(k) & 0xFFFFFFFF for k in key]])))


# stream tags
_T_LEN, _T_MASK, _T_K, _T_V, _T_Q, _T_REDRAW = 1, 2, 3, 4, 5, 6


# ----------------------------------------------------------------------------
# sequence lengths and delimiter masks (shared by all layers and heads)
# ----------------------------------------------------------------------------

def seq_lens(w: Workload) -> np.ndarray:
    """int32 [B] sequence lengths."""
    if w.ragged is None:
        return np.full((w.batch,), w.n_max, dtype=np.int32)
    lo, hi = w.ragged
    return _rng(w, _T_LEN).integers(lo, hi + 1, size=w.batch).astype(np.int32)


def _draw_gaps(w: Workload, rng: np.random.Generator, count: int) -> np.ndarray:
    if w.gap_kind == "geom":
        g = rng.geometric(1.0 / w.gap_param, size=count)
        return np.minimum(g, w.gap_cap).astype(np.int64)
    if w.gap_kind == "zipf":
        support = np.arange(1, w.gap_cap + 1, dtype=np.float64)
        p = support ** (-w.gap_param)
        p /= p.sum()
        return rng.choice(np.arange(1, w.gap_cap + 1), size=count, p=p).astype(np.int64)
    raise ValueError(w.gap_kind)


def delimiter_mask(w: Workload, b: int, n: Optional[int] = None) -> np.ndarray:
    """uint8 [N_max] mask for sequence b, nonzero = delimiter; zero beyond the sequence length."""
    if n is None:
        n = int(seq_lens(w)[b])
    rng = _rng(w, _T_MASK, b)
    mask = np.zeros((w.n_max,), dtype=np.uint8)
    pos = -1
    while True:
        gaps = _draw_gaps(w, rng, max(64, n // 8))
        p = pos + np.cumsum(gaps)
        p_in = p[p < n]
        mask[p_in] = 1
        if p_in.size < p.size:
            break
        pos = int(p[-1])
    return mask


def variant_mask(kind: str, delimiters: np.ndarray, n: int, block: int = 64) -> np.ndarray:
    """Chunk boundaries of the paper's chunking ablation (Sec. 3.4, Table 4) for a sequence of n tokens.

    "delimiters": the mask itself.  "fixed": every block-th token closes a chunk, wherever the real
    delimiters are (chunks of block - 1 tokens plus the closing token).  "global": no boundary at
    all, the whole sequence is one chunk.  Keys and values are always drawn from the real
    delimiter structure; only the boundaries handed to the segmentation change.
    """
    if kind == "delimiters":
        return delimiters.copy()
    out = np.zeros_like(delimiters)
    if kind == "fixed":
        out[block - 1:n:block] = 1
    elif kind != "global":
        raise ValueError("unknown chunking %r" % (kind,))
    return out


def _chunk_ids(mask: np.ndarray, n: int) -> Tuple[np.ndarray, int]:
    """chunk index of every token position (delimiters belong to the chunk they close)."""
    m = (mask[:n] != 0)
    cid = np.zeros((n,), dtype=np.int64)
    if n:
        cid[1:] = np.cumsum(m[:-1])
    return cid, (int(cid[-1]) + 1 if n else 1)


# ----------------------------------------------------------------------------
# keys / values
# ----------------------------------------------------------------------------

def _mixture_rows(rng: np.random.Generator, chunk_of_token: np.ndarray, n_chunks: int,
                  is_delim: np.ndarray, d: int, max_centers: int, noise_std: float) -> np.ndarray:
    n = chunk_of_token.shape[0]
    n_centers = rng.integers(1, max_centers + 1, size=n_chunks)
    centers = rng.standard_normal((n_chunks, max_centers, d), dtype=np.float32)
    pick = np.floor(rng.random(n) * n_centers[chunk_of_token]).astype(np.int64)
    rows = centers[chunk_of_token, pick]
    rows = rows + np.float32(noise_std) * rng.standard_normal((n, d), dtype=np.float32)
    # delimiter rows are independent N(0,1)^d
    nd = int(is_delim.sum())
    if nd:
        rows[is_delim] = rng.standard_normal((nd, d), dtype=np.float32)
    return rows.astype(np.float32)


def keys_values(w: Workload, layer: int, b: int, h: int, mask: np.ndarray, n: int):
    """(K, V): float32 [n, d] rows for (layer, sequence, KV head); bf16-exact for bf16 workloads."""
    chunk_of_token, n_chunks = _chunk_ids(mask, n)
    is_delim = mask[:n] != 0
    K = _mixture_rows(_rng(w, _T_K, layer, b, h), chunk_of_token, n_chunks, is_delim,
                      w.head_dim, w.max_centers, w.noise_std)
    V = _mixture_rows(_rng(w, _T_V, layer, b, h), chunk_of_token, n_chunks, is_delim,
                      w.head_dim, w.max_centers, w.noise_std)
    if w.dtype == "bf16":
        K, V = round_to_bf16(K), round_to_bf16(V)
    return K, V


def redraw_chunk_keys(w: Workload, layer: int, b: int, h: int, chunk: int, attempt: int, length: int) -> np.ndarray:
    """Fresh key rows [length, d] for one chunk (same mixture recipe, own sub-seed).

    Used by test harnesses that must keep every evaluated similarity away from
    the threshold: they ask for a new draw of the offending chunk.
    """
    rng = _rng(w, _T_REDRAW, layer, b, h, chunk, attempt)
    rows = _mixture_rows(rng, np.zeros((length,), dtype=np.int64), 1, np.zeros((length,), dtype=bool),
                         w.head_dim, w.max_centers, w.noise_std)
    return round_to_bf16(rows) if w.dtype == "bf16" else rows


def queries(w: Workload, layer: int, step: int) -> np.ndarray:
    """float32 [B, Hq, d] decode queries ~ N(0,1); bf16-exact for bf16 workloads."""
    q = _rng(w, _T_Q, layer, step).standard_normal((w.batch, w.q_heads, w.head_dim), dtype=np.float32)
    return round_to_bf16(q) if w.dtype == "bf16" else q
