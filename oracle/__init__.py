"""CPU oracle (fp64, single thread) for the SemantiCache compress-then-attend path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product path never imports this package and
this package never imports the product path.

The arithmetic lives in ``sc_oracle.c`` (one function per equation/algorithm
of the paper, Sec. 2.2-2.4); this file compiles it with gcc and wraps it with
numpy marshalling only.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sc_oracle.c")
_LIB = os.path.join(_HERE, "libsc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sc_oracle.c -> libsc_oracle.so (gcc -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        dp, ip, bp = c.POINTER(c.c_double), c.POINTER(c.c_int32), c.POINTER(c.c_uint8)
        lp = c.POINTER(c.c_int64)
        lib.sc_oracle_segment.restype = c.c_int32
        lib.sc_oracle_segment.argtypes = [bp, c.c_int32, ip]
        lib.sc_oracle_cosine.restype = c.c_double
        lib.sc_oracle_cosine.argtypes = [dp, dp, c.c_int32]
        lib.sc_oracle_gsc_chunk.restype = c.c_int32
        lib.sc_oracle_gsc_chunk.argtypes = [dp, c.c_int64, c.c_int32, c.c_int32, c.c_double, ip, dp, lp]
        lib.sc_oracle_compress_head.restype = c.c_int64
        lib.sc_oracle_compress_head.argtypes = [dp, dp, c.c_int32, c.c_int32, ip, c.c_int32, c.c_double,
                                                dp, dp, ip, c.c_int64, ip, dp, lp]
        lib.sc_oracle_decode_head.restype = None
        lib.sc_oracle_decode_head.argtypes = [dp, dp, dp, ip, c.c_int64, c.c_int32, c.c_double, dp, dp]
        _lib = lib
    return _lib


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- Eq. 1
def segment(mask: np.ndarray, n: Optional[int] = None) -> np.ndarray:
    """One sequence: uint8 mask[>=n] -> int32 offsets[M+1] (Eq. 1; see sc_oracle_segment)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if n is None:
        n = mask.shape[0]
    off = np.empty((n + 2,), dtype=np.int32)
    M = _load().sc_oracle_segment(mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), int(n), _ip(off))
    return off[: M + 1].copy()


def segment_batch(mask: np.ndarray, seq_lens: Sequence[int]) -> Tuple[List[np.ndarray], np.ndarray]:
    """mask [B, N_max] -> (list of per-sequence offsets, num_chunks int32 [B])."""
    offs = [segment(mask[b], int(seq_lens[b])) for b in range(mask.shape[0])]
    return offs, np.array([o.shape[0] - 1 for o in offs], dtype=np.int32)


# --------------------------------------------------------------------------- Eq. 2
def cosine(a, b) -> float:
    a, b = _f64(a), _f64(b)
    return float(_load().sc_oracle_cosine(_dp(a), _dp(b), a.shape[0]))


# --------------------------------------------------------------------------- Alg. 1
def gsc_chunk(K, tau: float):
    """One chunk of key rows [l, d] -> (cid int32 [l], p, min_margin, n_pairs)."""
    K = _f64(K)
    l, d = K.shape
    cid = np.full((l,), -7, dtype=np.int32)
    margin = ctypes.c_double(np.inf)
    pairs = ctypes.c_int64(0)
    p = _load().sc_oracle_gsc_chunk(_dp(K), d, l, d, float(tau), _ip(cid), ctypes.byref(margin), ctypes.byref(pairs))
    return cid, int(p), float(margin.value), int(pairs.value)


# --------------------------------------------------------------------------- Eq. 3
def compress_head(K, V, offsets: np.ndarray, tau: float, cap: Optional[int] = None):
    """One (sequence, head): K, V [n, d] -> dict(Kc, Vc, counts, n_rows, cid, chunk_margin, n_pairs)."""
    K, V = _f64(K), _f64(V)
    n, d = K.shape
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    M = offsets.shape[0] - 1
    if cap is None:
        cap = n
    Kc = np.zeros((cap, d), dtype=np.float64)
    Vc = np.zeros((cap, d), dtype=np.float64)
    counts = np.zeros((cap,), dtype=np.int32)
    cid = np.full((n,), -7, dtype=np.int32)
    margin = np.full((M,), np.inf, dtype=np.float64)
    pairs = ctypes.c_int64(0)
    rows = _load().sc_oracle_compress_head(_dp(K), _dp(V), n, d, _ip(offsets), M, float(tau),
                                           _dp(Kc), _dp(Vc), _ip(counts), cap, _ip(cid), _dp(margin),
                                           ctypes.byref(pairs))
    return dict(Kc=Kc, Vc=Vc, counts=counts, n_rows=int(rows), cid=cid, chunk_margin=margin, n_pairs=int(pairs.value))


# --------------------------------------------------------------------------- Eq. 4
def decode_head(q, Kc, Vc, counts, n_rows: int, scale: Optional[float] = None):
    """One query row q[d] vs merged cache rows [0, n_rows) -> (out[d], lse)."""
    q, Kc, Vc = _f64(q), _f64(Kc), _f64(Vc)
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    d = q.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.zeros((d,), dtype=np.float64)
    lse = ctypes.c_double(0.0)
    _load().sc_oracle_decode_head(_dp(q), _dp(Kc), _dp(Vc), _ip(counts), int(n_rows), d, float(scale),
                                  _dp(out), ctypes.byref(lse))
    return out, float(lse.value)


def decode_attn(Q, Kc, Vc, counts, comp_lens, scale: Optional[float] = None):
    """Q [B, Hq, d]; Kc, Vc [B, Hkv, cap, d]; counts [B, Hkv, cap]; comp_lens [B, Hkv].

    Query head hq reads KV head hq // (Hq // Hkv) (consecutive grouping).
    Returns (O [B, Hq, d] fp64, lse [B, Hq]).
    """
    Q = np.asarray(Q)
    B, Hq, d = Q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    O = np.zeros((B, Hq, d), dtype=np.float64)
    L = np.zeros((B, Hq), dtype=np.float64)
    for b in range(B):
        for h in range(Hkv):
            kc, vc = _f64(Kc[b, h]), _f64(Vc[b, h])
            cn = np.ascontiguousarray(counts[b, h], dtype=np.int32)
            for g in range(G):
                hq = h * G + g
                O[b, hq], L[b, hq] = decode_head(Q[b, hq], kc, vc, cn, int(comp_lens[b, h]), scale)
    return O, L


# ------------------------------------------------- decode-time growth (the paper leaves it open, Sec. 2.1)
def decode_attn_tail(Q, Kc, Vc, counts, comp_lens, Kt, Vt, tail_lens, scale: Optional[float] = None):
    """Eq. 4 over the merged cache followed by an uncompressed tail of new tokens.

    Kt, Vt [B, Hkv, tail_cap, d]; tail_lens [B].  A token that has not been merged is a cluster of
    one (s = 1, ln s = 0), exactly like a delimiter row of the merged cache, so the definition is
    Eq. 4 over the rows [merged rows of (b, h)] ++ [first tail_lens[b] tail rows of (b, h)].
    """
    Q = np.asarray(Q)
    B, Hq, d = Q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    O = np.zeros((B, Hq, d), dtype=np.float64)
    L = np.zeros((B, Hq), dtype=np.float64)
    for b in range(B):
        t = int(tail_lens[b])
        for h in range(Hkv):
            nc = int(comp_lens[b, h])
            k_all = np.concatenate([_f64(Kc[b, h, :nc]), _f64(Kt[b, h, :t])], axis=0)
            v_all = np.concatenate([_f64(Vc[b, h, :nc]), _f64(Vt[b, h, :t])], axis=0)
            s_all = np.concatenate([np.asarray(counts[b, h, :nc], dtype=np.int32), np.ones((t,), dtype=np.int32)])
            for g in range(G):
                hq = h * G + g
                O[b, hq], L[b, hq] = decode_head(Q[b, hq], k_all, v_all, s_all, nc + t, scale)
    return O, L


def append_head(state, K_new, V_new, offsets_new: np.ndarray, tau: float, cap: int):
    """Compress a further stretch of tokens of one (sequence, head) and append its rows.

    `state` is a dict(Kc, Vc, counts, n_rows) as returned by compress_head (arrays of at least `cap`
    rows are not required: they are copied).  Chunks never interact (Alg. 1 runs per chunk), so the
    rows of the new stretch are those of compress_head on the stretch alone, placed after the
    existing n_rows rows.  Returns a new dict(Kc, Vc, counts, n_rows) with `cap` rows of storage;
    n_rows is the true total even if it exceeds cap (rows beyond cap are dropped).
    """
    new = compress_head(K_new, V_new, offsets_new, tau, cap=max(1, np.asarray(K_new).shape[0]))
    d = np.asarray(K_new).shape[1]
    Kc = np.zeros((cap, d), dtype=np.float64)
    Vc = np.zeros((cap, d), dtype=np.float64)
    counts = np.zeros((cap,), dtype=np.int32)
    n0 = int(state["n_rows"])
    keep0 = min(n0, cap)
    Kc[:keep0], Vc[:keep0], counts[:keep0] = state["Kc"][:keep0], state["Vc"][:keep0], state["counts"][:keep0]
    keep1 = max(0, min(new["n_rows"], cap - n0))
    Kc[n0:n0 + keep1], Vc[n0:n0 + keep1] = new["Kc"][:keep1], new["Vc"][:keep1]
    counts[n0:n0 + keep1] = new["counts"][:keep1]
    return dict(Kc=Kc, Vc=Vc, counts=counts, n_rows=n0 + int(new["n_rows"]))


# ------------------------------------------------- Eq. 4 with several query rows (Q in R^{n x d}, Sec. 2.4)
def multi_attn(Q, Kc, Vc, counts, comp_lens, scale: Optional[float] = None):
    """Q [nq, B, Hq, d]: every query row attends to the whole merged cache of its KV head (no mask).

    Eq. 4 is row-wise in Q, so this is decode_attn once per query row.  Returns (O [nq, B, Hq, d], lse [nq, B, Hq]).
    """
    Q = np.asarray(Q)
    outs = [decode_attn(Q[j], Kc, Vc, counts, comp_lens, scale) for j in range(Q.shape[0])]
    return np.stack([o for o, _ in outs]), np.stack([l for _, l in outs])


# ------------------------------------------------- threshold for a cache budget (Sec. 3.1 reports at budgets)
def tau_for_budget(rows_at, budget_rows: int, tau_lo: float, tau_hi: float, iterations: int):
    """Largest threshold a bisection finds whose total number of merged rows stays within budget_rows.

    rows_at(tau) -> total rows of all (sequence, head) problems at that threshold, or None if some
    head does not fit its capacity.  The paper gives no rule from budget to threshold; this one is
    the plain bisection on fp32 midpoints: lo is assumed to fit, `iterations` midpoints are probed,
    a midpoint that fits becomes lo, one that does not becomes hi; the answer is lo.
    Returns (tau float32, list of probed thresholds).
    """
    lo, hi = np.float32(tau_lo), np.float32(tau_hi)
    probed = []
    for _ in range(iterations):
        mid = np.float32(0.5) * (lo + hi)
        probed.append(float(mid))
        r = rows_at(float(mid))
        if r is not None and r <= budget_rows:
            lo = mid
        else:
            hi = mid
    return lo, probed


def multi_attn_tail(Q, Kc, Vc, counts, comp_lens, Kt, Vt, tail_lens, causal: bool, scale: Optional[float] = None):
    """multi_attn over the merged cache followed by an uncompressed tail (rows of size 1).

    Q [nq, B, Hq, d]; Kt, Vt [B, Hkv, tail_cap, d]; tail_lens [B].  With causal, the last nq tail rows
    of a sequence are the query rows' own tokens: query j sees the merged rows and the tail rows
    0 .. tail_lens[b] - nq + j (itself included, none if that is negative); without it every query
    row sees the whole tail.
    """
    Q = np.asarray(Q)
    nq, B, Hq, d = Q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    O = np.zeros((nq, B, Hq, d), dtype=np.float64)
    L = np.zeros((nq, B, Hq), dtype=np.float64)
    for b in range(B):
        t = int(tail_lens[b])
        for h in range(Hkv):
            nc = int(comp_lens[b, h])
            k_all = np.concatenate([_f64(Kc[b, h, :nc]), _f64(Kt[b, h, :t])], axis=0)
            v_all = np.concatenate([_f64(Vc[b, h, :nc]), _f64(Vt[b, h, :t])], axis=0)
            s_all = np.concatenate([np.asarray(counts[b, h, :nc], dtype=np.int32), np.ones((t,), dtype=np.int32)])
            for j in range(nq):
                seen = max(0, t - nq + 1 + j) if causal else t
                for g in range(G):
                    hq = h * G + g
                    O[j, b, hq], L[j, b, hq] = decode_head(Q[j, b, hq], k_all, v_all, s_all, nc + seen, scale)
    return O, L

