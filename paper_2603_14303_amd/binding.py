"""Thin Python binding of libsemanticache (see include/semanticache.h).

Argument marshalling only: torch supplies device memory and the current stream, every step of the
path runs in the library's HIP kernels.  There is no CPU fallback: if the shared library is missing
or a call is refused, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsemanticache.so")

SC_OK = 0
SC_F32, SC_BF16 = 0, 1

_lib = None


class SemantiCacheError(RuntimeError):
    pass


def load_library() -> ctypes.CDLL:
    """Load libsemanticache.so built in-tree (python -m paper_2603_14303_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise SemantiCacheError(
            "libsemanticache.so is not built; run `python -m paper_2603_14303_amd.build` (needs hipcc)")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, sz, f32 = c.c_void_p, c.c_int, c.c_int64, c.c_size_t, c.c_float
    lib.sc_status_string.restype = c.c_char_p
    lib.sc_status_string.argtypes = [i32]
    lib.sc_last_runtime_error.restype = c.c_char_p
    lib.sc_last_runtime_error.argtypes = []
    lib.sc_version.restype = c.c_char_p
    lib.sc_version.argtypes = []
    lib.sc_tune_set.restype = i32
    lib.sc_tune_set.argtypes = [c.c_char_p, i32]
    lib.sc_tune_get.restype = i32
    lib.sc_tune_get.argtypes = [c.c_char_p]
    lib.sc_check_lengths.restype = i32
    lib.sc_check_lengths.argtypes = [vp, i32, c.POINTER(c.c_int), vp]
    lib.sc_stream_read_probe.restype = i32
    lib.sc_stream_read_probe.argtypes = [vp, sz, vp, vp]
    lib.sc_segment_workspace_bytes.restype = sz
    lib.sc_segment_workspace_bytes.argtypes = [i32, i32]
    lib.sc_segment.restype = i32
    lib.sc_segment.argtypes = [vp, i64, vp, i32, i32, vp, i64, i32, vp, vp, sz, vp]
    lib.sc_gsc_merge_workspace_bytes.restype = sz
    lib.sc_gsc_merge_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sc_gsc_merge_workspace_bytes_for.restype = sz
    lib.sc_gsc_merge_workspace_bytes_for.argtypes = [i32, i32, i32, i32, i32]
    lib.sc_gsc_merge.restype = i32
    lib.sc_gsc_merge.argtypes = [vp, vp, i32, i64, i64, i64, vp, vp, i64, vp, i32, i32, i32, i32, f32,
                                 vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.sc_decode_attn_workspace_bytes.restype = sz
    lib.sc_decode_attn_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.sc_decode_attn_init_workspace.restype = i32
    lib.sc_decode_attn_init_workspace.argtypes = [vp, sz, i32, i32, vp]
    lib.sc_decode_attn.restype = i32
    lib.sc_decode_attn.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, f32,
                                   vp, i32, vp, vp, sz, vp]
    lib.sc_decode_attn_static.restype = i32
    lib.sc_decode_attn_static.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, f32,
                                          vp, i32, vp, vp]
    lib.sc_decode_attn_tail.restype = i32
    lib.sc_decode_attn_tail.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, f32,
                                        vp, i32, vp, vp, sz, vp]
    lib.sc_gsc_merge_append.restype = i32
    lib.sc_gsc_merge_append.argtypes = [vp, vp, i32, i64, i64, i64, vp, vp, i64, vp, i32, i32, i32, i32, f32,
                                        vp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.sc_multi_attn_workspace_bytes.restype = sz
    lib.sc_multi_attn_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.sc_multi_attn.restype = i32
    lib.sc_multi_attn.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, f32,
                                  vp, i32, vp, vp, sz, vp]
    lib.sc_multi_attn_tail.restype = i32
    lib.sc_multi_attn_tail.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32,
                                       f32, vp, i32, vp, vp, sz, vp]
    lib.sc_gsc_merge_global_workspace_bytes.restype = sz
    lib.sc_gsc_merge_global_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sc_gsc_merge_global.restype = i32
    lib.sc_gsc_merge_global.argtypes = [vp, vp, i32, i64, i64, i64, vp, i32, i32, i32, i32, ctypes.c_float,
                                        vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.sc_gsc_merge_budget_workspace_bytes.restype = sz
    lib.sc_gsc_merge_budget_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sc_gsc_merge_budget.restype = i32
    lib.sc_gsc_merge_budget.argtypes = [vp, vp, i32, i64, i64, i64, vp, vp, i64, vp, i32, i32, i32, i32,
                                        i64, f32, f32, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    _lib = lib
    return lib


EXPORTED = [
    "sc_status_string", "sc_last_runtime_error", "sc_version", "sc_tune_set", "sc_tune_get",
    "sc_check_lengths", "sc_stream_read_probe", "sc_segment_workspace_bytes", "sc_segment",
    "sc_gsc_merge_workspace_bytes", "sc_gsc_merge_workspace_bytes_for", "sc_gsc_merge",
    "sc_decode_attn_workspace_bytes", "sc_decode_attn_init_workspace", "sc_decode_attn",
    "sc_decode_attn_static", "sc_decode_attn_tail", "sc_gsc_merge_append",
    "sc_multi_attn_workspace_bytes", "sc_multi_attn", "sc_multi_attn_tail",
    "sc_gsc_merge_budget_workspace_bytes", "sc_gsc_merge_budget",
    "sc_gsc_merge_global_workspace_bytes", "sc_gsc_merge_global",
]


def _check(status: int, what: str) -> None:
    if status != SC_OK:
        lib = load_library()
        msg = lib.sc_status_string(status).decode()
        extra = lib.sc_last_runtime_error().decode() if status == 5 else ""
        raise SemantiCacheError("%s failed: %s %s" % (what, msg, extra))


def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return SC_F32
    if t.dtype == torch.bfloat16:
        return SC_BF16
    raise SemantiCacheError("unsupported dtype %s" % t.dtype)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _require_cuda(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise SemantiCacheError("all tensors must live on the GPU")


def tune_set(key: str, value: int) -> None:
    if load_library().sc_tune_set(key.encode(), int(value)) != 0:
        raise SemantiCacheError("unknown tuning key %r" % key)


def tune_get(key: str) -> int:
    return int(load_library().sc_tune_get(key.encode()))


# ------------------------------------------------------------------------------------------------
def sc_segment(mask, seq_lens=None, offsets=None, num_chunks=None):
    """mask u8 [B, N_max] (device) -> (offsets i32 [B, N_max + 2], num_chunks i32 [B])."""
    torch = _torch()
    lib = load_library()
    _require_cuda(mask, seq_lens, offsets, num_chunks)
    if mask.dtype != torch.uint8 or mask.dim() != 2 or mask.stride(1) != 1:
        raise SemantiCacheError("mask must be uint8 [B, N_max] with contiguous rows")
    B, N = mask.shape
    if offsets is None:
        offsets = torch.empty((B, N + 2), dtype=torch.int32, device=mask.device)
    if num_chunks is None:
        num_chunks = torch.empty((B,), dtype=torch.int32, device=mask.device)
    st = lib.sc_segment(_ptr(mask), mask.stride(0), _ptr(seq_lens), B, N, _ptr(offsets), offsets.stride(0),
                        offsets.shape[1], _ptr(num_chunks), None, 0, _stream())
    _check(st, "sc_segment")
    return offsets, num_chunks


class Workspace:
    """Device scratch for one entry point; allocated once through torch, reused across calls."""

    def __init__(self, nbytes: int, device, zero_prefix: int = 0):
        torch = _torch()
        self.nbytes = int(nbytes)
        # torch's caching allocator returns 512-byte aligned blocks
        self.buf = torch.empty((max(self.nbytes, 256),), dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0

    @property
    def ptr(self) -> int:
        return self.buf.data_ptr()


def gsc_merge_workspace(B: int, Hkv: int, N_max: int, d: int, device, out_dtype=None) -> Workspace:
    """Workspace of sc_gsc_merge / sc_gsc_merge_append; with out_dtype (a torch dtype) sized for that output type only."""
    lib = load_library()
    if out_dtype is None:
        return Workspace(lib.sc_gsc_merge_workspace_bytes(B, Hkv, N_max, d), device)
    code = SC_BF16 if out_dtype == _torch().bfloat16 else SC_F32
    return Workspace(lib.sc_gsc_merge_workspace_bytes_for(B, Hkv, N_max, d, code), device)


def sc_gsc_merge(K, V, offsets, num_chunks, tau: float, seq_lens=None, cap: Optional[int] = None,
                 out_dtype=None, Kc=None, Vc=None, counts=None, comp_lens=None, cluster_id=None,
                 want_cluster_id: bool = False, workspace: Optional[Workspace] = None, base_lens=None):
    """K, V [B, Hkv, N_max, d] (device, last dim contiguous) -> (Kc, Vc, counts, comp_lens, cluster_id).

    With base_lens [B, Hkv] (sc_gsc_merge_append) the rows are written behind the base_lens[b, h] rows
    that Kc, Vc, counts already hold, and comp_lens (a different tensor) receives the new totals.
    """
    torch = _torch()
    lib = load_library()
    _require_cuda(K, V, offsets, num_chunks, seq_lens, Kc, Vc, counts, comp_lens, cluster_id)
    if K.dim() != 4 or K.shape != V.shape or K.stride() != V.stride() or K.stride(3) != 1 or K.dtype != V.dtype:
        raise SemantiCacheError("K and V must be [B, Hkv, N_max, d] with identical strides and dtype")
    B, H, N, d = K.shape
    cap = N if cap is None else int(cap)
    out_dtype = K.dtype if out_dtype is None else out_dtype
    dev = K.device
    if Kc is None:
        Kc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    if Vc is None:
        Vc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    if counts is None:
        counts = torch.empty((B, H, cap), dtype=torch.int32, device=dev)
    if comp_lens is None:
        comp_lens = torch.empty((B, H), dtype=torch.int32, device=dev)
    if cluster_id is None and want_cluster_id:
        cluster_id = torch.full((B, H, N), -9, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = gsc_merge_workspace(B, H, N, d, dev, Kc.dtype)
    for t in (Kc, Vc, counts, comp_lens):
        if not t.is_contiguous():
            raise SemantiCacheError("outputs must be contiguous")
    if base_lens is not None:
        _require_cuda(base_lens)
        if Kc.shape[2] != cap or not base_lens.is_contiguous():
            raise SemantiCacheError("append needs the existing Kc/Vc/counts (cap rows) and a contiguous base_lens")
        st = lib.sc_gsc_merge_append(_ptr(K), _ptr(V), _dtype_code(K), K.stride(0), K.stride(1), K.stride(2),
                                     _ptr(seq_lens), _ptr(offsets), offsets.stride(0), _ptr(num_chunks),
                                     B, H, N, d, float(tau), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap,
                                     _ptr(counts), _ptr(base_lens), _ptr(comp_lens), _ptr(cluster_id),
                                     workspace.ptr, workspace.nbytes, _stream())
        _check(st, "sc_gsc_merge_append")
        return Kc, Vc, counts, comp_lens, cluster_id
    st = lib.sc_gsc_merge(_ptr(K), _ptr(V), _dtype_code(K), K.stride(0), K.stride(1), K.stride(2),
                          _ptr(seq_lens), _ptr(offsets), offsets.stride(0), _ptr(num_chunks),
                          B, H, N, d, float(tau), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap,
                          _ptr(counts), _ptr(comp_lens), _ptr(cluster_id), workspace.ptr, workspace.nbytes, _stream())
    _check(st, "sc_gsc_merge")
    return Kc, Vc, counts, comp_lens, cluster_id


def decode_attn_workspace(B: int, Hq: int, Hkv: int, cap: int, d: int, device) -> Workspace:
    lib = load_library()
    ws = Workspace(lib.sc_decode_attn_workspace_bytes(B, Hq, Hkv, cap, d), device)
    _check(lib.sc_decode_attn_init_workspace(ws.ptr, ws.nbytes, B, Hkv, _stream()), "sc_decode_attn_init_workspace")
    return ws


def sc_decode_attn(Q, Kc, Vc, counts, comp_lens, scale: float = 0.0, O=None, lse=None, want_lse: bool = False,
                   workspace: Optional[Workspace] = None, Kt=None, Vt=None, tail_lens=None):
    """Q [B, Hq, d]; Kc, Vc [B, Hkv, cap, d]; counts [B, Hkv, cap]; comp_lens [B, Hkv] -> (O [B, Hq, d], lse).

    With Kt, Vt [B, Hkv, tail_cap, d] and tail_lens [B] (sc_decode_attn_tail) the first tail_lens[b]
    rows of the uncompressed tail attend behind the merged rows, with size 1.
    """
    torch = _torch()
    lib = load_library()
    _require_cuda(Q, Kc, Vc, counts, comp_lens, O, lse)
    B, Hq, d = Q.shape
    _, Hkv, cap, _ = Kc.shape
    for t in (Q, Kc, Vc, counts, comp_lens):
        if not t.is_contiguous():
            raise SemantiCacheError("inputs must be contiguous")
    if O is None:
        O = torch.empty((B, Hq, d), dtype=Q.dtype, device=Q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=Q.device)
    if workspace is None:
        workspace = decode_attn_workspace(B, Hq, Hkv, cap, d, Q.device)
    if Kt is not None:
        _require_cuda(Kt, Vt, tail_lens)
        if Kt.shape != Vt.shape or Kt.dtype != Kc.dtype or Vt.dtype != Kc.dtype or Kt.dim() != 4 or \
                Kt.shape[:2] != Kc.shape[:2] or Kt.shape[3] != d:
            raise SemantiCacheError("Kt, Vt must be [B, Hkv, tail_cap, d] of the cache's dtype")
        for t in (Kt, Vt, tail_lens):
            if not t.is_contiguous():
                raise SemantiCacheError("inputs must be contiguous")
        st = lib.sc_decode_attn_tail(_ptr(Q), _dtype_code(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                                     _ptr(comp_lens), _ptr(Kt), _ptr(Vt), int(Kt.shape[2]), _ptr(tail_lens),
                                     B, Hq, Hkv, d, float(scale), _ptr(O), _dtype_code(O), _ptr(lse),
                                     workspace.ptr, workspace.nbytes, _stream())
        _check(st, "sc_decode_attn_tail")
        return O, lse
    st = lib.sc_decode_attn(_ptr(Q), _dtype_code(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                            _ptr(comp_lens), B, Hq, Hkv, d, float(scale), _ptr(O), _dtype_code(O), _ptr(lse),
                            workspace.ptr, workspace.nbytes, _stream())
    _check(st, "sc_decode_attn")
    return O, lse


def sc_decode_attn_static(Q, Kc, Vc, counts, comp_lens, O, lse=None, scale: float = 0.0):
    """sc_decode_attn on the library's own per-GPU scratch: the caller passes inputs and outputs only, and
    neither this wrapper nor the library allocates anything."""
    lib = load_library()
    _require_cuda(Q, Kc, Vc, counts, comp_lens, O, lse)
    B, Hq, d = Q.shape
    _, Hkv, cap, _ = Kc.shape
    for t in (Q, Kc, Vc, counts, comp_lens, O):
        if not t.is_contiguous():
            raise SemantiCacheError("inputs and outputs must be contiguous")
    st = lib.sc_decode_attn_static(_ptr(Q), _dtype_code(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                                   _ptr(comp_lens), B, Hq, Hkv, d, float(scale), _ptr(O), _dtype_code(O), _ptr(lse),
                                   _stream())
    _check(st, "sc_decode_attn_static")
    return O, lse


def sc_multi_attn(Q, Kc, Vc, counts, comp_lens, scale: float = 0.0, O=None, lse=None, want_lse: bool = False,
                  workspace: Optional[Workspace] = None, Kt=None, Vt=None, tail_lens=None, causal: bool = False):
    """Q [nq, B, Hq, d] -> (O [nq, B, Hq, d], lse [nq, B, Hq]): every query row over the whole merged cache.

    With Kt, Vt [B, Hkv, tail_cap, d] and tail_lens [B] (sc_multi_attn_tail) an uncompressed tail follows the
    merged rows; with causal the last nq tail rows are the query rows' own tokens.
    """
    torch = _torch()
    lib = load_library()
    _require_cuda(Q, Kc, Vc, counts, comp_lens, O, lse)
    nq, B, Hq, d = Q.shape
    _, Hkv, cap, _ = Kc.shape
    for t in (Q, Kc, Vc, counts, comp_lens):
        if not t.is_contiguous():
            raise SemantiCacheError("inputs must be contiguous")
    if O is None:
        O = torch.empty((nq, B, Hq, d), dtype=Q.dtype, device=Q.device)
    if lse is None and want_lse:
        lse = torch.empty((nq, B, Hq), dtype=torch.float32, device=Q.device)
    tcap = int(Kt.shape[2]) if Kt is not None else 0
    if workspace is None:
        workspace = Workspace(lib.sc_multi_attn_workspace_bytes(B, Hq, Hkv, nq, cap + tcap, d), Q.device)
    if Kt is not None:
        _require_cuda(Kt, Vt, tail_lens)
        for t in (Kt, Vt, tail_lens):
            if not t.is_contiguous():
                raise SemantiCacheError("inputs must be contiguous")
        if Kt.shape != Vt.shape or Kt.dtype != Kc.dtype or Kt.shape[:2] != Kc.shape[:2] or Kt.shape[3] != d:
            raise SemantiCacheError("Kt, Vt must be [B, Hkv, tail_cap, d] of the cache's dtype")
        st = lib.sc_multi_attn_tail(_ptr(Q), _dtype_code(Q), nq, _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                                    _ptr(comp_lens), _ptr(Kt), _ptr(Vt), tcap, _ptr(tail_lens), int(bool(causal)),
                                    B, Hq, Hkv, d, float(scale), _ptr(O), _dtype_code(O), _ptr(lse),
                                    workspace.ptr, workspace.nbytes, _stream())
        _check(st, "sc_multi_attn_tail")
        return O, lse
    st = lib.sc_multi_attn(_ptr(Q), _dtype_code(Q), nq, _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                           _ptr(comp_lens), B, Hq, Hkv, d, float(scale), _ptr(O), _dtype_code(O), _ptr(lse),
                           workspace.ptr, workspace.nbytes, _stream())
    _check(st, "sc_multi_attn")
    return O, lse


def sc_gsc_merge_budget(K, V, offsets, num_chunks, budget_rows: int, tau_lo: float = -1.01, tau_hi: float = 1.0,
                        iterations: int = 12, seq_lens=None, cap: Optional[int] = None, out_dtype=None,
                        want_cluster_id: bool = False, workspace: Optional[Workspace] = None):
    """sc_gsc_merge at the largest threshold a bisection finds that keeps the total rows within budget_rows.

    Returns (Kc, Vc, counts, comp_lens, cluster_id, tau [1] f32, rows [1] i64), all on the device.
    """
    torch = _torch()
    lib = load_library()
    _require_cuda(K, V, offsets, num_chunks, seq_lens)
    if K.dim() != 4 or K.shape != V.shape or K.stride() != V.stride() or K.stride(3) != 1 or K.dtype != V.dtype:
        raise SemantiCacheError("K and V must be [B, Hkv, N_max, d] with identical strides and dtype")
    B, H, N, d = K.shape
    cap = N if cap is None else int(cap)
    out_dtype = K.dtype if out_dtype is None else out_dtype
    dev = K.device
    Kc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    Vc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    counts = torch.empty((B, H, cap), dtype=torch.int32, device=dev)
    comp_lens = torch.empty((B, H), dtype=torch.int32, device=dev)
    cluster_id = torch.full((B, H, N), -9, dtype=torch.int32, device=dev) if want_cluster_id else None
    tau = torch.empty((1,), dtype=torch.float32, device=dev)
    rows = torch.empty((1,), dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = Workspace(lib.sc_gsc_merge_budget_workspace_bytes(B, H, N, d), dev)
    st = lib.sc_gsc_merge_budget(_ptr(K), _ptr(V), _dtype_code(K), K.stride(0), K.stride(1), K.stride(2),
                                 _ptr(seq_lens), _ptr(offsets), offsets.stride(0), _ptr(num_chunks), B, H, N, d,
                                 int(budget_rows), float(tau_lo), float(tau_hi), int(iterations),
                                 _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts), _ptr(comp_lens),
                                 _ptr(cluster_id), _ptr(tau), _ptr(rows), workspace.ptr, workspace.nbytes, _stream())
    _check(st, "sc_gsc_merge_budget")
    return Kc, Vc, counts, comp_lens, cluster_id, tau, rows


def sc_gsc_merge_global(K, V, tau: float, seq_lens=None, cap: Optional[int] = None, out_dtype=None,
                        want_cluster_id: bool = False, workspace: Optional[Workspace] = None):
    """sc_gsc_merge with the whole sequence of every (sequence, KV head) as one chunk (no offsets).
    K, V [B, Hkv, N_max, d] -> (Kc, Vc, counts, comp_lens, cluster_id)."""
    torch = _torch()
    lib = load_library()
    _require_cuda(K, V, seq_lens)
    if K.dim() != 4 or K.shape != V.shape or K.stride() != V.stride() or K.stride(3) != 1 or K.dtype != V.dtype:
        raise SemantiCacheError("K and V must be [B, Hkv, N_max, d] with identical strides and dtype")
    B, H, N, d = K.shape
    cap = N if cap is None else int(cap)
    out_dtype = K.dtype if out_dtype is None else out_dtype
    dev = K.device
    Kc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    Vc = torch.empty((B, H, cap, d), dtype=out_dtype, device=dev)
    counts = torch.empty((B, H, cap), dtype=torch.int32, device=dev)
    comp_lens = torch.empty((B, H), dtype=torch.int32, device=dev)
    cluster_id = torch.full((B, H, N), -9, dtype=torch.int32, device=dev) if want_cluster_id else None
    if workspace is None:
        workspace = Workspace(lib.sc_gsc_merge_global_workspace_bytes(B, H, N, d), dev)
    st = lib.sc_gsc_merge_global(_ptr(K), _ptr(V), _dtype_code(K), K.stride(0), K.stride(1), K.stride(2), _ptr(seq_lens),
                                 B, H, N, d, float(tau), _ptr(Kc), _ptr(Vc), _dtype_code(Kc), cap, _ptr(counts),
                                 _ptr(comp_lens), _ptr(cluster_id), workspace.ptr, workspace.nbytes, _stream())
    _check(st, "sc_gsc_merge_global")
    return Kc, Vc, counts, comp_lens, cluster_id


def stream_read_probe(buf, sink) -> None:
    """Reads the device tensor `buf` once (measuring aid: time it to get the attainable HBM read bandwidth)."""
    _require_cuda(buf, sink)
    st = load_library().sc_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream())
    _check(st, "sc_stream_read_probe")


def check_lengths(lengths) -> int:
    """Waits for the current stream; -1 if no entry of the device tensor is negative, else the flat index of
    the first overflowed entry (num_chunks / comp_lens use -1 for "did not fit")."""
    lib = load_library()
    _require_cuda(lengths)
    if not lengths.is_contiguous():
        raise SemantiCacheError("lengths must be contiguous")
    bad = ctypes.c_int(-1)
    st = lib.sc_check_lengths(_ptr(lengths), int(lengths.numel()), ctypes.byref(bad), _stream())
    if st not in (0, 3):
        _check(st, "sc_check_lengths")
    return int(bad.value)

