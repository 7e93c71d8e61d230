"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2603_14303_amd import binding as sc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sc.LIB_PATH):
        from paper_2603_14303_amd import build
        build.build(force=True)
    return sc.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "semanticache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sc_[a-z_0-9]+)\s*\(", text)))


def test_exports_match_header(lib):
    declared = _declared_symbols()
    assert set(declared) == set(sc.EXPORTED)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings_and_version(lib):
    names = [lib.sc_status_string(i).decode() for i in range(6)]
    assert names == ["SC_OK", "SC_ERR_INVALID_ARG", "SC_ERR_UNSUPPORTED", "SC_ERR_CAPACITY", "SC_ERR_WORKSPACE",
                     "SC_ERR_RUNTIME"]
    assert lib.sc_status_string(99).decode() == "SC_ERR_UNKNOWN"
    assert re.fullmatch(r"\d+\.\d+\.\d+", lib.sc_version().decode())


def test_workspace_queries(lib):
    assert lib.sc_segment_workspace_bytes(4, 32768) == 0
    a = lib.sc_gsc_merge_workspace_bytes(1, 8, 32768, 128)
    b = lib.sc_gsc_merge_workspace_bytes(4, 8, 32768, 128)
    assert a > 0 and a % 256 == 0 and b >= 4 * a - 4096
    assert lib.sc_gsc_merge_workspace_bytes(0, 8, 32768, 128) == 0
    # sized for one output type: fp32 is the general size, bf16 halves the provisional rows
    assert lib.sc_gsc_merge_workspace_bytes_for(1, 8, 32768, 128, 0) == a
    half = lib.sc_gsc_merge_workspace_bytes_for(1, 8, 32768, 128, 1)
    assert half % 256 == 0 and a - half == 2 * 8 * 32768 * 128 * 2
    assert lib.sc_gsc_merge_workspace_bytes_for(1, 8, 32768, 128, 5) == 0
    d = lib.sc_decode_attn_workspace_bytes(1, 32, 8, 32768, 128)
    assert d > 0 and d % 256 == 0
    assert lib.sc_decode_attn_workspace_bytes(1, 30, 8, 32768, 128) == 0   # Hq not a multiple of Hkv


def test_tuning_knobs(lib):
    old = sc.tune_get("decode_min_rows")
    sc.tune_set("decode_min_rows", 77)
    assert sc.tune_get("decode_min_rows") == 77
    sc.tune_set("decode_min_rows", old)
    with pytest.raises(sc.SemantiCacheError):
        sc.tune_set("no_such_knob", 1)


FAKE = 0x10000  # a 256-byte aligned non-null address; never dereferenced because validation fails first


def test_segment_rejects_bad_arguments(lib):
    f = lib.sc_segment
    ok = dict(mask=FAKE, stride=64, lens=None, B=1, N=64, off=FAKE, ostride=66, ocap=66, nch=FAKE)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["mask"], a["stride"], a["lens"], a["B"], a["N"], a["off"], a["ostride"], a["ocap"], a["nch"],
                 None, 0, None)
    assert call(mask=None) == 1 and call(off=None) == 1 and call(nch=None) == 1
    assert call(B=0) == 1 and call(N=0) == 1
    assert call(ocap=1) == 3
    assert call(stride=10) == 1 and call(ostride=10) == 1
    assert call(off=FAKE + 2) == 1


def test_gsc_merge_rejects_bad_arguments(lib):
    f = lib.sc_gsc_merge
    need = lib.sc_gsc_merge_workspace_bytes(1, 2, 1024, 64)
    ok = dict(K=FAKE, V=FAKE, idt=0, sb=2 * 1024 * 64, sh=1024 * 64, sn=64, lens=None, off=FAKE, ostride=1026,
              nch=FAKE, B=1, H=2, N=1024, d=64, tau=0.7, Kc=FAKE, Vc=FAKE, odt=0, cap=1024, counts=FAKE,
              clens=FAKE, cid=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["K"], a["V"], a["idt"], a["sb"], a["sh"], a["sn"], a["lens"], a["off"], a["ostride"], a["nch"],
                 a["B"], a["H"], a["N"], a["d"], a["tau"], a["Kc"], a["Vc"], a["odt"], a["cap"], a["counts"],
                 a["clens"], a["cid"], a["ws"], a["wsb"], None)
    for k in ("K", "V", "off", "nch", "Kc", "Vc", "counts", "clens"):
        assert call(**{k: None}) == 1, k
    assert call(B=0) == 1 and call(H=0) == 1 and call(N=0) == 1
    assert call(cap=0) == 3
    assert call(d=96) == 2 and call(idt=7) == 2 and call(odt=-1) == 2
    assert call(sn=32) == 1                 # rows overlap
    assert call(sn=66) == 1                 # fp32 rows not 16-byte aligned
    assert call(K=FAKE + 4) == 1
    assert call(tau=float("nan")) == 1
    assert call(ws=None) == 4 and call(wsb=need - 1) == 4 and call(ws=FAKE + 8) == 4
    # a workspace sized for bf16 output is too small for fp32 output (odt=0 above), and enough for bf16
    small = lib.sc_gsc_merge_workspace_bytes_for(1, 2, 1024, 64, 1)
    assert small < need and call(wsb=small) == 4 and call(wsb=small - 1, odt=1) == 4


def test_decode_rejects_bad_arguments(lib):
    f = lib.sc_decode_attn
    need = lib.sc_decode_attn_workspace_bytes(1, 8, 2, 512, 128)
    ok = dict(Q=FAKE, qdt=1, Kc=FAKE, Vc=FAKE, kdt=1, cap=512, counts=FAKE, clens=FAKE, B=1, Hq=8, Hkv=2, d=128,
              scale=0.0, O=FAKE, odt=1, lse=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["Q"], a["qdt"], a["Kc"], a["Vc"], a["kdt"], a["cap"], a["counts"], a["clens"], a["B"], a["Hq"],
                 a["Hkv"], a["d"], a["scale"], a["O"], a["odt"], a["lse"], a["ws"], a["wsb"], None)
    for k in ("Q", "Kc", "Vc", "counts", "clens", "O"):
        assert call(**{k: None}) == 1, k
    assert call(B=0) == 1 and call(Hq=0) == 1 and call(Hkv=0) == 1
    assert call(cap=0) == 3
    assert call(d=80) == 2 and call(kdt=3) == 2
    assert call(Hq=9) == 2                  # not a multiple of Hkv
    assert call(Hq=18) == 2                 # 9 query heads per KV head: above the supported group size
    assert call(scale=float("nan")) == 1
    assert call(ws=None) == 4 and call(wsb=16) == 4
    assert lib.sc_decode_attn_init_workspace(None, 0, 1, 2, None) == 4
    assert lib.sc_decode_attn_init_workspace(FAKE, 4096, 0, 2, None) == 1


def test_decode_tail_rejects_bad_arguments(lib):
    f = lib.sc_decode_attn_tail
    need = lib.sc_decode_attn_workspace_bytes(1, 8, 2, 512, 128)
    ok = dict(Q=FAKE, qdt=1, Kc=FAKE, Vc=FAKE, kdt=1, cap=512, counts=FAKE, clens=FAKE, Kt=FAKE, Vt=FAKE, tcap=64,
              tlens=FAKE, B=1, Hq=8, Hkv=2, d=128, scale=0.0, O=FAKE, odt=1, lse=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["Q"], a["qdt"], a["Kc"], a["Vc"], a["kdt"], a["cap"], a["counts"], a["clens"], a["Kt"], a["Vt"],
                 a["tcap"], a["tlens"], a["B"], a["Hq"], a["Hkv"], a["d"], a["scale"], a["O"], a["odt"], a["lse"],
                 a["ws"], a["wsb"], None)
    for k in ("Q", "Kc", "Vc", "counts", "clens", "O", "Kt", "Vt", "tlens"):
        assert call(**{k: None}) == 1, k
    assert call(tcap=0) == 3 and call(cap=0) == 3
    assert call(cap=2**31 - 10, tcap=64) == 3        # cap + tail_cap must stay a 32-bit row index
    assert call(Kt=FAKE + 8) == 1
    assert call(d=80) == 2 and call(Hq=9) == 2
    assert call(ws=None) == 4 and call(wsb=16) == 4


def test_gsc_merge_append_rejects_bad_arguments(lib):
    f = lib.sc_gsc_merge_append
    need = lib.sc_gsc_merge_workspace_bytes(1, 2, 1024, 64)
    ok = dict(K=FAKE, V=FAKE, idt=0, sb=2 * 1024 * 64, sh=1024 * 64, sn=64, lens=None, off=FAKE, ostride=1026,
              nch=FAKE, B=1, H=2, N=1024, d=64, tau=0.7, Kc=FAKE, Vc=FAKE, odt=0, cap=4096, counts=FAKE,
              base=FAKE + 256, clens=FAKE, cid=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["K"], a["V"], a["idt"], a["sb"], a["sh"], a["sn"], a["lens"], a["off"], a["ostride"], a["nch"],
                 a["B"], a["H"], a["N"], a["d"], a["tau"], a["Kc"], a["Vc"], a["odt"], a["cap"], a["counts"],
                 a["base"], a["clens"], a["cid"], a["ws"], a["wsb"], None)
    for k in ("K", "V", "off", "nch", "Kc", "Vc", "counts", "clens", "base"):
        assert call(**{k: None}) == 1, k
    assert call(base=FAKE) == 1             # the old and the new lengths must be different arrays
    assert call(base=FAKE + 2) == 1
    assert call(cap=0) == 3 and call(d=96) == 2
    assert call(ws=None) == 4 and call(wsb=need - 1) == 4


def test_multi_attn_rejects_bad_arguments(lib):
    f = lib.sc_multi_attn
    need = lib.sc_multi_attn_workspace_bytes(1, 8, 2, 16, 512, 128)
    assert need > 0 and lib.sc_multi_attn_workspace_bytes(1, 8, 2, 0, 512, 128) == 0
    assert lib.sc_multi_attn_workspace_bytes(1, 8, 2, 16, 512, 64) >= lib.sc_decode_attn_workspace_bytes(1, 8, 2, 512, 64)
    ok = dict(Q=FAKE, qdt=1, nq=16, Kc=FAKE, Vc=FAKE, kdt=1, cap=512, counts=FAKE, clens=FAKE, B=1, Hq=8, Hkv=2,
              d=128, scale=0.0, O=FAKE, odt=1, lse=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["Q"], a["qdt"], a["nq"], a["Kc"], a["Vc"], a["kdt"], a["cap"], a["counts"], a["clens"], a["B"],
                 a["Hq"], a["Hkv"], a["d"], a["scale"], a["O"], a["odt"], a["lse"], a["ws"], a["wsb"], None)
    for k in ("Q", "Kc", "Vc", "counts", "clens", "O"):
        assert call(**{k: None}) == 1, k
    assert call(nq=0) == 1 and call(B=0) == 1
    assert call(nq=5000) == 2 and call(d=80) == 2 and call(Hq=9) == 2
    assert call(cap=0) == 3
    assert call(ws=None) == 4 and call(wsb=need - 1) == 4


def test_gsc_merge_budget_rejects_bad_arguments(lib):
    f = lib.sc_gsc_merge_budget
    need = lib.sc_gsc_merge_budget_workspace_bytes(1, 2, 1024, 64)
    assert need > lib.sc_gsc_merge_workspace_bytes(1, 2, 1024, 64)
    ok = dict(K=FAKE, V=FAKE, idt=0, sb=2 * 1024 * 64, sh=1024 * 64, sn=64, lens=None, off=FAKE, ostride=1026,
              nch=FAKE, B=1, H=2, N=1024, d=64, budget=700, lo=-1.01, hi=1.0, it=12, Kc=FAKE, Vc=FAKE, odt=0, cap=1024,
              counts=FAKE, clens=FAKE, cid=None, tau=FAKE, rows=FAKE + 8, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["K"], a["V"], a["idt"], a["sb"], a["sh"], a["sn"], a["lens"], a["off"], a["ostride"], a["nch"],
                 a["B"], a["H"], a["N"], a["d"], a["budget"], a["lo"], a["hi"], a["it"], a["Kc"], a["Vc"], a["odt"],
                 a["cap"], a["counts"], a["clens"], a["cid"], a["tau"], a["rows"], a["ws"], a["wsb"], None)
    for k in ("K", "V", "off", "nch", "Kc", "Vc", "counts", "clens", "tau"):
        assert call(**{k: None}) == 1, k
    assert call(it=-1) == 1 and call(it=33) == 1 and call(budget=-1) == 1
    assert call(lo=0.5, hi=0.25) == 1 and call(lo=float("nan")) == 1
    assert call(rows=FAKE + 4) == 1 and call(tau=FAKE + 2) == 1
    assert call(cap=0) == 3 and call(d=96) == 2
    assert call(ws=None) == 4 and call(wsb=need - 1) == 4


def test_gsc_merge_global_rejects_bad_arguments(lib):
    f = lib.sc_gsc_merge_global
    need = lib.sc_gsc_merge_global_workspace_bytes(1, 2, 1024, 128)
    # room for the one-chunk offsets, the ordinary kernels' workspace and the bit arrays (n^2 / 8 bytes per array and head)
    assert need > lib.sc_gsc_merge_workspace_bytes(1, 2, 1024, 128) and need > 2 * 2 * 1024 * 1024 // 16
    assert lib.sc_gsc_merge_global_workspace_bytes(0, 2, 1024, 128) == 0
    ok = dict(K=FAKE, V=FAKE, idt=1, sb=2 * 1024 * 128, sh=1024 * 128, sn=128, lens=None, B=1, H=2, N=1024, d=128, tau=0.7,
              Kc=FAKE, Vc=FAKE, odt=1, cap=1024, counts=FAKE, clens=FAKE, cid=None, ws=FAKE, wsb=need)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["K"], a["V"], a["idt"], a["sb"], a["sh"], a["sn"], a["lens"], a["B"], a["H"], a["N"], a["d"], a["tau"],
                 a["Kc"], a["Vc"], a["odt"], a["cap"], a["counts"], a["clens"], a["cid"], a["ws"], a["wsb"], None)
    for k in ("K", "V", "Kc", "Vc", "counts", "clens"):
        assert call(**{k: None}) == 1, k
    assert call(B=0) == 1 and call(N=0) == 1 and call(tau=float("nan")) == 1 and call(sn=64) == 1
    assert call(cap=0) == 3 and call(d=96) == 2 and call(idt=7) == 2
    assert call(ws=None) == 4 and call(wsb=need - 1) == 4 and call(ws=FAKE + 16) == 4


def test_check_lengths_rejects_bad_arguments(lib):
    import ctypes
    bad = ctypes.c_int(7)
    assert lib.sc_check_lengths(None, 4, ctypes.byref(bad), None) == 1
    assert lib.sc_check_lengths(FAKE, 0, ctypes.byref(bad), None) == 1
    assert lib.sc_check_lengths(FAKE + 2, 4, None, None) == 1


def test_binding_refuses_cpu_tensors(lib):
    import torch
    with pytest.raises(sc.SemantiCacheError):
        sc.sc_segment(torch.zeros((1, 16), dtype=torch.uint8))
