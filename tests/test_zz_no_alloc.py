"""sc_decode_attn_static (the entry point for callers that cannot allocate: its scratch is a file-scope
device array of the library) against sc_decode_attn on a caller-supplied workspace, through the C ABI:
two calls in a row, the second with a smaller input, outputs equal bit for bit (same kernels, same
fixed summation order)."""
import numpy as np
import pytest
import torch

from paper_2603_14303_amd import binding as sc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cache(B, Hkv, G, cap, rows, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    Kc = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16).to(DEV)
    Vc = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16).to(DEV)
    counts = torch.randint(1, 9, (B, Hkv, cap), generator=g, dtype=torch.int32).to(DEV)
    lens = torch.tensor(rows, dtype=torch.int32).reshape(B, Hkv).to(DEV)
    Q = torch.randn((B, Hkv * G, 128), generator=g).to(torch.bfloat16).to(DEV)
    return Q, Kc, Vc, counts, lens


def _both(B, Hkv, G, cap, rows, seed):
    Q, Kc, Vc, counts, lens = _cache(B, Hkv, G, cap, rows, seed)
    O_ref, lse_ref = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True)
    O = torch.full_like(O_ref, float("nan"))
    lse = torch.full_like(lse_ref, float("nan"))
    print("static call: B=%d Hkv=%d G=%d cap=%d rows=%s" % (B, Hkv, G, cap, rows), flush=True)
    sc.sc_decode_attn_static(Q, Kc, Vc, counts, lens, O, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
    assert torch.equal(O, O_ref), float((O.float() - O_ref.float()).abs().max())
    assert torch.equal(lse, lse_ref)


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    # first call: 2 sequences x 4 KV heads, several splits per head, ragged lengths incl. an empty head
    _both(2, 4, 4, 4096, [4096, 3000, 1, 0, 2500, 777, 4095, 1234], seed=11)
    # second call right behind it on the same scratch: smaller batch, fewer rows, other head grouping
    _both(1, 2, 2, 1024, [600, 1024], seed=12)
    # and once more at the first shape, so that state left by a smaller call does not matter either
    _both(2, 4, 4, 4096, [10, 4096, 2048, 300, 0, 4000, 64, 1], seed=13)


def test_static_scratch_refuses_shapes_beyond_its_size():
    lib = sc.load_library()
    B, Hkv, G, cap = 64, 8, 4, 1024
    assert lib.sc_decode_attn_workspace_bytes(B, Hkv * G, Hkv, cap, 128) > (16 << 20)
    Q, Kc, Vc, counts, lens = _cache(1, 1, 1, 8, [8], seed=1)
    O = torch.empty_like(Q)
    # the size check comes before anything else: the (too small) tensors passed here are never touched
    st = lib.sc_decode_attn_static(Q.data_ptr(), 1, Kc.data_ptr(), Vc.data_ptr(), 1, cap, counts.data_ptr(),
                                   lens.data_ptr(), B, Hkv * G, Hkv, 128, 0.0, O.data_ptr(), 1, None, None)
    assert st == 4   # SC_ERR_WORKSPACE
