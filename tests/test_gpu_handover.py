"""Hand-over of the split partials inside sc_decode_attn (Sec. 2.4, Eq. 4 computed split by split):
the two ways of moving partials give the same bits, and a hand-over that fails is reported (NaN outputs,
status word -1) and contained (no later call on that workspace returns a finite wrong result), with
every kernel still running to its end."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_14303_amd import binding as sc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cache(B, Hkv, G, cap, rows, seed, d=128, dtype=torch.bfloat16):
    g = torch.Generator(device="cpu").manual_seed(seed)
    Kc = torch.randn((B, Hkv, cap, d), generator=g).to(dtype).to(DEV)
    Vc = torch.randn((B, Hkv, cap, d), generator=g).to(dtype).to(DEV)
    counts = torch.randint(1, 9, (B, Hkv, cap), generator=g, dtype=torch.int32).to(DEV)
    lens = torch.tensor(rows, dtype=torch.int32).reshape(B, Hkv).to(DEV)
    Q = torch.randn((B, Hkv * G, d), generator=g).to(dtype).to(DEV)
    return Q, Kc, Vc, counts, lens


def _status(ws):
    return ws.buf[:4].view(torch.int32)


@pytest.mark.parametrize("B,Hkv,G,d,dtype", [(1, 8, 4, 128, torch.bfloat16), (2, 8, 2, 128, torch.bfloat16),
                                              (1, 8, 4, 64, torch.float32), (1, 3, 4, 128, torch.bfloat16)])
def test_local_and_remote_handover_agree_bit_for_bit(B, Hkv, G, d, dtype):
    cap = 3000
    rng = np.random.default_rng(5)
    rows = rng.integers(0, cap + 1, size=B * Hkv).tolist()
    rows[0] = cap
    Q, Kc, Vc, counts, lens = _cache(B, Hkv, G, cap, rows, seed=21, d=d, dtype=dtype)
    outs = []
    for mode in (1, 0):
        sc.tune_set("decode_local_handover", mode)
        try:
            O, lse = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True)
            torch.cuda.synchronize()
        finally:
            sc.tune_set("decode_local_handover", 1)
        outs.append((O, lse))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    # and both are right: the oracle on the same cache, one (sequence, head) with many splits
    b, h = 0, 0
    want, _ = oracle.decode_head(Q[b, h * G].float().cpu().numpy(), Kc[b, h].float().cpu().numpy(),
                                 Vc[b, h].float().cpu().numpy(), counts[b, h].cpu().numpy(), rows[0])
    got = outs[0][0][b, h * G].float().cpu().numpy()
    assert np.abs(got - want).max() <= (4e-3 if dtype == torch.bfloat16 else 2e-5) * max(1.0, np.abs(want).max())


def test_failed_handover_is_reported_and_contained():
    B, Hkv, G, cap = 1, 8, 4, 4096
    rows = [4096, 3000, 2000, 100, 4095, 2500, 1, 0]      # heads 3, 6, 7 have a single split: nothing to hand over
    Q, Kc, Vc, counts, lens = _cache(B, Hkv, G, cap, rows, seed=31)
    O_ref, lse_ref = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True)
    torch.cuda.synchronize()
    ws = sc.decode_attn_workspace(B, Hkv * G, Hkv, cap, 128, DEV)
    assert int(_status(ws).item()) == 0 and sc.check_lengths(_status(ws)) == -1
    # a good call first, so that the workspace holds real flags and partials of an earlier call
    O, lse = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(O, O_ref) and torch.equal(lse, lse_ref) and int(_status(ws).item()) == 0
    # the folding workgroups give up at once: every kernel still runs to its end
    sc.tune_set("decode_poll_budget", -1)
    try:
        O, lse = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
    finally:
        sc.tune_set("decode_poll_budget", 1 << 20)
    multi = [h for h in range(Hkv) if rows[h] > 192]
    single = [h for h in range(Hkv) if rows[h] <= 192]
    for h in multi:
        assert torch.isnan(O[0, h * G:(h + 1) * G].float()).all() and torch.isnan(lse[0, h * G:(h + 1) * G]).all()
    for h in single:
        assert torch.equal(O[0, h * G:(h + 1) * G], O_ref[0, h * G:(h + 1) * G])
    assert int(_status(ws).item()) == -1 and sc.check_lengths(_status(ws)) == 0
    # contained: the next call on the same workspace must not fold anything the failed call left behind
    O2, lse2 = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True, workspace=ws)
    torch.cuda.synchronize()
    for h in multi:
        assert torch.isnan(O2[0, h * G:(h + 1) * G].float()).all()
    for h in single:
        assert torch.equal(O2[0, h * G:(h + 1) * G], O_ref[0, h * G:(h + 1) * G])
    # initialising the workspace again makes it good again
    lib = sc.load_library()
    assert lib.sc_decode_attn_init_workspace(ws.ptr, ws.nbytes, B, Hkv, torch.cuda.current_stream().cuda_stream) == 0
    O3, lse3 = sc.sc_decode_attn(Q, Kc, Vc, counts, lens, want_lse=True, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(O3, O_ref) and torch.equal(lse3, lse_ref) and int(_status(ws).item()) == 0
