"""Randomised structures on the GPU: many small sequences with unusual chunk layouts (runs of delimiters,
no delimiter, chunks far longer than a window, chunks of one token), key mixtures with up to a dozen
centres, exact duplicates, zero rows, and thresholds inside the similarity bands.  Integers must match
the oracle bit for bit, merged rows within the usual bound.  Seeds are fixed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_14303_amd import binding as sc
from paper_2603_14303_amd import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_common as g


def _random_mask(rng, n):
    kind = rng.integers(0, 6)
    m = np.zeros(n, np.uint8)
    if kind == 0:                                   # geometric gaps, short
        p = np.cumsum(rng.geometric(1.0 / rng.integers(2, 30), size=n)) - 1
        m[p[p < n]] = 1
    elif kind == 1:                                 # a few very long chunks
        p = np.cumsum(rng.integers(60, 400, size=n // 60 + 1)) - 1
        m[p[p < n]] = 1
    elif kind == 2:                                 # runs of delimiters and single-token chunks
        m[rng.random(n) < 0.5] = 1
    elif kind == 3:                                 # no delimiter at all
        pass
    elif kind == 4:                                 # chunk lengths around the window size
        p = np.cumsum(rng.integers(28, 70, size=n // 28 + 1)) - 1
        m[p[p < n]] = 1
    else:                                           # leading and trailing delimiters, mixed gaps
        p = np.cumsum(rng.choice([1, 2, 17, 33, 64, 65, 129], size=n)) - 1
        m[p[p < n]] = 1
        m[0] = 1
        m[n - 1] = 1
    return m


def _random_keys(rng, mask, n, d, bf16):
    cid = np.concatenate([[0], np.cumsum(mask[:n - 1])]).astype(np.int64)
    n_chunks = int(cid.max()) + 1
    max_c = int(rng.integers(1, 13))
    centres = rng.standard_normal((n_chunks, max_c, d)).astype(np.float32)
    n_c = rng.integers(1, max_c + 1, size=n_chunks)
    pick = np.floor(rng.random(n) * n_c[cid]).astype(np.int64)
    noise = np.float32(rng.choice([0.0, 0.05, 0.15, 0.4]))
    K = centres[cid, pick] + noise * rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    K[rng.random(n) < 0.01] = 0.0                                   # zero-norm keys
    dup = np.nonzero(rng.random(n) < 0.05)[0]
    dup = dup[dup > 0]
    K[dup] = K[dup - 1]                                             # exact duplicates of the previous token
    K *= rng.choice([1.0, 0.01, 30.0], size=(n, 1)).astype(np.float32)   # cosine does not care about scale
    if bf16:
        K, V = wl.round_to_bf16(K), wl.round_to_bf16(V)
    return K, V


@pytest.mark.parametrize("bf16,d,seed", [(True, 128, s) for s in range(24)] + [(False, 64, s) for s in range(100, 106)])
def test_random_structures(bf16, d, seed):
    rng = np.random.default_rng(seed)
    B, H = 3, 2
    N = int(rng.integers(200, 1500))
    lens = rng.integers(1, N + 1, size=B).astype(np.int32)
    lens[0] = N
    mask = np.zeros((B, N), np.uint8)
    K = np.zeros((B, H, N, d), np.float32)
    V = np.zeros_like(K)
    for b in range(B):
        n = int(lens[b])
        mask[b, :n] = _random_mask(rng, n)
        for h in range(H):
            K[b, h, :n], V[b, h, :n] = _random_keys(rng, mask[b], n, d, bf16)
    tau = float(rng.choice([0.3, 0.7, 0.9, 0.97, 0.985, 0.995, 0.9999, -0.5]))
    dK, dV = g.to_device(K, bf16), g.to_device(V, bf16)
    off, nch, sl = g.check_segment(mask, lens)
    Kc, Vc, counts, clens, cid = sc.sc_gsc_merge(dK, dV, off, nch, tau, seq_lens=sl, out_dtype=torch.float32,
                                                 want_cluster_id=True)
    torch.cuda.synchronize()
    worst = 0.0
    compared = skipped = 0
    for b in range(B):
        n = int(lens[b])
        o = oracle.segment(mask[b], n)
        for h in range(H):
            r = oracle.compress_head(K[b, h, :n], V[b, h, :n], o, tau)
            if r["chunk_margin"].min() <= 1e-9:
                skipped += 1
                continue                                             # a coin toss in fp64 itself: not a parity case
            compared += 1
            rows = r["n_rows"]
            assert int(clens[b, h]) == rows, (seed, b, h, int(clens[b, h]), rows)
            assert np.array_equal(cid[b, h, :n].cpu().numpy(), r["cid"]), (seed, b, h)
            assert np.array_equal(counts[b, h, :rows].cpu().numpy(), r["counts"][:rows]), (seed, b, h)
            ek = g.rowwise_err(Kc[b, h, :rows].cpu().numpy(), r["Kc"][:rows])
            ev = g.rowwise_err(Vc[b, h, :rows].cpu().numpy(), r["Vc"][:rows])
            worst = max(worst, ek, ev)
            assert ek <= 1e-3 and ev <= 1e-3, (seed, b, h, ek, ev)
    # exact ties are possible (duplicated rows at tau just below 1) but must stay the exception
    assert compared >= (B * H + 1) // 2, (seed, compared, skipped)
    print("seed", seed, "compared", compared, "skipped", skipped, "N", N, "lens", lens.tolist(), "tau", tau, "rows", clens.cpu().numpy().tolist(), "err %.1e" % worst)


@pytest.mark.parametrize("bf16,d,seed", [(True, 128, 300), (False, 64, 301)])
def test_thousands_of_short_chunks(bf16, d, seed):
    """A delimiter every few tokens: more chunks than one round of the relocation's count sum holds (2048)
    and more tasks than the compress grid has workgroups per head, on a ragged batch."""
    rng = np.random.default_rng(seed)
    B, H, N = 2, 2, 24576
    lens = np.array([N, 15001], np.int32)
    mask = np.zeros((B, N), np.uint8)
    K = np.zeros((B, H, N, d), np.float32)
    V = np.zeros_like(K)
    for b in range(B):
        n = int(lens[b])
        p = np.cumsum(rng.integers(1, 8, size=n)) - 1
        mask[b, p[p < n]] = 1
        for h in range(H):
            K[b, h, :n], V[b, h, :n] = _random_keys(rng, mask[b], n, d, bf16)
    tau = 0.9
    dK, dV = g.to_device(K, bf16), g.to_device(V, bf16)
    off, nch, sl = g.check_segment(mask, lens)
    assert int(nch.min()) > 2048 and int(nch.max()) > 6000
    Kc, Vc, counts, clens, cid = sc.sc_gsc_merge(dK, dV, off, nch, tau, seq_lens=sl, out_dtype=torch.float32,
                                                 want_cluster_id=True)
    torch.cuda.synchronize()
    compared = 0
    for b in range(B):
        n = int(lens[b])
        o = oracle.segment(mask[b], n)
        for h in range(H):
            r = oracle.compress_head(K[b, h, :n], V[b, h, :n], o, tau)
            if r["chunk_margin"].min() <= 1e-9:
                continue
            compared += 1
            rows = r["n_rows"]
            assert int(clens[b, h]) == rows, (b, h, int(clens[b, h]), rows)
            assert np.array_equal(cid[b, h, :n].cpu().numpy(), r["cid"]), (b, h)
            assert np.array_equal(counts[b, h, :rows].cpu().numpy(), r["counts"][:rows]), (b, h)
            ek = g.rowwise_err(Kc[b, h, :rows].cpu().numpy(), r["Kc"][:rows])
            ev = g.rowwise_err(Vc[b, h, :rows].cpu().numpy(), r["Vc"][:rows])
            assert ek <= 1e-3 and ev <= 1e-3, (b, h, ek, ev)
    assert compared >= 2, compared


@pytest.mark.parametrize("seed,long_chunks", [(400, False), (401, True), (402, True)])
def test_threshold_inside_a_narrow_band_of_similarities(seed, long_chunks):
    """Every chunk is one tight bundle: all pairwise cosines lie within a few 1e-4 of each other and tau is
    their median, so a large share of the pairs falls inside the band that the fp32 Gram product cannot
    decide, "resembles" is far from transitive, and whether a row is a seed hinges on fp64 decisions about
    earlier rows.  Cluster indices must still equal the oracle's."""
    rng = np.random.default_rng(seed)
    B, H, N, d = 1, 3, 2600, 128
    lens = np.array([N], np.int32)
    mask = np.zeros((B, N), np.uint8)
    gaps = rng.integers(70, 260, size=N // 70 + 1) if long_chunks else rng.choice([9, 17, 24, 33, 48, 63], size=N // 9 + 1)
    p = np.cumsum(gaps) - 1
    mask[0, p[p < N]] = 1
    cid_tok = np.concatenate([[0], np.cumsum(mask[0, :N - 1])]).astype(np.int64)
    K = np.zeros((B, H, N, d), np.float32)
    V = wl.round_to_bf16(rng.standard_normal((B, H, N, d)).astype(np.float32))
    taus = []
    for h in range(H):
        centre = rng.standard_normal((int(cid_tok.max()) + 1, d)).astype(np.float32)
        centre /= np.linalg.norm(centre, axis=1, keepdims=True)
        noise = rng.standard_normal((N, d)).astype(np.float32) / np.sqrt(d)
        K[0, h] = wl.round_to_bf16(centre[cid_tok] + 0.05 * noise)
    # one threshold for all heads: the median cosine over the pairs inside the chunks of head 0
    k0 = K[0, 0].astype(np.float64)
    k0 /= np.linalg.norm(k0, axis=1, keepdims=True)
    cos = []
    for c in range(int(cid_tok.max()) + 1):
        rows = np.nonzero((cid_tok == c) & (mask[0] == 0))[0]
        if len(rows) > 1:
            gm = k0[rows] @ k0[rows].T
            cos.append(gm[np.triu_indices(len(rows), 1)])
    cos = np.concatenate(cos)
    tau = float(np.float32(np.median(cos)))
    in_band = float(np.mean(np.abs(cos - tau) < 1e-4))
    assert in_band > 0.1, in_band
    dK, dV = g.to_device(K, True), g.to_device(V, True)
    off, nch, sl = g.check_segment(mask, lens)
    Kc, Vc, counts, clens, cid = sc.sc_gsc_merge(dK, dV, off, nch, tau, seq_lens=sl, out_dtype=torch.float32,
                                                 want_cluster_id=True)
    torch.cuda.synchronize()
    o = oracle.segment(mask[0], N)
    compared = 0
    for h in range(H):
        r = oracle.compress_head(K[0, h], V[0, h], o, tau)
        if r["chunk_margin"].min() <= 1e-9:
            continue
        compared += 1
        rows = r["n_rows"]
        assert int(clens[0, h]) == rows, (h, int(clens[0, h]), rows)
        assert np.array_equal(cid[0, h].cpu().numpy(), r["cid"]), h
        assert np.array_equal(counts[0, h, :rows].cpu().numpy(), r["counts"][:rows]), h
        ek = g.rowwise_err(Kc[0, h, :rows].cpu().numpy(), r["Kc"][:rows])
        ev = g.rowwise_err(Vc[0, h, :rows].cpu().numpy(), r["Vc"][:rows])
        assert ek <= 1e-3 and ev <= 1e-3, (h, ek, ev)
    assert compared >= 2, compared
    print("seed", seed, "tau", tau, "pairs inside the band %.2f" % in_band, "rows", clens.cpu().numpy().tolist())


def test_chains_where_every_row_resembles_only_its_neighbours():
    """Keys that turn by a fixed angle from row to row: a row resembles its neighbours and nobody else, so
    seeds and members alternate along the chunk and whether a row is a seed depends on every row before
    it.  A set-at-once decision of the seeds needs as many steps as the chunk has rows; chunks of 10 to
    200 rows (inside a window, filling one, spanning several blocks) must come out as in the oracle."""
    rng = np.random.default_rng(77)
    d, H = 128, 2
    lengths = [10, 40, 63, 5, 100, 30, 200, 64, 17, 130, 48, 48, 90]
    N = sum(lengths) + len(lengths)
    mask = np.zeros((1, N), np.uint8)
    K = np.zeros((1, H, N, d), np.float32)
    pos = 0
    for L in lengths:
        for h in range(H):
            theta = 0.15 if h == 0 else 0.11                       # cos 0.9888 / 0.9940; two steps: 0.9553 / 0.9759
            basis = np.linalg.qr(rng.standard_normal((d, 2)))[0]    # a random plane
            # (a chunk too long for one turn of the circle repeats angles: runs of identical rows in the chain)
            ang = theta * np.arange(L) if theta * L < 6.0 else np.cumsum(np.r_[0.0, rng.choice([theta, 0.0], size=L - 1, p=[0.3, 0.7])])
            K[0, h, pos:pos + L] = np.cos(ang)[:, None] * basis[:, 0] + np.sin(ang)[:, None] * basis[:, 1]
            K[0, h, pos + L] = rng.standard_normal(d)
        mask[0, pos + L] = 1
        pos += L + 1
    K = wl.round_to_bf16(K * 3.0)
    V = wl.round_to_bf16(rng.standard_normal((1, H, N, d)).astype(np.float32))
    lens = np.array([N], np.int32)
    dK, dV = g.to_device(K, True), g.to_device(V, True)
    off, nch, sl = g.check_segment(mask, lens)
    o = oracle.segment(mask[0], N)
    for tau in (0.97, 0.985):
        Kc, Vc, counts, clens, cid = sc.sc_gsc_merge(dK, dV, off, nch, tau, seq_lens=sl, out_dtype=torch.float32,
                                                     want_cluster_id=True)
        torch.cuda.synchronize()
        for h in range(H):
            r = oracle.compress_head(K[0, h], V[0, h], o, tau)
            assert r["chunk_margin"].min() > 1e-9, (tau, h, r["chunk_margin"].min())
            rows = r["n_rows"]
            assert int(clens[0, h]) == rows, (tau, h, int(clens[0, h]), rows)
            assert np.array_equal(cid[0, h].cpu().numpy(), r["cid"]), (tau, h)
            assert np.array_equal(counts[0, h, :rows].cpu().numpy(), r["counts"][:rows]), (tau, h)
            ek = g.rowwise_err(Kc[0, h, :rows].cpu().numpy(), r["Kc"][:rows])
            ev = g.rowwise_err(Vc[0, h, :rows].cpu().numpy(), r["Vc"][:rows])
            assert ek <= 1e-3 and ev <= 1e-3, (tau, h, ek, ev)
        print("tau", tau, "rows", clens.cpu().numpy().tolist())
