"""Pins for the CPU oracle: every check here compares it with something other than itself.

Eq. 1 (segmentation): brute force by rebuilding the mask, hand cases.
Alg. 1 (GSC): hand-worked angle cases (tests/golden), an independent token-major
  formulation, strictness of ">", degenerate thresholds, structural invariants.
Eq. 3 (merge): mass conservation, sizes, identity at tau >= 1.
Eq. 4 (attention): textbook softmax attention via scipy, exactness on duplicated
  rows (log s == repeating the row s times), permutation/constant-V invariants,
  split-and-combine.
"""
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
from paper_2603_14303_amd import workloads as wl
from helpers import build_case, reference_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Eq. 1
def _chunks_from_offsets(off, n):
    """(list of (start, end) chunk ranges, list of delimiter positions)"""
    M = len(off) - 1
    chunks = [(int(off[m]), int(off[m + 1]) - 1) for m in range(M)]
    delims = [int(off[m + 1]) - 1 for m in range(M) if off[m + 1] - 1 < n]
    return chunks, delims


@pytest.mark.parametrize("seed", range(6))
def test_segment_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(0, 300))
    mask = (rng.random(n) < rng.choice([0.0, 0.05, 0.3, 1.0])).astype(np.uint8)
    off = oracle.segment(mask, n)
    chunks, delims = _chunks_from_offsets(off, n)
    # delimiters are exactly the nonzero positions, in order
    assert delims == list(np.nonzero(mask)[0])
    assert len(chunks) == len(delims) + 1
    # rebuild the mask and the cover: every index is in exactly one chunk or is a delimiter
    cover = np.zeros(n, dtype=np.int32)
    for s, e in chunks:
        assert 0 <= s <= e <= n
        cover[s:e] += 1
        assert not mask[s:e].any()
    cover[delims] += 1
    assert (cover == 1).all()
    assert sum(e - s for s, e in chunks) + len(delims) == n


def test_segment_hand_cases():
    # no delimiter: one chunk = the whole sequence
    assert list(oracle.segment(np.zeros(5, np.uint8))) == [0, 6]
    # empty sequence: one empty chunk
    assert list(oracle.segment(np.zeros(0, np.uint8), 0)) == [0, 1]
    # leading, trailing and adjacent delimiters give empty chunks; both delimiters stay
    mask = np.array([1, 0, 0, 1, 1, 0, 1], np.uint8)
    off = oracle.segment(mask)
    assert list(off) == [0, 1, 4, 5, 7, 8]
    chunks, delims = _chunks_from_offsets(off, 7)
    assert chunks == [(0, 0), (1, 3), (4, 4), (5, 6), (7, 7)]
    assert delims == [0, 3, 4, 6]
    # all delimiters
    assert list(oracle.segment(np.ones(3, np.uint8))) == [0, 1, 2, 3, 4]
    # positions beyond n are ignored
    assert list(oracle.segment(np.array([0, 1, 0, 1], np.uint8), 3)) == [0, 2, 4]


# ------------------------------------------------------------------ Eq. 2
def test_cosine_known_values():
    assert oracle.cosine([1, 0], [3, 0]) == 1.0
    assert oracle.cosine([1, 0], [0, 2]) == 0.0
    assert oracle.cosine([1, 0], [-4, 0]) == -1.0
    assert abs(oracle.cosine([1, 1], [1, 0]) - np.sqrt(0.5)) < 1e-15
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal(128), rng.standard_normal(128)
    want = float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))
    assert abs(oracle.cosine(a, b) - want) < 1e-14
    assert np.isnan(oracle.cosine([0, 0], [1, 0]))


# ------------------------------------------------------------------ Alg. 1
def _golden_cases():
    out = []
    with open(os.path.join(GOLDEN, "gsc_angle_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, t, c = [p.strip() for p in line.split("|")]
            out.append(([float(x) for x in a.split()], float(t), [int(x) for x in c.split()]))
    return out


@pytest.mark.parametrize("angles,thr_deg,expect", _golden_cases())
def test_gsc_hand_worked_angles(angles, thr_deg, expect):
    a = np.deg2rad(np.array(angles))
    K = np.stack([np.cos(a), np.sin(a)], axis=1)
    cid, p, _, _ = oracle.gsc_chunk(K, np.cos(np.deg2rad(thr_deg)))
    assert list(cid) == expect
    assert p == max(expect) + 1
    # similarity ignores the key's length (Eq. 2 normalises both sides)
    cid2, _, _, _ = oracle.gsc_chunk(K * np.linspace(0.1, 7.0, len(angles))[:, None], np.cos(np.deg2rad(thr_deg)))
    assert list(cid2) == expect


def _leader_clustering(K, tau):
    """Token-major restatement of Alg. 1: token j joins the earliest seed with Sim > tau, else seeds."""
    K = np.asarray(K, dtype=np.float64)
    norms = np.sqrt((K * K).sum(axis=1))
    seeds, cid = [], []
    for j in range(K.shape[0]):
        placed = -1
        for c, s in enumerate(seeds):
            with np.errstate(invalid="ignore", divide="ignore"):
                sim = float(K[s] @ K[j]) / (norms[s] * norms[j])
            if sim > tau:
                placed = c
                break
        if placed < 0:
            seeds.append(j)
            placed = len(seeds) - 1
        cid.append(placed)
    return cid, seeds


@pytest.mark.parametrize("seed", range(12))
def test_gsc_matches_token_major_formulation(seed):
    rng = np.random.default_rng(100 + seed)
    l = int(rng.integers(1, 60))
    d = int(rng.choice([2, 3, 16, 64]))
    centers = rng.standard_normal((int(rng.integers(1, 5)), d))
    K = centers[rng.integers(0, centers.shape[0], l)] + 0.3 * rng.standard_normal((l, d))
    tau = float(rng.choice([0.2, 0.5, 0.7, 0.9, 0.97]))
    cid, p, margin, pairs = oracle.gsc_chunk(K, tau)
    want, seeds = _leader_clustering(K, tau)
    assert margin > 1e-9  # the comparison is not on a knife edge for this draw
    assert list(cid) == want and p == len(seeds)


def test_gsc_strict_inequality_and_degenerate_thresholds():
    K = np.array([[1.0, 0.0], [3.0, 0.0], [0.0, 1.0]])
    # cosine((1,0),(3,0)) is exactly 1: not merged at tau = 1 (strict ">")
    assert list(oracle.gsc_chunk(K, 1.0)[0]) == [0, 1, 2]
    # cosine((1,0),(0,1)) is exactly 0: not merged at tau = 0, merged just below
    assert list(oracle.gsc_chunk(K, 0.0)[0]) == [0, 0, 1]
    assert list(oracle.gsc_chunk(K, -1e-9)[0]) == [0, 0, 0]
    rng = np.random.default_rng(5)
    K = rng.standard_normal((17, 8))
    assert list(oracle.gsc_chunk(K, 1.0)[0]) == list(range(17))      # tau >= 1: all singletons
    assert list(oracle.gsc_chunk(K, -1.01)[0]) == [0] * 17           # tau < -1: one cluster
    # duplicated rows merge with their first occurrence for any tau < 1
    K2 = np.concatenate([K[:3], K[:3]])
    cid = oracle.gsc_chunk(K2, 0.999)[0]
    assert list(cid[3:]) == list(cid[:3])
    # zero-norm key: similarity undefined -> never merged, never absorbs
    K3 = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 0.0], [2.0, 0.0]])
    assert list(oracle.gsc_chunk(K3, -1.01)[0]) == [0, 1, 2, 1]
    # empty chunk and single token
    assert oracle.gsc_chunk(np.zeros((0, 4)), 0.5)[1] == 0
    assert list(oracle.gsc_chunk(np.ones((1, 4)), 0.5)[0]) == [0]


def _sim_matrix(K):
    K = np.asarray(K, dtype=np.float64)
    nrm = np.sqrt((K * K).sum(axis=1))
    return (K @ K.T) / np.outer(nrm, nrm)


@pytest.mark.parametrize("tau", [0.7, 0.9745, 0.03])
def test_gsc_structural_invariants_on_workload_chunks(tau):
    w = wl.get_workload("tiny")
    mask = wl.delimiter_mask(w, 0)
    off = oracle.segment(mask, w.n_max)
    K, _ = wl.keys_values(w, 0, 0, 1, mask, w.n_max)
    checked = 0
    for m in range(len(off) - 1):
        s, e = int(off[m]), int(off[m + 1]) - 1
        if e - s < 2:
            continue
        cid, p, _, pairs = oracle.gsc_chunk(K[s:e], tau)
        S = _sim_matrix(K[s:e])
        seeds = [int(np.nonzero(cid == c)[0][0]) for c in range(p)]
        assert seeds == sorted(seeds) and seeds[0] == 0         # first token seeds cluster 0
        for c, i in enumerate(seeds):
            members = np.nonzero(cid == c)[0]
            assert (members >= i).all()
            assert all(S[i, j] > tau for j in members if j != i)   # every member beats tau against its seed
            for i2 in seeds[c + 1:]:
                assert not (S[i, i2] > tau)                         # later seeds were refused by earlier seeds
        for j in range(e - s):
            for i in seeds[: cid[j]]:
                if i < j:
                    assert not (S[i, j] > tau)                      # refused by every earlier seed before it
        # number of evaluated pairs == what the two loops visit
        visited = 0
        assigned = np.zeros(e - s, bool)
        for c, i in enumerate(seeds):
            assigned[i] = True
            visited += int((~assigned[i + 1:]).sum())
            assigned |= (cid == c)
        assert pairs == visited
        checked += 1
    assert checked > 10


# ------------------------------------------------------------------ Eq. 3
@pytest.mark.parametrize("tau", [0.7, 0.9745])
def test_merge_conservation_and_layout(tau):
    case = build_case(wl.get_workload("tiny"), tau)
    n = int(case["seq_lens"][0])
    off = case["offsets"][0]
    M = len(off) - 1
    for h in range(2):
        r = case["ref"][(0, h)]
        K, V = case["K"][0, h].astype(np.float64), case["V"][0, h].astype(np.float64)
        rows, counts, cid = r["n_rows"], r["counts"], r["cid"]
        assert counts[:rows].sum() == n                      # sizes add up to the sequence length
        assert (counts[:rows] >= 1).all()
        row = 0
        for m in range(M):
            s, e = int(off[m]), int(off[m + 1]) - 1
            p = int(cid[s:e].max()) + 1 if e > s else 0
            assert counts[row:row + p].sum() == e - s        # sizes add up to the chunk length
            for c in range(p):
                members = s + np.nonzero(cid[s:e] == c)[0]
                assert counts[row + c] == len(members)
                # Eq. 3 restated with numpy: the core is the arithmetic mean of its members
                assert np.allclose(r["Kc"][row + c], K[members].mean(axis=0), rtol=0, atol=1e-12)
                assert np.allclose(r["Vc"][row + c], V[members].mean(axis=0), rtol=0, atol=1e-12)
                if len(members) == 1:
                    assert (r["Kc"][row + c] == K[members[0]]).all() and (r["Vc"][row + c] == V[members[0]]).all()
            # mass conservation per chunk: sum_t s_t * core_t == sum of the chunk's rows
            assert np.allclose((counts[row:row + p, None] * r["Kc"][row:row + p]).sum(0), K[s:e].sum(0), atol=1e-10)
            assert np.allclose((counts[row:row + p, None] * r["Vc"][row:row + p]).sum(0), V[s:e].sum(0), atol=1e-10)
            row += p
            if e < n:                                         # the delimiter follows, untouched, size 1
                assert case["mask"][0, e] != 0 and cid[e] == -1
                assert counts[row] == 1
                assert (r["Kc"][row] == K[e]).all() and (r["Vc"][row] == V[e]).all()
                row += 1
        assert row == rows
        assert (case["mask"][0, :n][cid == -1] != 0).all() and ((cid == -1) == (case["mask"][0, :n] != 0)).all()


def test_merge_identity_when_nothing_merges():
    case = build_case(wl.get_workload("tiny"), 1.0)
    n = int(case["seq_lens"][0])
    for h in range(2):
        r = case["ref"][(0, h)]
        assert r["n_rows"] == n
        assert (r["counts"][:n] == 1).all()
        assert (r["Kc"][:n] == case["K"][0, h]).all() and (r["Vc"][:n] == case["V"][0, h]).all()


def test_merge_one_cluster_per_chunk_when_everything_merges():
    case = build_case(wl.get_workload("tiny"), -1.01)
    off = case["offsets"][0]
    n = int(case["seq_lens"][0])
    lens = np.diff(off) - 1
    n_delims = len(off) - 2
    for h in range(2):
        r = case["ref"][(0, h)]
        assert r["n_rows"] == int((lens > 0).sum()) + n_delims
        assert r["counts"][: r["n_rows"]].sum() == n


def test_merge_respects_capacity():
    w = wl.get_workload("tiny")
    mask = wl.delimiter_mask(w, 0)
    off = oracle.segment(mask, w.n_max)
    K, V = wl.keys_values(w, 0, 0, 0, mask, w.n_max)
    full = oracle.compress_head(K, V, off, 0.7)
    small = oracle.compress_head(K, V, off, 0.7, cap=10)
    assert small["n_rows"] == full["n_rows"] > 10
    assert (small["Kc"] == full["Kc"][:10]).all()


# ------------------------------------------------------------------ Eq. 4
def test_decode_counts_one_is_textbook_attention():
    rng = np.random.default_rng(1)
    for d, n in [(64, 1), (64, 37), (128, 300)]:
        K, V, q = rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal(d)
        out, lse = oracle.decode_head(q, K, V, np.ones(n, np.int32), n)
        want = reference_attention(q, K, V, 1.0 / np.sqrt(d))
        assert np.allclose(out, want, rtol=0, atol=1e-13)
        assert abs(lse - logsumexp(K @ q / np.sqrt(d))) < 1e-12


def test_decode_log_size_equals_repeating_rows():
    # Adding log s to a logit == listing that row s times (Sec. 2.4, remark after Eq. 4).
    rng = np.random.default_rng(2)
    d, r = 32, 9
    K, V, q = rng.standard_normal((r, d)), rng.standard_normal((r, d)), rng.standard_normal(d)
    s = rng.integers(1, 7, r).astype(np.int32)
    out, lse = oracle.decode_head(q, K, V, s, r, scale=0.3)
    Kx, Vx = np.repeat(K, s, axis=0), np.repeat(V, s, axis=0)
    want = softmax(Kx @ q * 0.3) @ Vx
    assert np.allclose(out, want, rtol=0, atol=1e-13)
    assert abs(lse - logsumexp(Kx @ q * 0.3)) < 1e-12
    # and it differs from ignoring the sizes
    plain, _ = oracle.decode_head(q, K, V, np.ones(r, np.int32), r, scale=0.3)
    assert np.abs(plain - out).max() > 1e-3


def test_decode_invariants():
    rng = np.random.default_rng(3)
    d, n = 16, 50
    K, V, q = rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal(d)
    s = rng.integers(1, 9, n).astype(np.int32)
    out, lse = oracle.decode_head(q, K, V, s, n)
    perm = rng.permutation(n)
    out_p, lse_p = oracle.decode_head(q, K[perm], V[perm], s[perm], n)
    assert np.allclose(out, out_p, atol=1e-13) and abs(lse - lse_p) < 1e-12
    const = np.tile(rng.standard_normal(d), (n, 1))
    assert np.allclose(oracle.decode_head(q, K, const, s, n)[0], const[0], atol=1e-13)
    assert (out <= V.max(0) + 1e-12).all() and (out >= V.min(0) - 1e-12).all()
    # split-and-combine of partial (lse, out)
    o1, l1 = oracle.decode_head(q, K[:20], V[:20], s[:20], 20)
    o2, l2 = oracle.decode_head(q, K[20:], V[20:], s[20:], 30)
    w1, w2 = np.exp(l1 - lse), np.exp(l2 - lse)
    assert abs(w1 + w2 - 1) < 1e-12 and np.allclose(w1 * o1 + w2 * o2, out, atol=1e-13)
    # only the first n_rows rows are read; empty cache gives zeros and lse = -inf
    assert np.allclose(oracle.decode_head(q, K, V, s, 20)[0], o1, atol=0)
    oe, le = oracle.decode_head(q, K, V, s, 0)
    assert (oe == 0).all() and le == -np.inf
    # the scale argument defaults to 1/sqrt(d)
    assert np.allclose(oracle.decode_head(q, K, V, s, n, scale=0.25)[0], out, atol=0)


def test_decode_gqa_head_mapping():
    rng = np.random.default_rng(4)
    B, Hkv, G, d, cap = 2, 3, 4, 8, 12
    Q = rng.standard_normal((B, Hkv * G, d))
    Kc, Vc = rng.standard_normal((B, Hkv, cap, d)), rng.standard_normal((B, Hkv, cap, d))
    counts = rng.integers(1, 5, (B, Hkv, cap)).astype(np.int32)
    lens = rng.integers(1, cap + 1, (B, Hkv)).astype(np.int32)
    O, L = oracle.decode_attn(Q, Kc, Vc, counts, lens)
    for b in range(B):
        for hq in range(Hkv * G):
            h, n = hq // G, lens[b, hq // G]
            z = Kc[b, h, :n] @ Q[b, hq] / np.sqrt(d) + np.log(counts[b, h, :n])
            assert np.allclose(O[b, hq], softmax(z) @ Vc[b, h, :n], atol=1e-13)


# ------------------------------------------------------------------ decode-time growth
def test_decode_tail_is_attention_over_cache_plus_new_tokens():
    rng = np.random.default_rng(11)
    B, Hkv, G, d, cap, tcap = 2, 2, 3, 16, 10, 7
    Q = rng.standard_normal((B, Hkv * G, d))
    Kc, Vc = rng.standard_normal((B, Hkv, cap, d)), rng.standard_normal((B, Hkv, cap, d))
    Kt, Vt = rng.standard_normal((B, Hkv, tcap, d)), rng.standard_normal((B, Hkv, tcap, d))
    counts = rng.integers(1, 6, (B, Hkv, cap)).astype(np.int32)
    lens = np.array([[10, 4], [0, 7]], dtype=np.int32)
    tails = np.array([5, 0], dtype=np.int32)
    O, L = oracle.decode_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, tails)
    for b in range(B):
        for hq in range(Hkv * G):
            h, n, t = hq // G, lens[b, hq // G], tails[b]
            # written out with scipy: merged rows carry ln s, new tokens carry nothing
            z = np.concatenate([Kc[b, h, :n] @ Q[b, hq] / np.sqrt(d) + np.log(counts[b, h, :n]),
                                Kt[b, h, :t] @ Q[b, hq] / np.sqrt(d)])
            vv = np.concatenate([Vc[b, h, :n], Vt[b, h, :t]])
            if n + t == 0:
                assert (O[b, hq] == 0).all() and L[b, hq] == -np.inf
            else:
                assert np.allclose(O[b, hq], softmax(z) @ vv, atol=1e-13)
                assert abs(L[b, hq] - logsumexp(z)) < 1e-12
    # no tail at all: the plain call
    O0, L0 = oracle.decode_attn(Q, Kc, Vc, counts, lens)
    O1, L1 = oracle.decode_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, np.zeros(B, np.int32))
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)
    # tail only, nothing merged: textbook attention over the new tokens
    O2, _ = oracle.decode_attn_tail(Q, Kc, Vc, counts, np.zeros((B, Hkv), np.int32), Kt, Vt, np.full(B, tcap, np.int32))
    for b in range(B):
        for hq in range(Hkv * G):
            want = reference_attention(Q[b, hq], Kt[b, hq // G], Vt[b, hq // G], 1.0 / np.sqrt(d))
            assert np.allclose(O2[b, hq], want, atol=1e-13)


def test_append_equals_compressing_the_whole_sequence_when_cut_at_a_delimiter():
    # Alg. 1 never looks across a delimiter, so compressing a prefix that ends with a delimiter and then
    # appending the rest must give the rows of compressing everything at once.
    w = wl.get_workload("tiny")
    mask = wl.delimiter_mask(w, 0)
    n = len(mask)
    K, V = wl.keys_values(w, 0, 0, 0, mask, n)
    tau = 0.7
    off = oracle.segment(mask)
    whole = oracle.compress_head(K, V, off, tau)
    delims = np.nonzero(mask)[0]
    for cut_at in (delims[0], delims[len(delims) // 2], delims[-1]):
        cut = int(cut_at) + 1                                  # first token after the delimiter
        head = oracle.compress_head(K[:cut], V[:cut], oracle.segment(mask[:cut]), tau)
        # the prefix ends with a delimiter, so its last chunk (after it) is empty and adds no row
        both = oracle.append_head(head, K[cut:], V[cut:], oracle.segment(mask[cut:]), tau, cap=n)
        assert both["n_rows"] == whole["n_rows"]
        r = whole["n_rows"]
        assert np.array_equal(both["counts"][:r], whole["counts"][:r])
        assert np.array_equal(both["Kc"][:r], whole["Kc"][:r]) and np.array_equal(both["Vc"][:r], whole["Vc"][:r])
    # capacity: the total is reported even when rows are dropped
    small = oracle.append_head(head, K[cut:], V[cut:], oracle.segment(mask[cut:]), tau, cap=head["n_rows"] + 1)
    assert small["n_rows"] == whole["n_rows"] and small["counts"][head["n_rows"]] == whole["counts"][head["n_rows"]]


def test_multi_query_attention_is_the_matrix_form_of_eq4():
    # A = softmax(Q Kc^T / sqrt(d) + log s) Vc with Q a matrix (Sec. 2.4), written with numpy matrices
    rng = np.random.default_rng(21)
    nq, B, Hkv, G, d, cap = 5, 2, 2, 3, 16, 11
    Q = rng.standard_normal((nq, B, Hkv * G, d))
    Kc, Vc = rng.standard_normal((B, Hkv, cap, d)), rng.standard_normal((B, Hkv, cap, d))
    counts = rng.integers(1, 6, (B, Hkv, cap)).astype(np.int32)
    lens = np.array([[11, 3], [7, 0]], dtype=np.int32)
    O, L = oracle.multi_attn(Q, Kc, Vc, counts, lens)
    for b in range(B):
        for hq in range(Hkv * G):
            h, n = hq // G, lens[b, hq // G]
            if n == 0:
                assert (O[:, b, hq] == 0).all() and np.isneginf(L[:, b, hq]).all()
                continue
            Z = Q[:, b, hq] @ Kc[b, h, :n].T / np.sqrt(d) + np.log(counts[b, h, :n])[None, :]
            assert np.allclose(O[:, b, hq], softmax(Z, axis=1) @ Vc[b, h, :n], atol=1e-13)
            assert np.allclose(L[:, b, hq], logsumexp(Z, axis=1), atol=1e-12)


def test_multi_query_tail_with_causal_mask_is_masked_softmax():
    # the matrix form with an explicit mask: -inf above the diagonal of the queries' own tokens
    rng = np.random.default_rng(31)
    nq, B, Hkv, G, d, cap, tcap = 4, 2, 2, 2, 8, 6, 7
    Q = rng.standard_normal((nq, B, Hkv * G, d))
    Kc, Vc = rng.standard_normal((B, Hkv, cap, d)), rng.standard_normal((B, Hkv, cap, d))
    Kt, Vt = rng.standard_normal((B, Hkv, tcap, d)), rng.standard_normal((B, Hkv, tcap, d))
    counts = rng.integers(1, 5, (B, Hkv, cap)).astype(np.int32)
    lens = np.array([[6, 2], [0, 5]], dtype=np.int32)
    tails = np.array([7, 2], dtype=np.int32)          # the second tail is shorter than the query block
    for causal in (True, False):
        O, L = oracle.multi_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, tails, causal)
        for b in range(B):
            for hq in range(Hkv * G):
                h, n, t = hq // G, lens[b, hq // G], tails[b]
                Z = np.concatenate([Q[:, b, hq] @ Kc[b, h, :n].T / np.sqrt(d) + np.log(counts[b, h, :n])[None, :],
                                    Q[:, b, hq] @ Kt[b, h, :t].T / np.sqrt(d)], axis=1)
                if causal:
                    for j in range(nq):
                        Z[j, n + max(0, t - nq + 1 + j):] = -np.inf
                VV = np.concatenate([Vc[b, h, :n], Vt[b, h, :t]])
                for j in range(nq):
                    if np.isneginf(Z[j]).all():
                        assert (O[j, b, hq] == 0).all() and np.isneginf(L[j, b, hq])
                    else:
                        assert np.allclose(O[j, b, hq], softmax(Z[j]) @ VV, atol=1e-13)
                        assert abs(L[j, b, hq] - logsumexp(Z[j])) < 1e-12
    # without a mask and with an empty tail it is multi_attn
    O0, L0 = oracle.multi_attn(Q, Kc, Vc, counts, lens)
    O1, L1 = oracle.multi_attn_tail(Q, Kc, Vc, counts, lens, Kt, Vt, np.zeros(B, np.int32), False)
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)


def test_budget_threshold_brackets_the_budget():
    # on real compression counts: the threshold found fits the budget, and raising it by the final
    # width of the bracket no longer does (when the bracket started valid); a brute-force scan of a
    # fine grid agrees on which side of the result fits
    w = wl.get_workload("tiny")
    mask = wl.delimiter_mask(w, 0)
    n = len(mask)
    off = oracle.segment(mask)
    KV = [wl.keys_values(w, 0, 0, h, mask, n) for h in range(2)]
    cache = {}

    def rows_at(tau):
        if tau not in cache:
            cache[tau] = sum(oracle.compress_head(K, V, off, tau)["n_rows"] for K, V in KV)
        return cache[tau]

    grid = np.linspace(-1.0, 1.0, 81)
    counts = [rows_at(float(t)) for t in grid]
    assert all(a <= b for a, b in zip(counts, counts[1:])), "rows must not shrink as the threshold rises (on this data)"
    total = 2 * n
    for frac in (0.2, 0.35, 0.5, 0.9):
        budget = int(round(frac * total))
        tau, probed = oracle.tau_for_budget(rows_at, budget, -1.01, 1.0, 14)
        assert len(probed) == 14 and probed[0] == float(np.float32(0.5) * (np.float32(-1.01) + np.float32(1.0)))
        if rows_at(-1.01) > budget:
            assert tau == np.float32(-1.01)
            continue
        assert rows_at(float(tau)) <= budget
        width = 2.01 / 2 ** 14
        assert rows_at(min(1.0, float(tau) + 1.01 * width)) > budget or float(tau) + 1.01 * width >= 1.0
        for t, c in zip(grid, counts):          # the grid agrees wherever it is clear of the bracket
            if t <= float(tau):
                assert c <= budget
            elif t > float(tau) + 1.01 * width:
                assert c > budget
    # no iterations: lo comes back unprobed
    assert oracle.tau_for_budget(rows_at, 5, 0.25, 0.75, 0)[0] == np.float32(0.25)


# ------------------------------------------------------------------ end to end
def test_pipeline_at_tau_one_is_full_cache_attention():
    w = wl.get_workload("tiny")
    case = build_case(w, 1.0)
    Q = wl.queries(w, 0, 0)
    n = int(case["seq_lens"][0])
    for h in range(2):
        r = case["ref"][(0, h)]
        out, _ = oracle.decode_head(Q[0, h], r["Kc"], r["Vc"], r["counts"], r["n_rows"])
        want = reference_attention(Q[0, h], case["K"][0, h, :n], case["V"][0, h, :n], 1.0 / np.sqrt(w.head_dim))
        assert np.allclose(out, want, rtol=0, atol=1e-13)


def test_merged_attention_underestimates_cluster_mass():
    # Jensen: s * exp(q . mean(k)) <= sum exp(q . k_i) for every cluster.
    w = wl.get_workload("tiny")
    case = build_case(w, 0.7)
    q = wl.queries(w, 0, 1)[0, 0].astype(np.float64) / np.sqrt(w.head_dim)
    r = case["ref"][(0, 0)]
    K = case["K"][0, 0].astype(np.float64)
    off, cid = case["offsets"][0], r["cid"]
    row = 0
    for m in range(len(off) - 1):
        s, e = int(off[m]), int(off[m + 1]) - 1
        p = int(cid[s:e].max()) + 1 if e > s else 0
        for c in range(p):
            members = s + np.nonzero(cid[s:e] == c)[0]
            merged = r["counts"][row + c] * np.exp(q @ r["Kc"][row + c])
            assert merged <= np.exp(K[members] @ q).sum() * (1 + 1e-12)
        row += p + (1 if e < int(case["seq_lens"][0]) else 0)
