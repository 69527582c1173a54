"""Pins for the oracle's mining and sampling functions (CPU only).

Each test checks the oracle against something other than its own formula: a
planted answer known by construction, pure-Python brute force, exhaustive
enumeration, published generator vectors, or a statistical law.
"""
import os

import numpy as np
import pytest

from oracle import astra_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- mining ----
def test_mine_planted_axis_rows():
    # w_l = c_l * e_{l mod d}, z_i = e_i  =>  score(i,l) = c_l if l mod d == i else 0.
    d, L, k = 5, 37, 4
    c = np.array([((7 * l) % 23) - 11 for l in range(L)], dtype=np.float64)
    W = np.zeros((L, d))
    for l in range(L):
        W[l, l % d] = c[l]
    Z = np.eye(d)[:3]
    ids, sc = orc.mine_negatives(Z, W, k)
    for i in range(3):
        known = [(c[l] if l % d == i else 0.0, l) for l in range(L)]
        known.sort(key=lambda t: (-t[0], t[1]))
        assert [int(x) for x in ids[i]] == [l for _, l in known[:k]]
        assert np.allclose(sc[i], [s for s, _ in known[:k]])


def test_mine_ties_prefer_small_id_and_negative_scores():
    L, d, k = 20, 3, 6
    W = np.tile(np.array([[1.0, -2.0, 0.5]]), (L, 1))
    Z = np.array([[1.0, 1.0, 1.0], [-1.0, -1.0, -1.0]])      # scores -0.5 and +0.5 for all l
    ids, sc = orc.mine_negatives(Z, W, k)
    assert (ids == np.arange(k)[None, :]).all()
    assert np.allclose(sc[0], -0.5) and np.allclose(sc[1], 0.5)
    # strictly negative scores: the least negative wins
    W2 = -np.arange(1, L + 1, dtype=np.float64)[:, None] * np.ones((1, d))
    ids2, _ = orc.mine_negatives(np.ones((1, d)), W2, 3)
    assert ids2[0].tolist() == [0, 1, 2]


def test_mine_equals_python_brute_force_and_chunking():
    rng = np.random.default_rng(3)
    Zq, L, d, k = 4, 53, 7, 9
    Z = rng.standard_normal((Zq, d))
    W = rng.standard_normal((L, d))
    W[11] = W[30]                                            # an exact tie
    ids_a, sc_a = orc.mine_negatives(Z, W, k, chunk=1 << 16)
    ids_b, sc_b = orc.mine_negatives(Z, W, k, chunk=7)
    assert (ids_a == ids_b).all() and np.allclose(sc_a, sc_b)
    for i in range(Zq):
        scores = []
        for l in range(L):
            s = 0.0
            for c in range(d):
                s += Z[i, c] * W[l, c]
            scores.append((s, l))
        # the duplicated row must give exactly equal scores on both paths
        scores.sort(key=lambda t: (-round(t[0], 12), t[1]))
        assert ids_a[i].tolist() == [l for _, l in scores[:k]]
    # invariants: unique ids, non-increasing scores
    for i in range(Zq):
        assert len(set(ids_a[i].tolist())) == k
        assert (np.diff(sc_a[i]) <= 0).all()


def test_mine_k_equals_L_returns_everything():
    rng = np.random.default_rng(5)
    Z = rng.standard_normal((2, 4))
    W = rng.standard_normal((6, 4))
    ids, _ = orc.mine_negatives(Z, W, 6)
    assert sorted(ids[0].tolist()) == list(range(6))


# -------------------------------------------------------------- sampling ----
def test_finaliser_matches_published_splitmix64_vectors():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "splitmix64_vectors.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 6
    for seed, n, out in rows:
        state = (int(seed) + int(n) * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
        assert orc._fmix64(state) == int(out, 0)


def test_bounded_edges_and_exact_floor():
    assert orc.bounded(0, 1000) == 0
    assert orc.bounded((1 << 64) - 1, 1000) == 999
    assert orc.bounded(1 << 63, 1000) == 500
    assert orc.bounded((1 << 63) - 1, 1000) == 499
    assert orc.bounded((1 << 64) - 1, 1) == 0
    from fractions import Fraction
    for u, m in [(0x123456789ABCDEF0, 119999950), (0xFEDCBA9876543210, 4088)]:
        assert orc.bounded(u, m) == int(Fraction(u, 1 << 64) * m)


def test_complement_select_exhaustive():
    L = 16
    for hs in ([2, 3, 9], [0, 1, 2], [13, 14, 15], [0, 15], [], [5]):
        comp = [x for x in range(L) if x not in hs]
        got = [orc.complement_select(hs, r) for r in range(L - len(hs))]
        assert got == comp
    rng = np.random.default_rng(0)
    for _ in range(50):
        L = int(rng.integers(5, 60))
        hs = sorted(rng.choice(L, size=int(rng.integers(0, L - 1)), replace=False).tolist())
        comp = [x for x in range(L) if x not in hs]
        assert [orc.complement_select(hs, r) for r in range(len(comp))] == comp


def test_sample_structure_and_logq_closed_form():
    B, k_h, k_r, L, seed = 6, 5, 40, 97, 12345
    rng = np.random.default_rng(1)
    sl = np.stack([rng.choice(L, size=k_h, replace=False) for _ in range(B)]).astype(np.int32)
    neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed)
    assert neg.shape == (B, k_h + k_r) and neg.dtype == np.int32
    assert (neg[:, :k_h] == sl).all()
    assert (logq[:, :k_h] == 0).all()
    for i in range(B):
        r = neg[i, k_h:]
        assert ((r >= 0) & (r < L)).all()
        assert not set(r.tolist()) & set(sl[i].tolist())
    import math
    assert np.allclose(logq[:, k_h:], math.log(k_r / (L - k_h)), rtol=1e-7)
    # exp(-logq) is the importance weight 1/(p k_r) with p = 1/(L-k_h)
    assert np.allclose(np.exp(-logq[:, k_h:].astype(np.float64)), (L - k_h) / k_r, rtol=1e-6)
    # deterministic, seed-sensitive, and row i does not depend on the batch size
    neg2, _ = orc.sample_negatives(sl, B, k_h, k_r, L, seed)
    assert (neg == neg2).all()
    neg3, _ = orc.sample_negatives(sl, B, k_h, k_r, L, seed + 1)
    assert (neg3[:, k_h:] != neg[:, k_h:]).mean() > 0.9
    neg4, _ = orc.sample_negatives(sl[:3], 3, k_h, k_r, L, seed)
    assert (neg4 == neg[:3]).all()
    # different queries get different streams
    assert (neg[0, k_h:] != neg[1, k_h:]).mean() > 0.9


def test_sample_uniform_on_complement_chi_square():
    from scipy.stats import chi2
    B, k_h, k_r, L = 64, 8, 512, 64
    sl = np.tile(np.array([[3, 60, 7, 8, 9, 31, 0, 63]], dtype=np.int32), (B, 1))
    neg, _ = orc.sample_negatives(sl, B, k_h, k_r, L, seed=99)
    draws = neg[:, k_h:].ravel()
    counts = np.bincount(draws, minlength=L)
    assert counts[sl[0]].sum() == 0
    allowed = np.setdiff1d(np.arange(L), sl[0])
    exp = draws.size / allowed.size
    stat = ((counts[allowed] - exp) ** 2 / exp).sum()
    assert stat < chi2.ppf(0.9999, allowed.size - 1)
    # consecutive draws are not correlated in the obvious way
    x = draws[:-1].astype(np.float64)
    y = draws[1:].astype(np.float64)
    assert abs(np.corrcoef(x, y)[0, 1]) < 0.02


def test_sample_duplicates_and_padding_in_shortlist_shrink_exclusion_set():
    # distinct in-range ids: {4, 9}; -1 and the repeat do not count.
    L, k_h, k_r = 12, 4, 300
    sl = np.array([[9, -1, 4, 9]], dtype=np.int32)
    neg, logq = orc.sample_negatives(sl, 1, k_h, k_r, L, seed=7)
    assert neg[0, :k_h].tolist() == [9, -1, 4, 9]
    r = neg[0, k_h:]
    assert set(r.tolist()) == set(range(L)) - {4, 9}
    assert np.allclose(logq[0, k_h:], np.log(k_r / (L - 2)))


def test_sample_warmup_mode_uniform_over_all_labels():
    B, k_h, k_r, L = 16, 3, 253, 32
    neg, logq = orc.sample_negatives(None, B, k_h, k_r, L, seed=5)
    assert neg.shape == (B, k_h + k_r)
    assert ((neg >= 0) & (neg < L)).all()
    assert np.allclose(logq, np.log((k_h + k_r) / L))
    counts = np.bincount(neg.ravel(), minlength=L)
    exp = neg.size / L
    from scipy.stats import chi2
    assert ((counts - exp) ** 2 / exp).sum() < chi2.ppf(0.9999, L - 1)
