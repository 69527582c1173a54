"""Pins of the oracle's sampler that draws the hard negatives from a wider stale shortlist WITHOUT
replacement, slot m with probability proportional to the sigmoid of its stale score (Sec. 3.1,
Observation 2 inside the mixture of Idea 2).  None re-uses the sampler's formula: exhaustive enumeration
of the random offset (exact inclusion counts), the warm-up sampler for the uniform slots, closed-form
expected counts from the library sigmoid, and Monte-Carlo unbiasedness of the weighted loss against
Eq. 1 through torch's BCE."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import astra_oracle as orc


def _word_for_offset(U, TT):
    """The smallest 64-bit word that the multiply-high draw maps to offset U of TT."""
    u = ((U << 64) + TT - 1) // TT
    assert orc.bounded(u, TT) == U
    return u


@pytest.mark.parametrize("w,k", [
    ([5, 1, 0, 9, 2, 2, 30, 3], 4),          # two slots so heavy that they are certain, one weightless
    ([3, 3, 3, 3, 3, 3], 2),                 # equal weights
    ([1, 2, 3, 4, 5, 6, 7], 3),
    ([10, 1, 1, 1], 3),                      # certainty found only in the second round: 10 first, then none
    ([8, 6, 1, 1], 3),                       # a second round of certainty: after 8, the slot with 6 is certain too
    ([4, 0, 0, 7], 2),                       # as many weighted slots as wanted: all certain
    ([2, 5], 1),
])
def test_every_offset_enumerated_gives_exact_inclusion_counts(w, k):
    """All T' equally likely offsets of the systematic step, one by one: every sample has k distinct
    weighted slots, and slot m is in exactly k' w_m of the T' samples (certain slots in all)."""
    _, pi = orc.pps_select(w, k, 0)
    assert sum(Fraction(n, d) for n, d in pi) == k                   # inclusion probabilities add up to k
    rest = [(n, d) for n, d in pi if n and (n, d) != (1, 1)]
    TT = rest[0][1] if rest else 1
    counts = [0] * len(w)
    for U in range(TT):
        taken, pi_u = orc.pps_select(w, k, _word_for_offset(U, TT))
        assert pi_u == pi                                            # they do not depend on the random word
        assert len(taken) == k and len(set(taken)) == k and taken == sorted(taken)
        assert all(w[m] > 0 for m in taken)
        for m in taken:
            counts[m] += 1
    for m in range(len(w)):
        assert Fraction(counts[m], TT) == Fraction(*pi[m])
        if w[m] == 0:
            assert counts[m] == 0
    # without certain slots the probability is k w / T; a certain slot is one whose share would exceed 1
    T = sum(w)
    for m in range(len(w)):
        if all(Fraction(k * x, T) < 1 for x in w):
            assert Fraction(*pi[m]) == Fraction(k * w[m], T)
        if Fraction(k * w[m], T) >= 1:
            assert pi[m] == (1, 1)


def test_structure_uniform_slots_and_fallback():
    L, M, k_h, k_r, B = 500, 12, 5, 9, 6
    rng = np.random.default_rng(1)
    sl = np.stack([rng.choice(L, size=M, replace=False) for _ in range(B)]).astype(np.int32)
    sc = rng.normal(size=(B, M)).astype(np.float32)
    sl[0, 3] = -1                        # padding slot
    sl[1, :] = -1                        # a row without any valid slot
    sc[2, 4] = np.float32("nan")         # a slot without a score
    sl[3, 3:] = -1                       # only three weighted slots: fewer than k_h
    neg, logq = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, seed=5)
    w_neg, w_logq = orc.sample_negatives(None, B, k_h, k_r, L, seed=5)
    assert ((neg >= 0) & (neg < L)).all()
    for i in range(B):
        valid = [int(v) for m, v in enumerate(sl[i]) if 0 <= v < L and not np.isnan(sc[i, m])]
        k = min(k_h, len(valid))
        got = neg[i, :k].tolist()
        assert len(set(got)) == k and set(got) <= set(valid)          # without replacement, from the shortlist
        assert [valid.index(g) for g in got] == sorted(valid.index(g) for g in got)     # in slot order
        assert (neg[i, k:] == w_neg[i, k:]).all()                     # the other slots: the warm-up sampler's draws
    assert set(neg[3, :3].tolist()) == set(sl[3, :3].tolist())        # all three weighted slots are taken
    assert (neg[1] == w_neg[1]).all() and np.allclose(logq[1], w_logq[1], rtol=1e-7)
    neg2, logq2 = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, seed=5, rows=[4])
    assert (neg2[4] == neg[4]).all() and (logq2[4] == logq[4]).all()


def test_expected_counts_follow_the_sigmoid_of_the_score():
    """No slot is certain here, so the expected number of copies of a shortlist label is
    k_h sigmoid(s_l) / sum of sigmoids + k_r / L, and the frequencies over many seeds agree."""
    L, M, k_h, k_r = 1000, 6, 3, 2
    ids = np.array([11, 500, 7, 999, 400, 42], dtype=np.int32)
    sc = np.array([1.0, -0.5, 0.5, -1.0, 0.0, 0.8], dtype=np.float32)
    B = 8000
    neg, logq = orc.sample_negatives_pps(np.tile(ids, (B, 1)), np.tile(sc, (B, 1)), B, M, k_h, k_r, L, seed=99)
    sig = 1.0 / (1.0 + np.exp(-sc.astype(np.float64)))
    pi = k_h * sig / sig.sum()
    assert pi.max() < 1.0
    hard = neg[:, :k_h]
    assert all(len(set(r.tolist())) == k_h for r in hard[:200])
    for l, p in zip(ids.tolist(), pi):
        freq = float((hard == l).any(axis=1).mean())
        assert abs(freq - p) < 4.5 * math.sqrt(p * (1 - p) / B) + 3e-4, (l, freq, p)
        c = float(np.exp(logq[neg == l][0]))
        assert abs(c - (p + k_r / L)) < 3e-4 * c
    rest = ~np.isin(neg[:, k_h:], ids)
    assert np.allclose(np.exp(logq[:, k_h:][rest]), k_r / L, rtol=1e-6) and rest.sum() > 0


def _torch_full_bce(Z, W, pos):
    Zt = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Y = torch.zeros((Z.shape[0], W.shape[0]), dtype=torch.float64)
    for i, row in enumerate(pos):
        for l in row:
            if l >= 0:
                Y[i, int(l)] = 1.0
    loss = F.binary_cross_entropy_with_logits(Zt @ Wt.T, Y, reduction="sum") / Z.shape[0]
    loss.backward()
    return loss.item(), Zt.grad.numpy(), Wt.grad.numpy()


def test_weighted_bce_is_unbiased_for_eq1_and_beats_sampling_with_replacement():
    """Pairs weighted by exp(-logq) estimate Eq. 1 without bias (loss and both gradients); and drawing the
    hard negatives without replacement gives a smaller variance than the same number of draws with it."""
    B, L, d, M, k_h, k_r = 2, 24, 4, 8, 3, 6
    rng = np.random.default_rng(7)
    Z = rng.standard_normal((B, d)) * 0.9
    W = rng.standard_normal((L, d)) * 0.9
    pos = np.array([[3, -1], [5, 17]], dtype=np.int32)
    sl, sc = orc.mine_negatives(Z, W, M)
    sl = sl.copy()
    sl[1, 2] = sl[1, 0]                  # a label listed twice
    sc = (sc - sc.mean() - 2.0).astype(np.float32)
    sc[0, 0] += 8.0                      # one slot of query 0 so far ahead that it is certain to be taken
    w0 = [orc.sigmoid_weight(x) for x in sc[0]]
    assert any(k_h * x >= sum(w0) for x in w0)
    ref, dZ_ref, dW_ref = _torch_full_bce(Z, W, pos)
    n = 6000
    losses, losses_wr = np.empty(n), np.empty(n)
    dWs = np.zeros((n, L, d))
    dZs = np.zeros((n, B, d))
    for t in range(n):
        neg, logq = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, seed=3000 + t)
        out = orc.xc_step(Z, W, pos, neg, logq, lr=1.0)
        losses[t] = out["loss"]
        dZs[t] = out["dZ"]
        for l, g in out["dW"].items():
            dWs[t, l] = g
        neg, logq = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, seed=3000 + t)
        losses_wr[t] = orc.xc_step(Z, W, pos, neg, logq, lr=1.0)["loss"]
    se = losses.std(ddof=1) / math.sqrt(n)
    assert abs(losses.mean() - ref) < 4.5 * se, (losses.mean(), ref, se)
    assert se < 0.03 * ref
    for arr, want in ((dZs, dZ_ref), (dWs, dW_ref)):
        mean = arr.mean(axis=0)
        sem = arr.std(axis=0, ddof=1) / math.sqrt(n)
        z = np.abs(mean - want) / np.maximum(sem, 1e-12)
        assert z.max() < 5.0, z.max()
    assert abs(losses.mean() - ref * 1.1) > 4 * se                    # power: a 10 % bias would be seen
    assert losses.std() < losses_wr.std()


def test_planted_mistakes_are_caught():
    """Each of these changes to the selection breaks the exact inclusion counts."""
    w, k = [5, 1, 0, 9, 2, 2, 30, 3], 4

    def counts(select):
        _, pi = orc.pps_select(w, k, 0)
        TT = [d for n, d in pi if n and (n, d) != (1, 1)][0]
        c = [0] * len(w)
        for U in range(TT):
            for m in select(U, TT):
                c[m] += 1
        return c, TT, pi

    def no_certainty(U, TT0):                 # systematic sampling over all slots: heavy slots taken twice or skipped
        T = sum(w)
        taken, c = [], 0
        for m, x in enumerate(w):
            lo, hi = k * c, k * (c + x)
            c += x
            if any(lo <= (U % T) + j * T < hi for j in range(k)):
                taken.append(m)
        return taken
    c, TT, pi = counts(no_certainty)
    assert any(Fraction(c[m], TT) != Fraction(*pi[m]) for m in range(len(w)))

    def one_point_only(U, TT0):               # the first of the k' points only: one slot taken besides the certain ones
        _, pi0 = orc.pps_select(w, k, 0)
        taken, c = [m for m, p in enumerate(pi0) if p == (1, 1)], 0
        for m, x in enumerate(w):
            if pi0[m] == (1, 1) or x == 0:
                continue
            if c <= U < c + x:
                taken.append(m)
            c += x
        return taken
    c2, _, _ = counts(one_point_only)
    assert any(Fraction(c2[m], TT) != Fraction(*pi[m]) for m in range(len(w)))
