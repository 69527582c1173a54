"""Pins of the oracle's mixture-proposal sampler (Sec. 3.1 Idea 2: negatives drawn from
(1-r) P_imp + r P_unif with P_imp proportional to the sigmoid of the stale score).  None of them
re-uses the sampler's own formula: the library sigmoid, exact label frequencies, the warm-up
sampler, and Monte-Carlo unbiasedness of the weighted loss against Eq. 1 through torch's BCE."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import astra_oracle as orc


def test_sigmoid_weight_tracks_the_library_sigmoid_and_is_monotone():
    xs = np.linspace(-30.0, 30.0, 6001).astype(np.float32)
    w = np.array([orc.sigmoid_weight(x) for x in xs], dtype=np.float64)
    ref = 1.0 / (1.0 + np.exp(-xs.astype(np.float64)))
    assert np.all(np.abs(w / 2.0 ** 32 - ref) <= 3e-5 + 2e-4 * ref)
    assert np.all(np.diff(w) >= 0)                      # a better score never weighs less
    assert orc.sigmoid_weight(np.float32(0.0)) == 1 << 31
    assert orc.sigmoid_weight(np.float32(-1e30)) >= 1   # never zero for a real score
    assert orc.sigmoid_weight(np.float32(1e30)) <= 1 << 32
    assert orc.sigmoid_weight(np.float32("nan")) == 0
    # clamped beyond +-30
    assert orc.sigmoid_weight(np.float32(31.0)) == orc.sigmoid_weight(np.float32(30.0))


def test_mixture_structure_and_fallback():
    L, M, k_h, k_r, B = 500, 12, 5, 9, 6
    rng = np.random.default_rng(1)
    sl = np.stack([rng.choice(L, size=M, replace=False) for _ in range(B)]).astype(np.int32)
    sc = rng.normal(size=(B, M)).astype(np.float32)
    sl[0, 3] = -1                        # padding slot
    sl[1, :] = -1                        # a row without any valid slot
    sc[2, 4] = np.float32("nan")         # a slot without a score
    neg, logq = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, seed=5)
    assert neg.shape == (B, k_h + k_r) and ((neg >= 0) & (neg < L)).all()
    for i in range(B):
        valid = {int(v) for m, v in enumerate(sl[i]) if 0 <= v < L and not np.isnan(sc[i, m])}
        if i != 1:
            assert set(neg[i, :k_h].tolist()) <= valid             # importance draws stay in the shortlist
    assert 4 not in [m for m in range(M) if sl[2, m] in neg[2, :k_h].tolist() and np.isnan(sc[2, m])]
    # no valid slot: the warm-up sampler, slot for slot
    w_neg, w_logq = orc.sample_negatives(None, B, k_h, k_r, L, seed=5)
    assert (neg[1] == w_neg[1]).all() and np.allclose(logq[1], w_logq[1], rtol=1e-7)
    # the uniform slots of every row are the warm-up sampler's draws for the same slot numbers
    assert (neg[:, k_h:] == w_neg[:, k_h:]).all()
    # determinism and independence of the batch split
    neg2, logq2 = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, seed=5, rows=[3])
    assert (neg2[3] == neg[3]).all() and (logq2[3] == logq[3]).all()


def test_importance_draws_follow_the_sigmoid_of_the_score():
    L, M, k_h, k_r = 1000, 6, 4, 2
    ids = np.array([11, 500, 7, 999, 500, 42], dtype=np.int32)        # label 500 sits in two slots
    sc = np.array([2.0, -1.0, 0.5, -3.0, 0.0, 1.0], dtype=np.float32)
    B = 6000
    sl = np.tile(ids, (B, 1))
    scs = np.tile(sc, (B, 1))
    neg, logq = orc.sample_negatives_mixture(sl, scs, B, M, k_h, k_r, L, seed=77)
    sig = 1.0 / (1.0 + np.exp(-sc.astype(np.float64)))
    want = {}
    for l, s in zip(ids.tolist(), sig):
        want[l] = want.get(l, 0.0) + s
    tot = sum(want.values())
    draws = neg[:, :k_h].ravel()
    chi2 = 0.0
    for l, p in want.items():
        e = len(draws) * p / tot
        o = float((draws == l).sum())
        chi2 += (o - e) ** 2 / e
    assert chi2 < 25.0, chi2                                       # 4 degrees of freedom: p < 1e-4
    # expected count of a label = exp(logq) of any slot that holds it: k_h p_l + k_r / L
    for l, p in want.items():
        c = float(np.exp(logq[neg == l][0]))
        assert abs(c - (k_h * p / tot + k_r / L)) < 3e-4 * c
    outside = neg[:, k_h:][~np.isin(neg[:, k_h:], ids)]
    assert np.allclose(np.exp(logq[:, k_h:][~np.isin(neg[:, k_h:], ids)]), k_r / L, rtol=1e-6) and len(outside) > 0


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


def test_mixture_weighted_bce_is_unbiased_for_eq1():
    """The loss of Eq. 2's form with every sampled pair weighted by exp(-logq) estimates Eq. 1
    without bias when logq is the log expected count under the mixture (importance sampling)."""
    B, L, d, M, k_h, k_r = 2, 24, 4, 8, 3, 6
    rng = np.random.default_rng(7)
    Z = rng.standard_normal((B, d)) * 0.9
    W = rng.standard_normal((L, d)) * 0.9
    pos = np.array([[3, -1], [5, 17]], dtype=np.int32)
    sl, sc = orc.mine_negatives(Z, W, M)
    sl = sl.copy()
    sl[1, 2] = sl[1, 0]                  # a label listed twice
    ref, dZ_ref, dW_ref = _torch_full_bce(Z, W, pos)
    n = 6000
    losses = np.empty(n)
    dWs = np.zeros((n, L, d))
    dZs = np.zeros((n, B, d))
    for t in range(n):
        neg, logq = orc.sample_negatives_mixture(sl, sc.astype(np.float32), B, M, k_h, k_r, L, seed=3000 + t)
        out = orc.xc_step(Z, W, pos, neg, logq, lr=1.0)
        losses[t] = out["loss"]
        dZs[t] = out["dZ"]
        for l, g in out["dW"].items():
            dWs[t, l] = g
    se = losses.std(ddof=1) / math.sqrt(n)
    assert abs(losses.mean() - ref) < 4.5 * se, (losses.mean(), ref, se)
    assert se < 0.03 * ref
    for arr, want in ((dZs, dZ_ref), (dWs, dW_ref)):
        mean = arr.mean(axis=0)
        sem = arr.std(axis=0, ddof=1) / math.sqrt(n)
        z = np.abs(mean - want) / np.maximum(sem, 1e-12)
        assert z.max() < 5.0, z.max()
    # power: dropping the uniform part's share from the expected count would overshoot
    assert abs(losses.mean() - ref * 1.1) > 4 * se
