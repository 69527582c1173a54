"""Pins for the oracle's training step (CPU only).

The sampled loss of Eq. 2 is checked against Eq. 1 evaluated over all labels by
a library BCE (PyTorch CPU, float64), in the full-coverage special case and in
expectation (Lemma 1, part 1); gradients against finite differences and
against autograd; the update against the sparsity of the gradient of W.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import astra_oracle as orc


def _problem(seed=0, B=3, L=40, d=6, k_p=2, scale=0.7):
    rng = np.random.default_rng(seed)
    Z = rng.standard_normal((B, d)) * scale
    W = rng.standard_normal((L, d)) * scale
    pos = np.full((B, k_p), -1, dtype=np.int32)
    for i in range(B):
        n = int(rng.integers(1, k_p + 1))
        pos[i, :n] = rng.choice(L, size=n, replace=False)
    return Z, W, pos


def _torch_full_bce(Z, W, pos):
    """Eq. 1 through torch's BCE-with-logits over the dense multi-hot target."""
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


# ----------------------------------------------------------- full coverage --
def test_full_bce_equals_library_bce():
    Z, W, pos = _problem(1)
    ref, _, _ = _torch_full_bce(Z, W, pos)
    assert math.isclose(orc.full_bce_loss(Z, W, pos), ref, rel_tol=1e-12)


def test_bce_with_every_label_as_negative_is_eq1():
    Z, W, pos = _problem(2)
    B, L = Z.shape[0], W.shape[0]
    neg = np.tile(np.arange(L, dtype=np.int32), (B, 1))       # positives among them: masked
    logq = np.zeros((B, L), dtype=np.float32)
    out = orc.xc_step(Z, W, pos, neg, logq, lr=0.1)
    ref, dZ_ref, dW_ref = _torch_full_bce(Z, W, pos)
    assert math.isclose(out["loss"], ref, rel_tol=1e-12)
    assert np.allclose(out["dZ"], dZ_ref, rtol=1e-10, atol=1e-13)
    assert out["touched"].tolist() == list(range(L))
    assert np.allclose(out["W_rows"], W - 0.1 * dW_ref, rtol=1e-10, atol=1e-13)


def test_softmax_with_every_label_is_plain_cross_entropy():
    Z, W, pos = _problem(3, k_p=1)
    B, L = Z.shape[0], W.shape[0]
    neg = np.tile(np.arange(L, dtype=np.int32), (B, 1))
    logq = np.zeros((B, L), dtype=np.float32)
    out = orc.xc_step(Z, W, pos, neg, logq, lr=0.2, kind=orc.LOSS_SOFTMAX)
    Zt = torch.tensor(Z, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    tgt = torch.tensor(pos[:, 0].astype(np.int64))
    loss = F.cross_entropy(Zt @ Wt.T, tgt, reduction="mean")
    loss.backward()
    assert math.isclose(out["loss"], loss.item(), rel_tol=1e-12)
    assert math.isclose(orc.full_softmax_loss(Z, W, pos), loss.item(), rel_tol=1e-12)
    assert np.allclose(out["dZ"], Zt.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(out["W_rows"], W - 0.2 * Wt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_softmax_multi_positive_full_coverage():
    Z, W, pos = _problem(4, k_p=3)
    B, L = Z.shape[0], W.shape[0]
    neg = np.tile(np.arange(L, dtype=np.int32), (B, 1))
    out = orc.xc_step(Z, W, pos, neg, np.zeros((B, L), np.float32), 0.0, kind=orc.LOSS_SOFTMAX)
    logp = F.log_softmax(torch.tensor(Z) @ torch.tensor(W).T, dim=1).numpy()
    ref = np.mean([-np.mean([logp[i, l] for l in pos[i] if l >= 0]) for i in range(B)])
    assert math.isclose(out["loss"], ref, rel_tol=1e-12)
    assert math.isclose(orc.full_softmax_loss(Z, W, pos), ref, rel_tol=1e-12)


# -------------------------------------------------------------- closed form --
def test_zero_classifier_closed_forms():
    B, L, d, k_h, k_r = 4, 50, 5, 3, 7
    rng = np.random.default_rng(0)
    Z = rng.standard_normal((B, d))
    W = np.zeros((L, d))
    pos = np.array([[1, -1], [2, 3], [4, -1], [5, 6]], dtype=np.int32)
    sl = np.array([[10, 11, 12], [13, 14, 2], [16, 17, 18], [19, 20, 21]], dtype=np.int32)  # query 1: a positive mined
    neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=3)
    neg[2, k_h] = 4            # force a positive among the random draws of query 2
    out = orc.xc_step(Z, W, pos, neg, logq, lr=1.0)
    a = (L - k_h) / k_r
    kp = [1, 2, 1, 2]
    kh_eff = [3, 2, 3, 3]
    kr_eff = [sum(1 for l in neg[i, k_h:] if l not in pos[i]) for i in range(B)]
    assert kr_eff[2] <= k_r - 1
    want = sum((kp[i] + kh_eff[i] + a * kr_eff[i]) * math.log(2.0) for i in range(B)) / B
    assert math.isclose(out["loss"], want, rel_tol=1e-6)    # logq is float32
    assert np.allclose(out["dZ"], 0.0)
    # every coefficient is +-1/2 (times weight) / B; row update = -lr * sum coef * z_i
    dense = np.zeros((L, d))
    for i in range(B):
        for l in pos[i]:
            if l >= 0:
                dense[l] += -0.5 / B * Z[i]
        for j, l in enumerate(neg[i]):
            if l in pos[i]:
                continue
            dense[l] += (1.0 if j < k_h else a) * 0.5 / B * Z[i]
    got = np.zeros((L, d))
    got[out["touched"]] = out["W_rows"]
    assert np.allclose(got, -dense, rtol=1e-6, atol=1e-12)
    # soft-max: loss_i = log(k_p + sum of weights)
    out2 = orc.xc_step(Z, W, pos, neg, logq, lr=1.0, kind=orc.LOSS_SOFTMAX)
    want2 = sum(math.log(kp[i] + kh_eff[i] + a * kr_eff[i]) for i in range(B)) / B
    assert math.isclose(out2["loss"], want2, rel_tol=1e-6)
    assert np.allclose(out2["dZ"], 0.0)


# --------------------------------------------------- Lemma 1(1): unbiased ----
def test_sampled_bce_is_unbiased_for_eq1():
    B, L, d, k_h, k_r = 2, 24, 4, 3, 6
    Z, W, pos = _problem(7, B=B, L=L, d=d, k_p=2, scale=0.9)
    sl, _ = orc.mine_negatives(Z, W, k_h)
    ref, dZ_ref, dW_ref = _torch_full_bce(Z, W, pos)
    n = 6000
    losses = np.empty(n)
    dZs = np.zeros((n, B, d))
    dWs = np.zeros((n, L, d))
    for t in range(n):
        neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=1000 + t)
        out = orc.xc_step(Z, W, pos, neg, logq, lr=1.0)
        losses[t] = out["loss"]
        dZs[t] = out["dZ"]
        for l, g in out["dW"].items():
            dWs[t, l] = g
    se = losses.std(ddof=1) / math.sqrt(n)
    assert abs(losses.mean() - ref) < 4.5 * se, (losses.mean(), ref, se)
    assert se < 0.02 * ref                      # the test has power: a wrong weight shifts the mean
    for arr, want in ((dZs, dZ_ref), (dWs, dW_ref)):
        mean = arr.mean(axis=0)
        sem = arr.std(axis=0, ddof=1) / math.sqrt(n)
        z = np.abs(mean - want) / np.maximum(sem, 1e-12)
        assert z.max() < 5.0, z.max()
    # a plausible mistake: weight k_r/(L-k_h) inverted or p = 1/L would be off by far more
    wrong = ref * (L / (L - k_h))
    assert abs(losses.mean() - wrong) > 6 * se or k_h == 0


def test_sampled_softmax_partition_function_is_unbiased():
    B, L, d, k_h, k_r = 1, 30, 4, 4, 8
    Z, W, pos = _problem(8, B=B, L=L, d=d, k_p=1, scale=0.8)
    sl, _ = orc.mine_negatives(Z, W, k_h)
    s = W @ Z[0]
    mask = np.ones(L, bool)
    mask[pos[0, 0]] = False
    exact = np.exp(s).sum()                     # positive + all negatives
    n = 6000
    est = np.empty(n)
    for t in range(n):
        neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=50 + t)
        out = orc.xc_step(Z, W, pos, neg, logq, lr=0.0, kind=orc.LOSS_SOFTMAX)
        # loss = -(s_pos - lse)  =>  partition estimate = exp(loss + s_pos)
        est[t] = math.exp(out["loss"] + s[pos[0, 0]])
    se = est.std(ddof=1) / math.sqrt(n)
    assert abs(est.mean() - exact) < 4.5 * se


# -------------------------------------------------------------- gradients ----
def _loss_only(Z, W, pos, neg, logq, kind):
    return orc.xc_step(Z, W, pos, neg, logq, lr=0.0, kind=kind)["loss"]


@pytest.mark.parametrize("kind", [orc.LOSS_BCE, orc.LOSS_SOFTMAX])
def test_finite_differences(kind):
    B, L, d, k_h, k_r = 3, 30, 5, 3, 6
    Z, W, pos = _problem(11, B=B, L=L, d=d, k_p=2)
    pos[0] = [4, 17]                            # one query with two positives
    pos[1] = [9, -1]
    sl, _ = orc.mine_negatives(Z, W, k_h)
    neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=5)
    neg[0, k_h + 1] = neg[0, k_h]               # a duplicate draw counts twice
    out = orc.xc_step(Z, W, pos, neg, logq, lr=1.0, kind=kind)
    h = 1e-6
    for i in range(B):
        for c in range(d):
            Zp, Zm = Z.copy(), Z.copy()
            Zp[i, c] += h
            Zm[i, c] -= h
            fd = (_loss_only(Zp, W, pos, neg, logq, kind) - _loss_only(Zm, W, pos, neg, logq, kind)) / (2 * h)
            assert math.isclose(out["dZ"][i, c], fd, rel_tol=2e-6, abs_tol=1e-8)
    new = W.copy()
    new[out["touched"]] = out["W_rows"]
    dW = W - new                                # lr = 1
    for l in range(L):
        for c in range(d):
            Wp, Wm = W.copy(), W.copy()
            Wp[l, c] += h
            Wm[l, c] -= h
            fd = (_loss_only(Z, Wp, pos, neg, logq, kind) - _loss_only(Z, Wm, pos, neg, logq, kind)) / (2 * h)
            assert math.isclose(dW[l, c], fd, rel_tol=2e-6, abs_tol=1e-8)


def test_autograd_second_opinion_bce():
    B, L, d, k_h, k_r = 4, 60, 8, 5, 9
    Z, W, pos = _problem(12, B=B, L=L, d=d, k_p=3)
    sl, _ = orc.mine_negatives(Z, W, k_h)
    neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=8)
    out = orc.xc_step(Z, W, pos, neg, logq, lr=0.3)
    Zt = torch.tensor(Z, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    total = 0.0
    for i in range(B):
        p = [int(l) for l in pos[i] if l >= 0]
        keep = [j for j in range(neg.shape[1]) if int(neg[i, j]) not in p]
        ids = torch.tensor(p + [int(neg[i, j]) for j in keep])
        y = torch.tensor([1.0] * len(p) + [0.0] * len(keep), dtype=torch.float64)
        w = torch.tensor([1.0] * len(p) + [math.exp(-float(logq[i, j])) for j in keep], dtype=torch.float64)
        logits = Wt[ids] @ Zt[i]
        total = total + F.binary_cross_entropy_with_logits(logits, y, weight=w, reduction="sum")
    total = total / B
    total.backward()
    assert math.isclose(out["loss"], total.item(), rel_tol=1e-12)
    assert np.allclose(out["dZ"], Zt.grad.numpy(), rtol=1e-10, atol=1e-14)
    new = W.copy()
    new[out["touched"]] = out["W_rows"]
    assert np.allclose(new, W - 0.3 * Wt.grad.numpy(), rtol=1e-10, atol=1e-14)


# ------------------------------------------------------ masking / sparsity ----
def test_positive_among_negatives_is_the_same_as_removing_the_slot():
    Z, W, pos = _problem(13, B=2, L=30, d=4, k_p=2)
    pos[0] = [3, 7]
    neg = np.array([[1, 3, 9, 9, -1], [2, 4, 6, 8, 10]], dtype=np.int32)
    logq = np.array([[0, 0, -1.0, -1.0, -1.0], [0, 0, -1, -1, -1]], dtype=np.float32)
    negr = np.array([[1, -1, 9, 9, -1], [2, 4, 6, 8, 10]], dtype=np.int32)
    pos[1] = [20, -1]
    for kind in (orc.LOSS_BCE, orc.LOSS_SOFTMAX):
        a = orc.xc_step(Z, W, pos, neg, logq, 0.1, kind=kind)
        b = orc.xc_step(Z, W, pos, negr, logq, 0.1, kind=kind)
        assert a["loss"] == b["loss"]
        assert (a["dZ"] == b["dZ"]).all() and (a["touched"] == b["touched"]).all()
        assert (a["W_rows"] == b["W_rows"]).all()
        assert a["touched"].tolist() == sorted({3, 7, 1, 9, 20, 2, 4, 6, 8, 10})


def test_out_of_range_ids_are_padding():
    Z, W, pos = _problem(14, B=1, L=10, d=3, k_p=3)
    pos[0] = [2, 10, -5]
    neg = np.array([[4, 10, 99, -1]], dtype=np.int32)
    logq = np.zeros((1, 4), np.float32)
    a = orc.xc_step(Z, W, pos, neg, logq, 0.1)
    assert a["touched"].tolist() == [2, 4]


def test_shared_positive_accumulates_over_the_batch_and_rest_untouched():
    B, L, d = 5, 20, 3
    rng = np.random.default_rng(1)
    Z = rng.standard_normal((B, d))
    W = rng.standard_normal((L, d))
    pos = np.full((B, 1), 6, dtype=np.int32)
    neg = np.full((B, 1), -1, dtype=np.int32)
    out = orc.xc_step(Z, W, pos, neg, np.zeros((B, 1), np.float32), lr=0.5)
    assert out["touched"].tolist() == [6]
    s = Z @ W[6]
    g = (1.0 / (1.0 + np.exp(-s)) - 1.0) / B
    assert np.allclose(out["W_rows"][0], W[6] - 0.5 * (g[:, None] * Z).sum(0), rtol=1e-12)
    assert math.isclose(out["loss"], np.log1p(np.exp(-s)).mean(), rel_tol=1e-12)


def test_sparse_update_equals_dense_scatter():
    B, L, d, k_h, k_r = 6, 25, 4, 3, 10
    Z, W, pos = _problem(15, B=B, L=L, d=d, k_p=2)
    sl, _ = orc.mine_negatives(Z, W, k_h)
    neg, logq = orc.sample_negatives(sl, B, k_h, k_r, L, seed=2)
    out = orc.xc_step(Z, W, pos, neg, logq, lr=0.25)
    dense = np.zeros((L, d))
    for i in range(B):
        for l, g in out["coef"][i]:
            dense[l] += g * Z[i]
    new = W.copy()
    new[out["touched"]] = out["W_rows"]
    assert np.allclose(new, W - 0.25 * dense, rtol=1e-12, atol=1e-15)
    untouched = np.setdiff1d(np.arange(L), out["touched"])
    assert (new[untouched] == W[untouched]).all()
    assert (np.abs(dense[untouched]) == 0).all()
    # dZ from the same coefficients
    for i in range(B):
        want = sum(g * W[l] for l, g in out["coef"][i])
        assert np.allclose(out["dZ"][i], want, rtol=1e-12)


# ------------------------------------------------------------- rounding ------
def test_round_to_bf16_matches_library_and_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40]])
    x32 = x.astype(np.float32)                   # float32-exact inputs: torch rounds these RNE
    want = torch.tensor(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(x32.astype(np.float64))
    ok = np.isfinite(want)
    assert (got[ok] == want[ok]).all()
    # 1 + 2^-8 is exactly half-way between 1 and 1+2^-7: tie goes to even (1.0);
    # 1 + 3*2^-8 is half-way between 1+2^-7 and 1+2^-6: tie goes to 1+2^-6
    assert orc.round_to_bf16(np.array([1.00390625]))[0] == 1.0
    assert orc.round_to_bf16(np.array([1.01171875]))[0] == 1.015625
    # a float64 just above the tie must round up even though float32 would first hit the tie
    assert orc.round_to_bf16(np.array([1.00390625 + 1e-12]))[0] == 1.0078125


def test_storage_rounding_of_updated_rows():
    Z, W, pos = _problem(16, B=2, L=12, d=4, k_p=1)
    Wb = orc.round_to_bf16(W)
    Zb = orc.round_to_bf16(Z)
    neg = np.array([[0, 1, 2], [3, 4, 5]], dtype=np.int32)
    logq = np.zeros((2, 3), np.float32)
    a = orc.xc_step(Zb, Wb, pos, neg, logq, 0.1, storage="f64")
    b = orc.xc_step(Zb, Wb, pos, neg, logq, 0.1, storage="bf16")
    assert (b["W_rows"] == orc.round_to_bf16(a["W_rows"])).all()
    assert np.abs(b["W_rows"] - a["W_rows"]).max() <= np.abs(a["W_rows"]).max() * 2.0 ** -8


# ---------------------------------------------------------------------------
# outer loop of Alg. 1 (warm-up, refresh every tau_r steps, stale hard negatives)
# ---------------------------------------------------------------------------
def _schedule_inputs(seed=3, L=200, d=8, pool=12):
    rng = np.random.default_rng(seed)
    # float32-representable, as the stored matrices are
    W = (rng.normal(size=(L, d)) / np.sqrt(d)).astype(np.float32).astype(np.float64)
    Z = (rng.normal(size=(pool, d)) / np.sqrt(d)).astype(np.float32).astype(np.float64)
    pos = rng.integers(0, L, size=(pool, 1)).astype(np.int32)
    return W, Z, pos


def test_schedule_refresh_times_and_stale_hard_negatives():
    W, Z, pos = _schedule_inputs()
    B, k_h, k_r, steps, tau_s, tau_r = 4, 3, 5, 9, 2, 3
    out = orc.train_schedule(Z, W.copy(), pos, B, k_h, k_r, steps, tau_s, tau_r, 0.5, list(range(100, 100 + steps)))
    assert [t for t, _ in out["shortlists"]] == [2, 5, 8]          # t = tau_s + m * tau_r
    assert len(out["overlap"]) == 2 and len(out["loss"]) == steps
    nbatch = Z.shape[0] // B
    for t in range(steps):
        neg = out["neg"][t]
        lo = (t % nbatch) * B
        if t < tau_s:
            # warm-up: no hard slots; the first k_h ids are uniform draws, not a shortlist row
            assert neg.shape == (B, k_h + k_r)
        else:
            last = [sl for tt, sl in out["shortlists"] if tt <= t][-1]   # the newest refresh not after t
            assert (neg[:, :k_h] == last[lo:lo + B]).all()                # hard negatives are that (stale) list
            for i in range(B):
                assert not set(neg[i, k_h:].tolist()) & set(last[lo + i].tolist())
    # the first refresh is the exact search on the matrix as it stood after the warm-up steps:
    # replay those steps by hand with the warm-up sampler
    W2 = W.copy()
    for t in range(tau_s):
        lo = (t % nbatch) * B
        neg, logq = orc.sample_negatives(None, B, k_h, k_r, W.shape[0], 100 + t)
        assert (neg == out["neg"][t]).all()
        r = orc.xc_step(Z[lo:lo + B], W2, pos[lo:lo + B], neg, logq, 0.5)
        W2[r["touched"]] = r["W_rows"]
    brute = np.argsort(-(Z @ W2.T), axis=1, kind="stable")[:, :k_h]
    assert (np.sort(brute, axis=1) == np.sort(out["shortlists"][0][1], axis=1)).all()


def test_schedule_with_zero_learning_rate_is_stationary():
    W, Z, pos = _schedule_inputs(seed=5)
    B, k_h, k_r, steps = 4, 3, 5, 10
    nbatch = Z.shape[0] // B                      # 3 batches
    seeds = [7 + (t % nbatch) for t in range(steps)]         # same seed whenever the same batch returns
    W0 = W.copy()
    out = orc.train_schedule(Z, W, pos, B, k_h, k_r, steps, 0, 2, 0.0, seeds)
    assert (W == W0).all()
    assert out["overlap"] == [1.0] * (len(out["shortlists"]) - 1)       # nothing moved between refreshes
    for t in range(nbatch, steps):
        assert out["loss"][t] == out["loss"][t - nbatch]                # batches cycle through the pool
    assert len(set(round(x, 12) for x in out["loss"][:nbatch])) == nbatch   # ... and differ from each other


def test_schedule_lag_delays_the_takeover_of_a_refresh():
    W, Z, pos = _schedule_inputs(seed=9)
    B, k_h, k_r, steps, tau_s, tau_r, lag = 4, 3, 5, 9, 1, 3, 2
    seeds = list(range(50, 50 + steps))
    out = orc.train_schedule(Z, W.copy(), pos, B, k_h, k_r, steps, tau_s, tau_r, 0.5, seeds, lag=lag)
    built = dict(out["shortlists"])                      # searched at steps 1, 4, 7
    assert sorted(built) == [1, 4, 7]
    nbatch = Z.shape[0] // B
    for t in range(steps):
        lo = (t % nbatch) * B
        active = [tt for tt in built if tt + lag <= t]   # a search started at tt serves from tt + lag on
        neg = out["neg"][t]
        if not active:
            # still warm-up negatives: identical to the sampler's warm-up mode for this seed
            want, _ = orc.sample_negatives(None, B, k_h, k_r, W.shape[0], seeds[t])
            assert (neg == want).all()
        else:
            assert (neg[:, :k_h] == built[max(active)][lo:lo + B]).all()
    # the search itself used the matrix of its own step, not of the takeover step: with lag = 0
    # the same schedule builds the same first shortlist at step 1
    out0 = orc.train_schedule(Z, W.copy(), pos, B, k_h, k_r, 2, tau_s, tau_r, 0.5, seeds, lag=0)
    assert (out0["shortlists"][0][1] == built[1]).all()
