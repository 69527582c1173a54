"""GPU parity of xc_sample_negatives: ids bit-exact with the oracle for a seed."""
import numpy as np
import pytest
import torch

from oracle import astra_oracle as orc

pytestmark = pytest.mark.gpu


def _gpu(sl, k_h, k_r, L, seed, B=None):
    import paper_2409_20156_amd as xc
    t = None if sl is None else torch.tensor(sl, dtype=torch.int32, device="cuda:0")
    neg, logq = xc.sample_negatives(t, k_h, k_r, L, seed, B=B, device="cuda:0")
    torch.cuda.synchronize()
    return neg.cpu().numpy(), logq.cpu().numpy()


def _shortlists(rng, B, k_h, L):
    return np.stack([rng.choice(L, size=k_h, replace=False) for _ in range(B)]).astype(np.int32)


@pytest.mark.parametrize("B,k_h,k_r,L,seed", [
    (32, 8, 16, 4096, 20240930),                 # Tiny
    (17, 64, 256, 131072, 1),                    # config-2 shape, ragged batch
    (5, 100, 1024, 1300000, 2 ** 63 + 12345),    # seed above 2^63
    (3, 50, 2048, 120000000, 7),                 # 120 M labels
    (4, 1, 3, 5, 9),                             # tiny label space
    (2, 1000, 50, 1001, 3),                      # almost every label excluded
    (6, 0, 40, 1000, 11),                        # no hard negatives
    (6, 33, 0, 1000, 11),                        # no random negatives
])
def test_sample_bit_exact(B, k_h, k_r, L, seed):
    print("case", B, k_h, k_r, L, seed, flush=True)
    rng = np.random.default_rng(B * 1000 + k_h)
    sl = _shortlists(rng, B, k_h, L) if k_h else np.zeros((B, 0), np.int32)
    neg, logq = _gpu(sl, k_h, k_r, L, seed)
    neg_o, logq_o = orc.sample_negatives(sl, B, k_h, k_r, L, seed)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)


def test_sample_with_padding_and_duplicates_in_the_shortlist():
    L, k_h, k_r = 50, 6, 400
    sl = np.array([[9, -1, 4, 9, 70, 0], [1, 2, 3, 4, 5, 6]], dtype=np.int32)
    neg, logq = _gpu(sl, k_h, k_r, L, 99)
    neg_o, logq_o = orc.sample_negatives(sl, 2, k_h, k_r, L, 99)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7)
    assert not set(neg[0, k_h:].tolist()) & {9, 4, 0}


def test_sample_warmup_mode():
    B, k_h, k_r, L = 9, 8, 120, 4096
    neg, logq = _gpu(None, k_h, k_r, L, 5, B=B)
    neg_o, logq_o = orc.sample_negatives(None, B, k_h, k_r, L, 5)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7)


# ------------------------------------------------- mixture proposal (importance + uniform) ----
def _gpu_mixture(sl, sc, k_h, k_r, L, seed):
    import paper_2409_20156_amd as xc
    neg, logq = xc.sample_negatives_mixture(torch.tensor(sl, dtype=torch.int32, device="cuda:0"),
                                            torch.tensor(sc, dtype=torch.float32, device="cuda:0"),
                                            k_h, k_r, L, seed)
    torch.cuda.synchronize()
    return neg.cpu().numpy(), logq.cpu().numpy()


@pytest.mark.parametrize("B,M,k_h,k_r,L,seed,scale", [
    (32, 12, 8, 16, 4096, 20240930, 1.0),        # Tiny-like
    (9, 100, 30, 200, 131072, 5, 0.2),           # scores of the size the random data gives
    (4, 1024, 64, 256, 1300000, 2 ** 63 + 1, 8.0),   # widest shortlist, saturated sigmoids
    (3, 1, 5, 0, 10, 3, 1.0),                    # one slot, no uniform part
    (5, 37, 0, 50, 120000000, 8, 1.0),           # no importance part
    (6, 16, 700, 300, 1000, 9, 40.0),            # more draws than threads, clamped scores
])
def test_mixture_sample_bit_exact(B, M, k_h, k_r, L, seed, scale):
    print("case", B, M, k_h, k_r, L, seed, flush=True)
    rng = np.random.default_rng(B * 131 + M)
    sl = np.stack([rng.choice(L, size=M, replace=M > L) for _ in range(B)]).astype(np.int32)
    sc = (rng.standard_normal((B, M)) * scale).astype(np.float32)
    neg, logq = _gpu_mixture(sl, sc, k_h, k_r, L, seed)
    neg_o, logq_o = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, seed)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)


def test_mixture_sample_degenerate_rows():
    B, M, k_h, k_r, L = 6, 20, 7, 13, 3000
    rng = np.random.default_rng(4)
    sl = np.stack([rng.choice(L, size=M, replace=False) for _ in range(B)]).astype(np.int32)
    sc = rng.standard_normal((B, M)).astype(np.float32)
    sl[0, :] = -1                                   # no valid slot: falls back to uniform draws
    sl[1, 5] = sl[1, 2]; sl[1, 9] = sl[1, 2]        # one label in three slots
    sl[2, ::2] = L + 5                              # out-of-range ids are padding
    sc[3, :] = np.float32("nan"); sc[3, 4] = 0.25   # a single usable slot
    sc[4, 0] = np.float32("inf"); sc[4, 1] = -np.float32("inf")
    sc[5, :] = -30.0                                # all weights at the floor of the clamp
    neg, logq = _gpu_mixture(sl, sc, k_h, k_r, L, 99)
    neg_o, logq_o = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, 99)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)
    assert (neg[3, :k_h] == sl[3, 4]).all()


def test_mixture_sample_sigmoid_weights_over_the_score_range():
    """Every float32 pattern class of the score goes through the same fixed-point weight on both
    sides: with two slots per row and many draws the ids agree bit for bit."""
    xs = np.concatenate([np.linspace(-31, 31, 400), [0.0, -0.0, 1e-30, -1e-30, 29.999, -29.999, 1e-8]]).astype(np.float32)
    B, L = len(xs), 50
    sl = np.tile(np.array([[3, 9]], dtype=np.int32), (B, 1))
    sc = np.stack([xs, -xs[::-1]], axis=1).astype(np.float32)
    neg, logq = _gpu_mixture(sl, sc, 64, 0, L, 1234)
    neg_o, logq_o = orc.sample_negatives_mixture(sl, sc, B, 2, 64, 0, L, 1234)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)


def test_mixture_pipeline_from_mined_scores():
    """Mine a shortlist wider than k_h with scores, sample from the mixture, take one step: the
    whole chain on the GPU against the oracle fed with the oracle's own mining."""
    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import synth
    from tests.parity import TOL, check_rows_close, f64
    dev = "cuda:0"
    B, L, d, M, k_h, k_r = 24, 3000, 64, 32, 8, 40
    W = synth.make_matrix(21, synth.TAG_W, L, d, torch.float32, dev)
    Z = synth.make_matrix(21, synth.TAG_Z, B, d, torch.float32, dev) * 4.0       # scores of order one
    pos = synth.zipf_positives(21, B, L, 1.0, "uniform:1:2", 2)
    Z64, W64 = f64(Z), f64(W)
    sl_o, sc_o = orc.mine_negatives(Z64, W64, M)
    sc_o32 = sc_o.astype(np.float32)
    sl_g, sc_g = xc.mine_negatives(Z, W, M, want_scores=True)
    assert (sl_g.cpu().numpy() == sl_o).all()
    # the stale scores enter the weights through floor(score * 2^16): feed both samplers the
    # oracle's scores rounded to float32 so that a last-bit difference in a score cannot move an id
    neg_g, logq_g = xc.sample_negatives_mixture(sl_g, torch.tensor(sc_o32, device=dev), k_h, k_r, L, 17)
    neg_o, logq_o = orc.sample_negatives_mixture(sl_o, sc_o32, B, M, k_h, k_r, L, 17)
    assert (neg_g.cpu().numpy() == neg_o).all()
    out = xc.xc_step(Z, W.clone(), torch.tensor(pos, device=dev), neg_g, logq_g, 0.3)
    ref = orc.xc_step(Z64, W64, pos, neg_o, logq_o, 0.3, storage="f32")
    assert abs(float(out["loss"].item()) - ref["loss"]) <= TOL["f32"] * abs(ref["loss"])
    check_rows_close(out["dZ"].cpu().numpy(), ref["dZ"], TOL["f32"], "dZ")


# ------------------------------------- hard negatives sampled without replacement from a wider shortlist ----
def _gpu_pps(sl, sc, k_h, k_r, L, seed):
    import paper_2409_20156_amd as xc
    neg, logq = xc.sample_negatives_pps(torch.tensor(sl, dtype=torch.int32, device="cuda:0"),
                                        torch.tensor(sc, dtype=torch.float32, device="cuda:0"),
                                        k_h, k_r, L, seed)
    torch.cuda.synchronize()
    return neg.cpu().numpy(), logq.cpu().numpy()


@pytest.mark.parametrize("B,M,k_h,k_r,L,seed,scale", [
    (32, 24, 8, 16, 4096, 20240930, 1.0),        # Tiny-like, shortlist three times as wide as k_h
    (9, 200, 50, 200, 131072, 5, 0.2),           # scores of the size the random data gives: no slot certain
    (4, 1024, 64, 256, 1300000, 2 ** 63 + 1, 8.0),   # widest shortlist, saturated sigmoids: many certain slots
    (3, 1, 5, 0, 10, 3, 1.0),                    # one slot for five places: the rest uniform
    (5, 37, 0, 50, 120000000, 8, 1.0),           # no importance part
    (6, 16, 700, 300, 1000, 9, 40.0),            # more places than slots and than threads, clamped scores
    (7, 64, 63, 5, 5000, 11, 3.0),               # all but one slot taken: rounds of certain slots
    (8, 100, 100, 0, 120000000, 12, 1.0),        # as many places as slots: all certain
])
def test_pps_sample_bit_exact(B, M, k_h, k_r, L, seed, scale):
    print("case", B, M, k_h, k_r, L, seed, flush=True)
    rng = np.random.default_rng(B * 137 + M)
    sl = np.stack([rng.choice(L, size=M, replace=M > L) for _ in range(B)]).astype(np.int32)
    sc = (rng.standard_normal((B, M)) * scale).astype(np.float32)
    neg, logq = _gpu_pps(sl, sc, k_h, k_r, L, seed)
    neg_o, logq_o = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, seed)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)
    for i in range(B):                             # without replacement: distinct shortlist slots (distinct ids here)
        k = min(k_h, M)
        if M <= L:
            assert len(set(neg[i, :k].tolist())) == k


def test_pps_sample_degenerate_rows():
    B, M, k_h, k_r, L = 6, 20, 7, 13, 3000
    rng = np.random.default_rng(4)
    sl = np.stack([rng.choice(L, size=M, replace=False) for _ in range(B)]).astype(np.int32)
    sc = rng.standard_normal((B, M)).astype(np.float32)
    sl[0, :] = -1                                   # no valid slot: uniform draws only
    sl[1, 5] = sl[1, 2]; sl[1, 9] = sl[1, 2]        # one label in three slots
    sl[2, ::2] = L + 5                              # out-of-range ids are padding
    sc[3, :] = np.float32("nan"); sc[3, 4] = 0.25   # a single usable slot
    sc[4, 0] = np.float32("inf"); sc[4, 1] = -np.float32("inf")
    sc[5, :] = -30.0                                # all weights at the floor of the clamp
    neg, logq = _gpu_pps(sl, sc, k_h, k_r, L, 99)
    neg_o, logq_o = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, 99)
    assert (neg == neg_o).all()
    assert np.allclose(logq, logq_o, rtol=2e-7, atol=0)
    assert neg[3, 0] == sl[3, 4]


def test_pps_pipeline_from_mined_scores():
    """Mine a shortlist wider than k_h with scores, sample the hard negatives from it without replacement,
    take one step: the whole chain on the GPU against the oracle fed with the oracle's own mining."""
    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import synth
    from tests.parity import TOL, check_rows_close, f64
    dev = "cuda:0"
    B, L, d, M, k_h, k_r = 24, 3000, 64, 32, 8, 40
    W = synth.make_matrix(21, synth.TAG_W, L, d, torch.float32, dev)
    Z = synth.make_matrix(21, synth.TAG_Z, B, d, torch.float32, dev) * 4.0       # scores of order one
    pos = synth.zipf_positives(21, B, L, 1.0, "uniform:1:2", 2)
    Z64, W64 = f64(Z), f64(W)
    sl_o, sc_o = orc.mine_negatives(Z64, W64, M)
    sc_o32 = sc_o.astype(np.float32)
    sl_g, sc_g = xc.mine_negatives(Z, W, M, want_scores=True)
    assert (sl_g.cpu().numpy() == sl_o).all()
    # (both samplers get the oracle's scores rounded to float32: a last-bit difference in a score cannot move an id)
    neg_g, logq_g = xc.sample_negatives_pps(sl_g, torch.tensor(sc_o32, device=dev), k_h, k_r, L, 17)
    neg_o, logq_o = orc.sample_negatives_pps(sl_o, sc_o32, B, M, k_h, k_r, L, 17)
    assert (neg_g.cpu().numpy() == neg_o).all()
    out = xc.xc_step(Z, W.clone(), torch.tensor(pos, device=dev), neg_g, logq_g, 0.3)
    ref = orc.xc_step(Z64, W64, pos, neg_o, logq_o, 0.3, storage="f32")
    assert abs(float(out["loss"].item()) - ref["loss"]) <= TOL["f32"] * abs(ref["loss"])
    check_rows_close(out["dZ"].cpu().numpy(), ref["dZ"], TOL["f32"], "dZ")
