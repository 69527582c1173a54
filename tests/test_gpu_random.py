"""GPU parity on randomly drawn shapes: each seed draws a step, a cold and a warm search and a sampling call
from the ranges the library accepts and compares every one with the oracle.  The hand-picked cases of the other
files aim at known boundaries; these aim at the combinations nobody thought of (a search over 128-byte rows with
a mostly empty query tile was found this way)."""
import numpy as np
import pytest
import torch

from oracle import astra_oracle as orc
from paper_2409_20156_amd import synth
from tests.parity import check_topk, f64
from tests.test_gpu_step import _run_and_check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _draw_step(rng, it):
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    d = int(rng.choice([8, 16, 40, 64, 72, 128, 256, 768]))
    if dtype == torch.float32 and d == 768:
        d = 64
    B = int(rng.integers(1, 200))
    L = int(rng.choice([2, 3, 17, 300, 5000, 40000, 700000]))
    k_p = int(rng.integers(1, 5))
    n_neg = int(rng.integers(1, 300))
    Z = synth.make_matrix(it, synth.TAG_Z, B, d, dtype, DEV)
    W = synth.make_matrix(it, synth.TAG_W, L, d, dtype, DEV)
    pos = rng.integers(0, L, size=(B, k_p)).astype(np.int32)
    for i in range(B):                               # a label is positive once per row
        _, first = np.unique(pos[i], return_index=True)
        dup = np.ones(k_p, bool)
        dup[first] = False
        pos[i, dup] = -1
    neg = rng.integers(0, L, size=(B, n_neg)).astype(np.int32)
    neg[rng.random((B, n_neg)) < rng.choice([0.0, 0.05, 0.5])] = -1
    logq = np.log(rng.uniform(0.05, 1.0, size=(B, n_neg))).astype(np.float32)
    kind = orc.LOSS_BCE if rng.random() < 0.7 else orc.LOSS_SOFTMAX
    return Z, W, pos, neg, logq, kind


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_steps(seed):
    rng = np.random.default_rng(seed)
    for it in range(6):
        Z, W, pos, neg, logq, kind = _draw_step(rng, seed * 100 + it)
        print("step", seed, it, tuple(Z.shape), W.shape[0], Z.dtype, pos.shape[1], neg.shape[1], kind, flush=True)
        _run_and_check(Z, W, pos, neg, logq, f64(Z), f64(W), 0.2, kind)


@pytest.mark.parametrize("seed", [201, 202, 203, 204])
def test_random_searches_cold_then_warm(seed):
    import paper_2409_20156_amd as xc
    rng = np.random.default_rng(seed)
    for it in range(5):
        Zq = int(rng.integers(1, 600))
        L = int(rng.choice([130, 1000, 5000, 30000, 70000]))
        k = int(rng.integers(1, min(128, L)))
        d = int(rng.choice([8, 32, 40, 64, 72, 256]))
        dt = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        Z = synth.make_matrix(seed * 100 + it, synth.TAG_Z, Zq, d, dt, DEV)
        W = synth.make_matrix(seed * 100 + it, synth.TAG_W, L, d, dt, DEV)
        code = xc.XC_BF16 if dt == torch.bfloat16 else xc.XC_F32
        ws = torch.empty(xc.mine_workspace(Zq, L, d, k, code), dtype=torch.uint8, device=DEV)
        print("search", seed, it, Zq, L, d, dt, k, flush=True)
        ids, sc = xc.mine_negatives(Z, W, k, want_scores=True, workspace=ws)
        ids_o, sc_o = orc.mine_negatives(f64(Z), f64(W), k)
        check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o, f64(Z), f64(W))
        # the rows move by a random factor, little or much, and the next search starts from the old thresholds
        scale = float(rng.choice([0.0, 0.01, 0.3]))
        W2 = (W.float() * (1.0 + scale * torch.randn(L, 1, device=DEV))).to(dt)
        margin = float(rng.choice([0.0, 0.1, 1.0]))
        ids, sc = xc.mine_negatives(Z, W2, k, want_scores=True, workspace=ws, warm_margin=margin)
        ids_o, sc_o = orc.mine_negatives(f64(Z), f64(W2), k)
        check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o, f64(Z), f64(W2))


@pytest.mark.parametrize("seed", [301, 302])
def test_random_sampling(seed):
    import paper_2409_20156_amd as xc
    rng = np.random.default_rng(seed)
    for it in range(8):
        B = int(rng.integers(1, 40))
        L = int(rng.choice([5, 200, 4096, 131072, 8_600_000, 120_000_000]))
        k_h = int(rng.integers(0, min(128, L - 1) + 1))
        k_r = int(rng.integers(0 if k_h else 1, 600))
        s = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        sl = np.stack([rng.choice(L, size=k_h, replace=False) for _ in range(B)]).astype(np.int32).reshape(B, k_h)
        sl[rng.random(sl.shape) < rng.choice([0.0, 0.2])] = -1
        print("sample", seed, it, B, L, k_h, k_r, s, flush=True)
        t = torch.tensor(sl, dtype=torch.int32, device=DEV)
        neg, logq = xc.sample_negatives(t, k_h, k_r, L, s, B=B, device=DEV)
        neg_o, logq_o = orc.sample_negatives(sl, B, k_h, k_r, L, s)
        assert (neg.cpu().numpy() == neg_o).all()
        assert np.allclose(logq.cpu().numpy(), logq_o, rtol=2e-7, atol=0)


@pytest.mark.parametrize("seed", [401, 402])
def test_random_mixture_sampling(seed):
    import paper_2409_20156_amd as xc
    rng = np.random.default_rng(seed)
    for it in range(8):
        B = int(rng.integers(1, 40))
        L = int(rng.choice([10, 200, 4096, 131072, 8_600_000, 120_000_000]))
        M = int(rng.integers(1, 1025))
        k_h = int(rng.integers(0, 300))
        k_r = int(rng.integers(0 if k_h else 1, 400))
        s = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        sl = np.stack([rng.choice(L, size=M, replace=M > L) for _ in range(B)]).astype(np.int32)
        sl[rng.random(sl.shape) < rng.choice([0.0, 0.2])] = -1
        sc = (rng.standard_normal((B, M)) * float(rng.choice([0.2, 1.0, 8.0, 40.0]))).astype(np.float32)
        print("mixture", seed, it, B, L, M, k_h, k_r, s, flush=True)
        neg, logq = xc.sample_negatives_mixture(torch.tensor(sl, device=DEV), torch.tensor(sc, device=DEV),
                                                k_h, k_r, L, s)
        neg_o, logq_o = orc.sample_negatives_mixture(sl, sc, B, M, k_h, k_r, L, s)
        assert (neg.cpu().numpy() == neg_o).all()
        assert np.allclose(logq.cpu().numpy(), logq_o, rtol=2e-7, atol=0)


@pytest.mark.parametrize("seed", [501, 502])
def test_random_sampling_without_replacement(seed):
    import paper_2409_20156_amd as xc
    rng = np.random.default_rng(seed)
    for it in range(8):
        B = int(rng.integers(1, 30))
        L = int(rng.choice([10, 200, 4096, 131072, 8_600_000, 120_000_000]))
        M = int(rng.integers(1, 1025))
        k_h = int(rng.integers(0, 300))
        k_r = int(rng.integers(0 if k_h else 1, 400))
        s = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        sl = np.stack([rng.choice(L, size=M, replace=M > L) for _ in range(B)]).astype(np.int32)
        sl[rng.random(sl.shape) < rng.choice([0.0, 0.2])] = -1
        sc = (rng.standard_normal((B, M)) * float(rng.choice([0.2, 1.0, 8.0, 40.0]))).astype(np.float32)
        print("pps", seed, it, B, L, M, k_h, k_r, s, flush=True)
        neg, logq = xc.sample_negatives_pps(torch.tensor(sl, device=DEV), torch.tensor(sc, device=DEV), k_h, k_r, L, s)
        neg_o, logq_o = orc.sample_negatives_pps(sl, sc, B, M, k_h, k_r, L, s)
        assert (neg.cpu().numpy() == neg_o).all()
        assert np.allclose(logq.cpu().numpy(), logq_o, rtol=2e-7, atol=0)
