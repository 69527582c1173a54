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
