"""GPU parity of the outer loop of Alg. 1 (warm-up, periodic refresh, synchronous or
running beside the steps with a fixed lag, hard + random steps):
the library driven by paper_2409_20156_amd.schedule against the oracle's train_schedule, each on
its own copy of the same generated inputs (no state is copied between the two)."""
import numpy as np
import pytest
import torch

from oracle import astra_oracle as orc
from paper_2409_20156_amd import synth
from tests.parity import TOL, check_rows_close, check_topk, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("kind,lag,warm", [(orc.LOSS_BCE, 0, None), (orc.LOSS_SOFTMAX, 0, None), (orc.LOSS_BCE, 2, None),
                                           (orc.LOSS_BCE, 1, None), (orc.LOSS_BCE, 0, 0.1), (orc.LOSS_BCE, 2, 0.0)])
def test_schedule_matches_oracle(kind, lag, warm):
    from paper_2409_20156_amd.schedule import Schedule
    L, d, B, pool, k_p, k_h, k_r = 4096, 64, 32, 64, 2, 8, 16
    steps, tau_s, tau_r, lr = 7, 1, 2, 0.3
    W = synth.make_matrix(11, synth.TAG_W, L, d, torch.float32, DEV)
    Z = synth.make_matrix(11, synth.TAG_Z, pool, d, torch.float32, DEV)
    pos = synth.zipf_positives(11, pool, L, 1.0, "uniform:1:2", k_p)
    Z = synth.add_positive_signal(Z, W, pos)
    seeds = [synth.step_seed(synth.BASE_SEED, 9, t) for t in range(steps)]
    W64, Z64 = f64(W), f64(Z)
    ref = orc.train_schedule(Z64, W64, pos, B, k_h, k_r, steps, tau_s, tau_r, lr, seeds, kind=kind, storage="f32",
                             lag=lag)

    # warm: refreshes after the first start from the last thresholds (same shortlists, by either route)
    sch = Schedule(Z, W, torch.tensor(pos, device=DEV), B, k_h, k_r, tau_s, tau_r, lr, kind=kind, lag=lag,
                   warm_margin=warm)
    tol = 20 * TOL["f32"]                  # rounding differences compound over the steps
    n_ref, overlaps = 0, []
    for t in range(steps):
        out = sch.step(seeds[t])
        torch.cuda.synchronize()
        loss = float(out["loss"].item())
        assert abs(loss - ref["loss"][t]) <= tol * abs(ref["loss"][t]), (t, loss, ref["loss"][t])
        if sch.refreshed:
            t_ref, sl_ref = ref["shortlists"][n_ref]
            assert t_ref == t
            got = sch.shortlist[sch.built].cpu().numpy()
            assert (np.sort(got, axis=1) == np.sort(sl_ref, axis=1)).all(), "refresh at step %d" % t
            pair = sch.previous_and_fresh()
            if pair is not None:
                stale, fresh = (x.cpu().numpy() for x in pair)
                overlaps.append(np.mean([len(set(fresh[q]) & set(stale[q])) for q in range(pool)]) / k_h)
            n_ref += 1
    assert n_ref == len(ref["shortlists"]) == 3
    assert np.allclose(overlaps, ref["overlap"], atol=1e-12)
    assert 0.0 < min(overlaps) and max(overlaps) < 1.0      # the refresh did change the lists
    check_rows_close(f64(W), W64, tol, "W after the schedule")


@pytest.mark.parametrize("lag,warm,cut", [(0, None, 3), (2, None, 4), (0, 0.1, 4), (2, 0.0, 2)])
def test_schedule_resumes_from_a_saved_state_bit_for_bit(lag, warm, cut):
    """Stop after `cut` steps (with lag 2 and refreshes at 1, 3, 5 a search is then waiting to take over), save,
    build a new schedule on other tensors, load, go on: losses and the final W equal the uninterrupted run's bits."""
    from paper_2409_20156_amd.schedule import Schedule
    L, d, B, pool, k_p, k_h, k_r = 4096, 64, 32, 64, 2, 8, 16
    steps, tau_s, tau_r, lr = 8, 1, 2, 0.3
    W0 = synth.make_matrix(12, synth.TAG_W, L, d, torch.float32, DEV)
    Z = synth.make_matrix(12, synth.TAG_Z, pool, d, torch.float32, DEV)
    pos = synth.zipf_positives(12, pool, L, 1.0, "uniform:1:2", k_p)
    Z = synth.add_positive_signal(Z, W0, pos)
    pos_t = torch.tensor(pos, device=DEV)
    seeds = [synth.step_seed(synth.BASE_SEED, 10, t) for t in range(steps)]

    def run(sch, ts):
        losses = []
        for t in ts:
            losses.append(sch.step(seeds[t])["loss"].clone())
        torch.cuda.synchronize()
        return [float(x.item()) for x in losses]

    Wa = W0.clone()
    a = Schedule(Z, Wa, pos_t, B, k_h, k_r, tau_s, tau_r, lr, lag=lag, warm_margin=warm)
    loss_a = run(a, range(steps))

    Wb = W0.clone()
    b = Schedule(Z, Wb, pos_t, B, k_h, k_r, tau_s, tau_r, lr, lag=lag, warm_margin=warm)
    loss_b = run(b, range(cut))
    sd = b.state_dict()
    if lag == 2 and cut in (2, 4):
        assert sd["pending"] is not None               # saved between the start of a search and its takeover
    del b
    Wc = torch.zeros_like(W0)                           # whatever it holds: the saved W replaces it
    c = Schedule(Z, Wc, pos_t, B, k_h, k_r, tau_s, tau_r, lr, lag=lag, warm_margin=warm)
    c.load_state_dict(sd)
    assert c.t == cut
    loss_c = run(c, range(cut, steps))
    assert loss_b + loss_c == loss_a
    assert torch.equal(Wc, Wa)
