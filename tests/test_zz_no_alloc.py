"""xc_step_static, the entry point that allocates nothing, against xc_step: same bits, on two calls
in a row of which the second has the smaller input (the static scratch array then still holds the
first call's temporaries)."""
import numpy as np
import pytest
import torch

from paper_2409_20156_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, B, L, d, dtype, k_p, n_neg):
    rng = np.random.default_rng(seed)
    W = synth.make_matrix(seed, synth.TAG_W, L, d, dtype, DEV)
    Z = synth.make_matrix(seed, synth.TAG_Z, B, d, dtype, DEV)
    pos = synth.zipf_positives(seed, B, L, 1.0, "uniform:1:%d" % k_p if k_p > 1 else "one", k_p)
    neg = rng.integers(0, L, size=(B, n_neg)).astype(np.int32)
    neg[:, :8] = (rng.zipf(1.5, size=(B, 8)) * 131) % L            # shared ids: segments of several pairs
    neg[0, 1] = -1
    neg[1, 2] = pos[1, 0]
    logq = np.log(rng.uniform(0.05, 1.0, size=(B, n_neg))).astype(np.float32)
    return Z, W, torch.tensor(pos, device=DEV), torch.tensor(neg, device=DEV), torch.tensor(logq, device=DEV)


def _outputs(B, d, n, dtype):
    return {"loss": torch.full((1,), -7.0, dtype=torch.float32, device=DEV),
            "dZ": torch.full((B, d), -7.0, dtype=torch.float32, device=DEV),
            "touched": torch.full((B * n,), -7, dtype=torch.int32, device=DEV),
            "n_touched": torch.full((1,), -7, dtype=torch.int32, device=DEV),
            "W_rows": torch.zeros((B * n, d), dtype=dtype, device=DEV)}


def _same(a, b, n):
    assert torch.equal(a["loss"], b["loss"]) and torch.equal(a["dZ"], b["dZ"])
    assert torch.equal(a["n_touched"], b["n_touched"])
    assert torch.equal(a["touched"][:n], b["touched"][:n])
    assert torch.equal(a["W_rows"][:n].view(torch.uint8), b["W_rows"][:n].view(torch.uint8))


@pytest.mark.parametrize("kind", [0, 1])
def test_static_entry_point_matches_xc_step_on_two_calls_in_a_row(kind):
    import paper_2409_20156_amd as xc
    shapes = [(512, 131072, 768, torch.bfloat16, 4, 320),     # the c2 step; about 13 MB of temporaries
              (37, 5000, 72, torch.bfloat16, 3, 45),          # then a smaller, ragged one
              (32, 4096, 64, torch.float32, 1, 24)]           # and Tiny (fp32)
    cases = [_case(11 + i, *s) for i, s in enumerate(shapes)]
    want = []
    for (Z, W, pos, neg, logq), s in zip(cases, shapes):
        Wg = W.clone()
        o = xc.xc_step(Z, Wg, pos, neg, logq, 0.05, kind=kind, want_rows=True)
        torch.cuda.synchronize()
        want.append((o, Wg))
    for (Z, W, pos, neg, logq), s, (o, Wg) in zip(cases, shapes, want):     # back to back, no allocation in between
        B, L, d, dtype, k_p, n_neg = s
        Ws = W.clone()
        out = _outputs(B, d, k_p + n_neg, dtype)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        xc.xc_step_static(Z, Ws, pos, neg, logq, 0.05, kind=kind, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        n = int(out["n_touched"].item())
        assert n > 0
        _same(out, o, n)
        assert torch.equal(Ws.view(torch.uint8), Wg.view(torch.uint8))


def test_static_entry_point_refuses_what_does_not_fit():
    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import binding
    assert xc.step_workspace(2048, 768, 8, 1124, xc.XC_BF16) > binding.STATIC_SCRATCH_BYTES
    Z = torch.zeros((2048, 768), dtype=torch.bfloat16, device=DEV)
    W = torch.zeros((1000, 768), dtype=torch.bfloat16, device=DEV)
    pos = torch.zeros((2048, 8), dtype=torch.int32, device=DEV)
    neg = torch.zeros((2048, 1124), dtype=torch.int32, device=DEV)
    logq = torch.zeros((2048, 1124), dtype=torch.float32, device=DEV)
    out = _outputs(2048, 768, 1, torch.bfloat16)
    with pytest.raises(xc.XcError) as e:
        xc.xc_step_static(Z, W, pos, neg, logq, 0.05, out=out)
    assert e.value.status == -6
