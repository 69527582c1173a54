"""Comparison helpers shared by the GPU parity tests (no method arithmetic:
the expected values always come from the oracle)."""
import numpy as np
import torch

TOL = {"f32": 1e-5, "bf16": 2e-3}


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def dtype_name(t: torch.Tensor) -> str:
    return "f32" if t.dtype == torch.float32 else "bf16"


def check_topk(ids_gpu, sc_gpu, ids_or, sc_or, Z64, W64, tie_rel=1e-5, score_rtol=1e-5):
    """Top-k parity with the tie clause: an id may differ from the oracle's only
    where its exact score is within tie_rel (relative) of the oracle's k-th
    score, resp. of the score at the same rank.  Returns the number of queries
    that needed the clause.  W64 is the float64 matrix, or, where that is too
    large to hold, a function (ids) -> float64 rows together with the label count."""
    ids_gpu = np.asarray(ids_gpu)
    n_tied = 0
    if isinstance(W64, tuple):
        rows_of, n_labels = W64

        class _Rows:
            shape = (n_labels,)

            def __getitem__(self, idx):
                return rows_of(np.atleast_1d(np.asarray(idx, dtype=np.int64)))[0 if np.ndim(idx) == 0 else slice(None)]
        W64 = _Rows()
    for i in range(ids_or.shape[0]):
        if (ids_gpu[i] == ids_or[i]).all():
            continue
        n_tied += 1
        g, o = ids_gpu[i], ids_or[i]
        assert len(set(g.tolist())) == len(g), "duplicate id in row %d" % i
        assert ((g >= 0) & (g < W64.shape[0])).all()
        sk = sc_or[i, -1]
        tol = tie_rel * max(abs(sk), 1e-30)
        exact_g = W64[g] @ Z64[i]                       # oracle-precision scores of the GPU's ids
        for l in set(g.tolist()) ^ set(o.tolist()):
            s = float(W64[l] @ Z64[i])
            assert abs(s - sk) <= tol, (i, l, s, sk)
        # rank by rank the exact scores must agree up to the tie tolerance
        assert np.all(np.abs(exact_g - sc_or[i]) <= tie_rel * np.maximum(np.abs(sc_or[i]), 1e-30)), i
    if sc_gpu is not None:
        sg = np.asarray(sc_gpu, dtype=np.float64)
        assert np.allclose(sg, sc_or, rtol=score_rtol, atol=score_rtol * np.abs(sc_or).max()), \
            np.abs(sg - sc_or).max()
    return n_tied


def check_rows_close(got, want, tol, what, floor=None):
    """Per row: max abs error relative to the row's largest magnitude, or to `floor`
    (per row) where that is larger: the size of the terms of a sum that cancels."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.size == 0:
        return 0.0
    scale = np.maximum(np.abs(want).max(axis=-1, keepdims=True), 1e-30)
    if floor is not None:
        scale = np.maximum(scale, np.asarray(floor, dtype=np.float64).reshape(-1, 1))
    err = (np.abs(got - want) / scale).max()
    assert err <= tol, "%s: relative error %.3e > %.1e" % (what, err, tol)
    return err


def check_bf16_rows(got, want, old, what, max_mismatch_frac=2e-3, slack=None):
    """Stored bf16 rows: norm-wise 2e-3 (the stated bar), and element-wise at
    most one bf16 ulp apart, on a small fraction of elements only: an fp32 sum
    and an fp64 sum can straddle a rounding boundary.  Where the update nearly
    cancels the old value the ulp of the result is tiny, so the fp32 error of
    the operands (2^-18 of the larger of old and new element: sums in float32 and
    hardware exp2/log2/rcp in the coefficients) is allowed on top.  `slack`
    (per row, optional) adds the float32 error of a gradient sum whose terms cancel:
    the caller passes about 2e-6 * lr * sum|g| * max|z| of the row.
    One ulp is up to 2^-7 of the element, so in a row of fewer than 64 elements a
    single such straddle can by itself exceed 2e-3 of the row's norm: there the
    norm-wise bar is applied to the differences beyond one ulp, and the straddles
    are bounded by the element-wise test and their count alone."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    old = np.asarray(old, dtype=np.float64)
    assert got.shape == want.shape == old.shape
    if got.size == 0:
        return
    _, e = np.frexp(np.maximum(np.abs(want), np.abs(got)))
    ulp = np.ldexp(1.0, np.maximum(e, -125) - 8)
    diff = np.abs(got - want)
    counted = diff if got.shape[-1] >= 64 else np.where(diff <= ulp * 1.0000001, 0.0, diff)
    num = np.linalg.norm(counted, axis=-1)
    den = np.maximum(np.linalg.norm(want, axis=-1), 1e-30)
    assert (num / den).max() <= 2e-3, (what, (num / den).max())
    allowed = ulp * 1.0000001 + 2.0 ** -18 * np.maximum(np.abs(old), np.abs(want))
    if slack is not None:
        allowed = allowed + np.asarray(slack, dtype=np.float64).reshape(-1, 1)
    assert (diff <= allowed).all(), (what, (diff / allowed).max())
    frac = (diff > 0).mean()
    assert frac <= max_mismatch_frac, (what, frac)
