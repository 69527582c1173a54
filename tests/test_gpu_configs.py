"""GPU parity at the full sizes of the benchmark configurations (c2..c5), in the
launch configuration bench.py uses (whole query pool for mining, whole batch for
sampling and the step).  Outputs are compared with the oracle on sampled queries
and labels that it can compute one by one; what cannot be sampled is checked
through properties that hold at any size.  All oracle inputs are synthetic or
oracle-made (never an output of the HIP path): the oracle gets a renumbered
sub-problem holding exactly the rows of W that the sampled pairs use.
"""
import numpy as np
import pytest
import torch

from oracle import astra_oracle as orc
from paper_2409_20156_amd import synth
from tests.parity import TOL, check_bf16_rows, check_rows_close, check_topk, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N_SAMPLE = 6          # queries of the first batch the oracle recomputes per configuration
SUB_BATCH = 160       # queries of the reduced batch that is compared in full (loss included)


class Job:
    def __init__(self, name):
        wl = synth.WORKLOADS[name]
        self.wl = wl
        self.W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, DEV)
        self.Z = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, wl.pool, wl.d, wl.torch_dtype, DEV)
        self.pos = synth.zipf_positives(synth.BASE_SEED, wl.B, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
        # first batch: positives pull their query (structured variant of the input recipe)
        self.Z[:wl.B] = synth.add_positive_signal(self.Z[:wl.B], self.W, self.pos)
        rng = np.random.default_rng(wl.config_id)
        self.sample_q = np.sort(rng.choice(wl.B, size=N_SAMPLE, replace=False))     # for the step tests (one batch)

    def original_rows(self, ids):
        """float64 rows of W as generated (W itself may have been updated in place)."""
        t = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=DEV)
        return f64(synth.gaussian_rows_at(synth.BASE_SEED, synth.TAG_W, t, self.wl.d, self.wl.torch_dtype))

    def restore(self, ids):
        """Put the generated rows back after an in-place step."""
        t = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=DEV)
        for a in range(0, t.numel(), 1 << 16):
            sel = t[a:a + (1 << 16)]
            self.W[sel] = synth.gaussian_rows_at(synth.BASE_SEED, synth.TAG_W, sel, self.wl.d, self.wl.torch_dtype)


@pytest.fixture(scope="module", params=["c2", "c3", "c4", "c5"])
def job(request):
    free, _ = torch.cuda.mem_get_info()
    wl = synth.WORKLOADS[request.param]
    if free < wl.L * wl.d * 2 * 1.1 + 6e9:
        pytest.skip("not enough device memory for %s" % request.param)
    print("building", request.param, flush=True)
    j = Job(request.param)
    yield j
    del j
    torch.cuda.empty_cache()


def _rows64(W, ids):
    return f64(W[torch.as_tensor(np.asarray(ids, dtype=np.int64), device=W.device)])


# ------------------------------------------------------------------ mining ----
def _mining_sample(wl):
    """Queries the search is compared on, drawn from the whole pool: every query of one whole tile of 256
    that lies outside the first batch (all positions of a tile), 64 more spread over the pool (tiles that
    the search's schedule binds to other compute units and dies), queries of the first batch (structured
    rows) and the last query."""
    rng = np.random.default_rng(40 + wl.config_id)
    n_tiles = (wl.pool + 255) // 256
    tile = max(wl.B // 256 + 1, (2 * n_tiles) // 3) if n_tiles > wl.B // 256 + 1 else n_tiles - 1
    whole = np.arange(tile * 256, min(wl.pool, tile * 256 + 256))
    spread = rng.choice(wl.pool, size=min(64, wl.pool), replace=False)
    first = rng.choice(wl.B, size=N_SAMPLE, replace=False)
    return np.unique(np.concatenate([whole, spread, first, [wl.pool - 1]]))


def _oracle_topk_streamed(job, Zs, k, chunk_rows=1 << 20):
    """The oracle's exhaustive search over a label set too large for one float64 matrix: its search on one
    chunk of rows after the other, and again on the winners so far together with the chunk's winners
    (candidates kept in label order, so the oracle's tie rule holds across chunks)."""
    nq = Zs.shape[0]
    best_ids = [np.zeros(0, np.int64) for _ in range(nq)]
    best_rows = [np.zeros((0, Zs.shape[1])) for _ in range(nq)]
    for n_done, l0 in enumerate(range(0, job.wl.L, chunk_rows)):
        Wc = f64(job.W[l0:l0 + chunk_rows])
        ids_c, _ = orc.mine_negatives(Zs, Wc, min(k, Wc.shape[0]))
        for r in range(nq):
            ids = np.concatenate([best_ids[r], l0 + ids_c[r].astype(np.int64)])
            rows = np.concatenate([best_rows[r], Wc[ids_c[r]]])
            o = np.argsort(ids)
            sel, _ = orc.mine_negatives(Zs[r:r + 1], rows[o], min(k, len(ids)))
            best_ids[r], best_rows[r] = ids[o][sel[0]], rows[o][sel[0]]
        if n_done % 16 == 0:
            print("  oracle search, labels from", l0, flush=True)
    ids = np.stack(best_ids)
    sc = np.stack([best_rows[r] @ Zs[r] for r in range(nq)])
    return ids.astype(np.int32), sc


def test_mining_full_pool(job):
    import paper_2409_20156_amd as xc
    wl = job.wl
    print("mine", wl.name, wl.pool, wl.L, flush=True)
    ids, sc = xc.mine_negatives(job.Z, job.W, wl.k_h, want_scores=True)
    torch.cuda.synchronize()
    qs = _mining_sample(wl)
    assert len(qs) >= 64 + 256
    qt = torch.as_tensor(qs, device=DEV)
    ids_s = ids[qt].cpu().numpy()
    sc_s = sc[qt].cpu().numpy().astype(np.float64)
    Zs = f64(job.Z[qt])
    for r in range(len(qs)):                     # invariants at any size
        assert len(set(ids_s[r].tolist())) == wl.k_h
        assert ((ids_s[r] >= 0) & (ids_s[r] < wl.L)).all()
        assert (np.diff(sc_s[r]) <= 0).all()
    if wl.L * wl.d <= 1.1e9:
        # exact search by the oracle over all L labels for the sampled queries
        W64 = f64(job.W)
        ids_o, sc_o = orc.mine_negatives(Zs, W64, wl.k_h)
        check_topk(ids_s, sc_s, ids_o, sc_o, Zs, W64)
    else:
        # (a) every returned score is the oracle's inner product with that label, one by one;
        # (b) no label outside the list beats the k-th score: counted over all L by a library
        #     matmul (float32 on the GPU, chunked), with the tie tolerance;
        # (c) for two of the queries (one of the whole tile, one elsewhere) the oracle's own exhaustive
        #     search, streamed over all L rows in float64
        for r in range(len(qs)):
            rows = _rows64(job.W, ids_s[r])
            _, exact = orc.mine_negatives(Zs[r:r + 1], rows, wl.k_h)   # these rows' scores, best first
            assert np.allclose(sc_s[r], exact[0], rtol=1e-5, atol=1e-7)
        zq = job.Z[qt].float()
        kth = torch.as_tensor(sc_s[:, -1], device=DEV, dtype=torch.float32)
        thresh = kth + 2e-5 * kth.abs() + 1e-7
        beat = torch.zeros(len(qs), dtype=torch.int64, device=DEV)
        step = 1 << 21
        for l0 in range(0, wl.L, step):
            s = job.W[l0:l0 + step].float() @ zq.T                     # [chunk, nq]
            beat += (s > thresh[None, :]).sum(dim=0)
        # the labels clearly above the k-th score are at most the k-1 listed before it
        assert (beat.cpu().numpy() <= wl.k_h - 1).all(), beat
        two = [int(np.searchsorted(qs, qs[len(qs) // 2])), len(qs) - 1]
        ids_o, sc_o = _oracle_topk_streamed(job, Zs[two], wl.k_h)
        check_topk(ids_s[two], sc_s[two], ids_o, sc_o, Zs[two], (lambda idx: _rows64(job.W, idx), wl.L))


def test_c2_search_from_earlier_thresholds_after_real_steps():
    """The benchmark's own refresh at its full size: a search from scratch over the c2 pool, 20 real steps
    (sampling from the shortlists, row updates at the benchmark's learning rate), then the search started
    from the earlier thresholds with the benchmark's margin.  Its result is compared with the oracle's
    exhaustive search on the moved matrix for every query of two whole tiles outside the first batch and
    of the ragged last tile (the pool is shortened by 100 queries so that there is one)."""
    import paper_2409_20156_amd as xc
    wl = synth.WORKLOADS["c2"]
    pool = wl.pool - 100
    W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, DEV)
    Z = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, pool, wl.d, wl.torch_dtype, DEV)
    pos_np = synth.zipf_positives(synth.BASE_SEED, pool, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
    Z = synth.add_positive_signal(Z, W, pos_np)            # shortlists move between the two searches
    pos = torch.tensor(pos_np, device=DEV)
    code = xc.XC_BF16
    ws = torch.empty(xc.mine_workspace(pool, wl.L, wl.d, wl.k_h, code), dtype=torch.uint8, device=DEV)
    print("c2 search from scratch", flush=True)
    sl0 = xc.mine_negatives(Z, W, wl.k_h, workspace=ws)
    for t in range(20):
        b = t % (pool // wl.B)
        lo, hi = b * wl.B, (b + 1) * wl.B
        neg, logq = xc.sample_negatives(sl0[lo:hi], wl.k_h, wl.k_r, wl.L, synth.step_seed(synth.BASE_SEED, 2, t))
        xc.xc_step(Z[lo:hi], W, pos[lo:hi], neg, logq, wl.lr)
    print("c2 search from the earlier thresholds", flush=True)
    sl1, sc1 = xc.mine_negatives(Z, W, wl.k_h, workspace=ws, warm_margin=0.1, want_scores=True)
    torch.cuda.synchronize()
    repeated = int(ws[:4].view(torch.int32).item())
    n_tiles = (pool + 255) // 256
    qs = np.concatenate([np.arange(t * 256, min(pool, t * 256 + 256)) for t in (7, n_tiles // 2 + 3, n_tiles - 1)])
    assert qs.min() >= wl.B and len(qs) == 2 * 256 + pool % 256
    qt = torch.as_tensor(qs, device=DEV)
    Zs, W64 = f64(Z[qt]), f64(W)
    ids_o, sc_o = orc.mine_negatives(Zs, W64, wl.k_h)
    n_tied = check_topk(sl1[qt].cpu().numpy(), sc1[qt].cpu().numpy().astype(np.float64), ids_o, sc_o, Zs, W64)
    moved = (sl1[qt] != sl0[qt]).any(dim=1).float().mean().item()
    print("full search repeated for some tile: %d; rows needing the tie clause: %d; shortlists changed: %.2f"
          % (repeated, n_tied, moved), flush=True)
    assert moved > 0.05                                     # the steps did move the classifier


# ---------------------------------------------------------------- sampling ----
def test_sampling_full_batch(job):
    import paper_2409_20156_amd as xc
    wl = job.wl
    rng = np.random.default_rng(7)
    # a synthetic shortlist (distinct ids per query); the sampler does not care where it came from
    sl = np.stack([rng.choice(wl.L, size=wl.k_h, replace=False) for _ in range(wl.B)]).astype(np.int32)
    seed = synth.step_seed(synth.BASE_SEED, wl.config_id, 3)
    neg, logq = xc.sample_negatives(torch.tensor(sl, device=DEV), wl.k_h, wl.k_r, wl.L, seed)
    torch.cuda.synchronize()
    neg = neg.cpu().numpy()
    logq = logq.cpu().numpy()
    rows = [int(q) for q in job.sample_q[:3]] + [wl.B - 1]
    neg_o, logq_o = orc.sample_negatives(sl, wl.B, wl.k_h, wl.k_r, wl.L, seed, rows=rows)
    assert (neg[rows] == neg_o[rows]).all()
    assert np.allclose(logq[rows], logq_o[rows], rtol=2e-7)
    # properties over the whole batch
    assert (neg[:, :wl.k_h] == sl).all()
    assert ((neg >= 0) & (neg < wl.L)).all()
    for i in range(0, wl.B, max(1, wl.B // 64)):
        assert not set(neg[i, wl.k_h:].tolist()) & set(sl[i].tolist())


# -------------------------------------------------------------------- step ----
def _synthetic_negatives(wl, rng):
    """Negatives with the shape and statistics of the sampler's output, made on the host: k_h
    'hard' ids concentrated on few labels (queries share them) and k_r uniform ids."""
    hot = (rng.zipf(1.5, size=(wl.B, wl.k_h)).astype(np.int64) * 7919) % wl.L
    rnd = rng.integers(0, wl.L, size=(wl.B, wl.k_r))
    neg = np.concatenate([hot, rnd], axis=1).astype(np.int32)
    logq = np.zeros(neg.shape, dtype=np.float32)
    logq[:, wl.k_h:] = np.float32(np.log(wl.k_r / (wl.L - wl.k_h)))
    return neg, logq


def _compact(job, pos, neg, queries):
    """The sub-problem of `queries` with labels renumbered to the rows it uses.
    Returns (used label ids, original float64 rows, pos', neg')."""
    L = job.wl.L
    p, ng = pos[queries].astype(np.int64), neg[queries].astype(np.int64)
    used = np.unique(np.concatenate([p[(p >= 0) & (p < L)], ng[(ng >= 0) & (ng < L)]]))

    def remap(a):
        inside = (a >= 0) & (a < L)
        return np.where(inside, np.searchsorted(used, np.clip(a, 0, L - 1)), -1).astype(np.int32)
    return used, job.original_rows(used), remap(p), remap(ng)


def _masks(wl, pos, neg, kind):
    """Which (query, negative slot) pairs count, and which queries count at all."""
    masked = (neg[:, :, None] == pos[:, None, :]).any(axis=2) | (neg < 0) | (neg >= wl.L)
    pos_ok = (pos >= 0) & (pos < wl.L)
    active = pos_ok.any(axis=1) if kind == orc.LOSS_SOFTMAX else np.ones(len(pos), bool)
    return masked, pos_ok, active


@pytest.mark.parametrize("kind", [orc.LOSS_BCE, orc.LOSS_SOFTMAX])
def test_step_full_batch(job, kind):
    import paper_2409_20156_amd as xc
    wl = job.wl
    name, tol = wl.dtype, TOL[wl.dtype]
    rng = np.random.default_rng(100 + wl.config_id)
    neg, logq = _synthetic_negatives(wl, rng)
    pos = job.pos.copy()
    neg[1, 3] = pos[1, 0]                       # a positive among the hard negatives
    neg[2, wl.k_h + 1] = -1                     # padding
    Zb = job.Z[:wl.B]
    print("step", wl.name, kind, flush=True)
    out = xc.xc_step(Zb, job.W, torch.tensor(pos, device=DEV), torch.tensor(neg, device=DEV),
                     torch.tensor(logq, device=DEV), wl.lr, kind=kind)       # W updated in place
    torch.cuda.synchronize()
    nt = int(out["n_touched"].item())
    touched = out["touched"][:nt].cpu().numpy()
    try:
        masked, pos_ok, active = _masks(wl, pos, neg, kind)
        # property: touched = sorted distinct ids of the unmasked pairs of the active queries
        ids_all = np.concatenate([pos[active][pos_ok[active]], neg[active][~masked[active]]])
        want_ids = np.unique(ids_all)
        assert nt == len(want_ids) and (touched == want_ids).all()
        # property: rows outside the touched list are the generated ones, bit for bit (sampled)
        others = np.setdiff1d(rng.integers(0, wl.L, size=2000), touched)
        assert (_rows64(job.W, others) == job.original_rows(others)).all()

        # sampled queries: dZ row by the oracle on the one-query problem (coefficients carry 1/B)
        for q in job.sample_q:
            used, rows, p1, n1 = _compact(job, pos, neg, np.array([q]))
            ref = orc.xc_step(f64(Zb[q:q + 1]), rows, p1, n1, logq[[q]], wl.lr, kind=kind)
            check_rows_close(out["dZ"][q:q + 1].cpu().numpy() * wl.B, ref["dZ"], tol, "dZ row %d" % q)

        # sampled labels: the updated row by the oracle on the queries that use the label
        vals, counts = np.unique(ids_all, return_counts=True)
        shared = vals[(counts >= 2) & (counts <= 48)]
        labels = [int(touched[0]), int(touched[nt // 2]), int(touched[-1])] + [int(x) for x in shared[:3]]
        got_rows = _rows64(job.W, labels)
        for l, got in zip(labels, got_rows):
            uses = ((pos == l) & pos_ok).any(axis=1) | ((neg == l) & ~masked).any(axis=1)
            qsel = np.where(uses & active)[0]
            assert 1 <= len(qsel)
            if len(qsel) > 48:
                continue
            used, rows, pq, nq = _compact(job, pos, neg, qsel)
            ref = orc.xc_step(f64(Zb[torch.as_tensor(qsel, device=DEV)]), rows, pq, nq, logq[qsel],
                              wl.lr * len(qsel) / wl.B, kind=kind, storage=name)     # lr rescaled: 1/|sub| -> 1/B
            r = int(np.searchsorted(used, l))
            k = int(np.where(ref["touched"] == r)[0][0])
            old = rows[r]
            if name == "bf16":
                gsum = sum(abs(g) for q in range(len(qsel)) for ll, g in ref["coef"][q] if ll == r)
                slack = 2e-6 * wl.lr * len(qsel) / wl.B * gsum * np.abs(f64(Zb[torch.as_tensor(qsel, device=DEV)])).max()
                # one row at a time: the share of elements that may sit one ulp off (an fp32 and an fp64 sum on
                # two sides of a rounding boundary) has a granularity of 1/d here, so the bound that is 0.2 % over
                # many rows is "at most four elements of the row"
                check_bf16_rows(got[None, :], ref["W_rows"][k][None, :], old[None, :], "row %d" % l,
                                max_mismatch_frac=4.0 / wl.d, slack=[slack])
            else:
                check_rows_close(got[None, :], ref["W_rows"][k][None, :], tol, "row %d" % l)
    finally:
        job.restore(touched)


@pytest.mark.parametrize("kind", [orc.LOSS_BCE, orc.LOSS_SOFTMAX])
def test_step_reduced_batch_in_full(job, kind):
    """The same shapes with a batch the oracle can redo completely: loss, all of dZ, all rows."""
    import paper_2409_20156_amd as xc
    wl = job.wl
    name, tol = wl.dtype, TOL[wl.dtype]
    rng = np.random.default_rng(200 + wl.config_id)
    neg, logq = _synthetic_negatives(wl, rng)
    nb = SUB_BATCH
    pos, neg, logq = job.pos[:nb].copy(), neg[:nb], logq[:nb]
    neg[0, 0] = pos[0, 0]
    Zb = job.Z[:nb]
    print("reduced step", wl.name, kind, flush=True)
    out = xc.xc_step(Zb, job.W, torch.tensor(pos, device=DEV), torch.tensor(neg, device=DEV),
                     torch.tensor(logq, device=DEV), wl.lr, kind=kind, want_rows=True)
    torch.cuda.synchronize()
    nt = int(out["n_touched"].item())
    touched = out["touched"][:nt].cpu().numpy()
    try:
        used, rows, pq, nq = _compact(job, pos, neg, np.arange(nb))
        ref = orc.xc_step(f64(Zb), rows, pq, nq, logq, wl.lr, kind=kind, storage=name)
        loss = float(out["loss"].item())
        assert abs(loss - ref["loss"]) <= tol * abs(ref["loss"]), (loss, ref["loss"])
        check_rows_close(out["dZ"].cpu().numpy(), ref["dZ"], tol, "dZ")
        assert nt == len(ref["touched"]) and (touched == used[ref["touched"]]).all()
        got = f64(out["W_rows"][:nt])
        if name == "bf16":
            gsum = np.zeros(len(used))                     # sum of |d loss/d score| per label
            for q in range(nb):
                for l, g in ref["coef"][q]:
                    gsum[l] += abs(g)
            slack = 2e-6 * wl.lr * gsum[ref["touched"]] * np.abs(f64(Zb)).max()
            check_bf16_rows(got, ref["W_rows"], rows[ref["touched"]], "W rows", slack=slack)
        else:
            check_rows_close(got, ref["W_rows"], tol, "W rows")
        assert (_rows64(job.W, touched) == got).all()
    finally:
        job.restore(touched)


# ------------------------------------------------------- several steps in a row ----
@pytest.mark.parametrize("name,nb", [("c2", None), ("c3", None), ("c5", SUB_BATCH)])
def test_steps_in_sequence_each_side_on_its_own_trajectory(name, nb):
    """Three BCE steps, the library on its W and the oracle on its own float64 copy of the generated rows
    (rounded to bf16 after every step, as stored): no state passes between the two.  c2 and c3 at full batch
    size with the whole matrix on the oracle's side; c5 (rows updated inside the gather, wide sort keys) with a
    reduced batch and, for the oracle, the renumbered sub-problem of the rows that the three steps use.  Per step:
    the touched list is equal, loss and dZ within the one-step tolerance times the number of steps so far (a row
    that came out one ulp apart feeds the next step).  At the end every row that was touched is compared:
    norm-wise 2e-3, element-wise at most two bf16 ulps of the largest value the element held, and different at all
    on at most 0.6 % of the elements (0.2 % per step)."""
    import paper_2409_20156_amd as xc
    free, _ = torch.cuda.mem_get_info()
    wl = synth.WORKLOADS[name]
    if free < wl.L * wl.d * 2 * 1.1 + 6e9:
        pytest.skip("not enough device memory for %s" % name)
    job = Job(name)
    tol = TOL[wl.dtype]
    B = nb if nb is not None else wl.B
    n_steps = 3
    Zb = job.Z[:B]
    Z64 = f64(Zb)
    pos = job.pos[:B]
    negs = [_synthetic_negatives(wl, np.random.default_rng(300 + 10 * wl.config_id + t)) for t in range(n_steps)]
    negs = [(ng[:B], lq[:B]) for ng, lq in negs]
    if nb is None:
        ids_of = np.arange(wl.L)                       # the oracle holds every row
        W64 = f64(job.W)
        pos_o, negs_o = pos, [ng for ng, _ in negs]
    else:
        allids = np.concatenate([pos.reshape(-1)] + [ng.reshape(-1) for ng, _ in negs]).astype(np.int64)
        ids_of = np.unique(allids[(allids >= 0) & (allids < wl.L)])
        W64 = job.original_rows(ids_of)

        def remap(a):
            a = a.astype(np.int64)
            inside = (a >= 0) & (a < wl.L)
            return np.where(inside, np.searchsorted(ids_of, np.clip(a, 0, wl.L - 1)), -1).astype(np.int32)
        pos_o, negs_o = remap(pos), [remap(ng) for ng, _ in negs]
    U = len(ids_of)
    pos_t = torch.tensor(pos, device=DEV)
    ever = np.zeros(U, dtype=bool)
    gsum = np.zeros(U)                                 # per label: sum of |d loss / d score| over all steps
    peak = np.abs(W64).astype(np.float32)              # per element: the largest magnitude it had at any step
    for t in range(n_steps):
        neg, logq = negs[t]
        print("sequence", name, "step", t, flush=True)
        out = xc.xc_step(Zb, job.W, pos_t, torch.tensor(neg, device=DEV), torch.tensor(logq, device=DEV), wl.lr)
        torch.cuda.synchronize()
        ref = orc.xc_step(Z64, W64, pos_o, negs_o[t], logq, wl.lr, storage=wl.dtype)
        W64[ref["touched"]] = ref["W_rows"]
        peak[ref["touched"]] = np.maximum(peak[ref["touched"]], np.abs(ref["W_rows"]).astype(np.float32))
        ever[ref["touched"]] = True
        for lst in ref["coef"]:
            for l, g in lst:
                gsum[l] += abs(g)
        nt = int(out["n_touched"].item())
        assert nt == len(ref["touched"]) and (out["touched"][:nt].cpu().numpy() == ids_of[ref["touched"]]).all()
        loss = float(out["loss"].item())
        assert abs(loss - ref["loss"]) <= (t + 1) * tol * abs(ref["loss"]), (t, loss, ref["loss"])
        check_rows_close(out["dZ"].cpu().numpy(), ref["dZ"], (t + 1) * tol, "dZ of step %d" % t)
    rows = np.where(ever)[0]
    got, want = _rows64(job.W, ids_of[rows]), W64[rows]
    diff = np.abs(got - want)
    # the ulp of the largest value the element held on the way: a rounding that fell differently at one step
    # stays in the element as an absolute difference, also where later updates shrink the element
    big = np.maximum(peak[rows].astype(np.float64), np.abs(got))
    _, e = np.frexp(big)
    ulp = np.ldexp(1.0, np.maximum(e, -125) - 8)
    assert (np.linalg.norm(diff, axis=1) / np.maximum(np.linalg.norm(want, axis=1), 1e-30)).max() <= 2e-3
    # (plus the float32 error of the operands and of a gradient sum whose terms cancel, as in check_bf16_rows)
    allowed = 2.0000001 * ulp + 2.0 ** -17 * big + (2e-6 * wl.lr * gsum[rows] * np.abs(Z64).max())[:, None]
    assert (diff <= allowed).all(), float((diff / allowed).max())
    assert (diff > 0).mean() <= 0.002 * n_steps, float((diff > 0).mean())
    if nb is None:
        others = np.where(~ever)[0][:4000]
    else:
        others = np.setdiff1d(np.random.default_rng(7).integers(0, wl.L, size=4000), ids_of)
    assert (_rows64(job.W, others) == job.original_rows(others)).all()   # never touched: the generated bits
