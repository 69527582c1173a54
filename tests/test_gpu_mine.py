"""GPU parity of xc_mine_negatives against the oracle's exact top-k."""
import numpy as np
import pytest
import torch

from oracle import astra_oracle as orc
from paper_2409_20156_amd import synth
from tests.parity import check_topk, f64

pytestmark = pytest.mark.gpu


def _run(Z, W, k):
    import paper_2409_20156_amd as xc
    ids, sc = xc.mine_negatives(Z, W, k, want_scores=True)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), sc.cpu().numpy()


def _case(seed, Zq, L, d, dtype, k):
    dev = "cuda:0"
    W = synth.make_matrix(seed, synth.TAG_W, L, d, dtype, dev)
    Z = synth.make_matrix(seed, synth.TAG_Z, Zq, d, dtype, dev)
    ids, sc = _run(Z, W, k)
    Z64, W64 = f64(Z), f64(W)
    ids_o, sc_o = orc.mine_negatives(Z64, W64, k)
    n_tied = check_topk(ids, sc, ids_o, sc_o, Z64, W64)
    for i in range(Zq):                      # invariants that hold at any size
        assert len(set(ids[i].tolist())) == k
        assert (np.diff(sc[i]) <= 0).all()
    return n_tied


@pytest.mark.parametrize("Zq,L,d,dtype,k", [
    (32, 4096, 64, torch.float32, 8),          # the Tiny configuration
    (200, 5000, 72, torch.bfloat16, 50),       # ragged query tile, ragged label tile, K tail
    (130, 1000, 40, torch.float32, 100),       # fp32 K tail (160-byte rows)
    (1, 300, 64, torch.bfloat16, 1),
    (3, 64, 64, torch.bfloat16, 64),           # k = L, single partial tile
    (257, 3000, 768, torch.bfloat16, 128),     # maximum k, d of the large configurations
    (5, 129, 8, torch.bfloat16, 7),            # minimum row (16 bytes)
    # 128-byte rows are one pipeline stage per tile, and query tiles with few real queries leave half
    # of the waves with nothing to filter: they run a tile ahead of the others
    (78, 30000, 64, torch.bfloat16, 63),
    (200, 30000, 64, torch.bfloat16, 63),
    (600, 30000, 64, torch.bfloat16, 63),
    (78, 30000, 32, torch.float32, 63),
    (78, 16384, 64, torch.bfloat16, 8),
    # bf16 rows of 128, 256, 384 and 512 bytes take the kernel that keeps the query tile in registers
    (300, 70000, 256, torch.bfloat16, 50),     # the row shape of the largest configuration
    (513, 9000, 192, torch.bfloat16, 100),     # three query tiles, the last with one query; ragged last label tile
    (64, 200, 256, torch.bfloat16, 128),       # maximum k, fewer labels than two tiles
    (257, 40000, 128, torch.bfloat16, 64),
    (31, 127, 64, torch.bfloat16, 127),        # a single ragged label tile, k = L
])
def test_mine_matches_oracle(Zq, L, d, dtype, k):
    print("case", Zq, L, d, dtype, k, flush=True)
    _case(11, Zq, L, d, dtype, k)


def test_mine_long_slices_exercise_list_reduction():
    # 512 queries x 131072 labels: 4096 labels per slice, so candidate lists fill and are reduced
    print("case long slices", flush=True)
    _case(5, 512, 131072, 64, torch.bfloat16, 64)


@pytest.mark.parametrize("L,Zq,k,d", [(40000, 140, 33, 16), (300000, 260, 128, 16), (40000, 140, 33, 64),
                                      (300000, 260, 128, 256), (150000, 700, 100, 128)])
def test_mine_increasing_scores_worst_case_for_the_threshold(L, Zq, k, d):
    # score(i, l) grows with l: every label beats the running threshold, in every phase, so every
    # accumulator is parked and the candidate lists are cut all the time (32-byte rows: the general kernel,
    # its pools and shared lists; 128..512-byte rows: the lists of the kernel with register-resident queries)
    dev = "cuda:0"
    base = torch.ones(d, dtype=torch.float32)
    W = (torch.arange(L, dtype=torch.float32)[:, None] / 65536.0 * base[None, :]).to(torch.bfloat16).to(dev)
    Z = torch.ones((Zq, d), dtype=torch.bfloat16, device=dev)
    Z[1::2] *= -1.0                                  # odd queries prefer small ids
    ids, sc = _run(Z, W, k)
    Z64, W64 = f64(Z), f64(W)
    ids_o, sc_o = orc.mine_negatives(Z64, W64, k)
    check_topk(ids, sc, ids_o, sc_o, Z64, W64)
    assert (ids == ids_o).all()                      # bf16 products of these values are exact: no tolerance needed


@pytest.mark.parametrize("mode", ["narrow", "wide"])
@pytest.mark.parametrize("Zq,L,d,k", [(300, 70000, 256, 50), (513, 9000, 192, 100), (1100, 20000, 128, 64),
                                      (40, 3000, 64, 128)])
def test_row_kernel_layouts_match_oracle(monkeypatch, mode, Zq, L, d, k):
    # the kernel for short bf16 rows has two wave layouts (work items of 256 or of 512 queries) and picks one
    # by the pool size; XC_MINE_ROWS in the environment, read at every call, forces either
    monkeypatch.setenv("XC_MINE_ROWS", mode)
    print("case", mode, Zq, L, d, k, flush=True)
    _case(17, Zq, L, d, torch.bfloat16, k)


@pytest.mark.parametrize("mode", ["narrow", "wide"])
def test_row_kernel_layouts_worst_case_lists(monkeypatch, mode):
    # increasing scores (every label passes, lists are cut all the time) in both layouts
    monkeypatch.setenv("XC_MINE_ROWS", mode)
    dev = "cuda:0"
    L, Zq, k, d = 150000, 700, 100, 128
    W = (torch.arange(L, dtype=torch.float32)[:, None] / 65536.0 * torch.ones(d)[None, :]).to(torch.bfloat16).to(dev)
    Z = torch.ones((Zq, d), dtype=torch.bfloat16, device=dev)
    Z[1::2] *= -1.0
    ids, sc = _run(Z, W, k)
    ids_o, sc_o = orc.mine_negatives(f64(Z), f64(W), k)
    assert (ids == ids_o).all()


@pytest.mark.parametrize("mode", ["narrow", "wide"])
def test_row_kernel_layouts_warm_repeat_of_some_tiles(monkeypatch, mode):
    # a warm search that has to repeat the full search for one 256-query tile out of three: a work item of
    # 512 queries then holds a tile that repeats and one that keeps the result of the sweep
    import paper_2409_20156_amd as xc
    monkeypatch.setenv("XC_MINE_ROWS", mode)
    dev = "cuda:0"
    Zq, L, d, k = 700, 20000, 128, 50
    Z = synth.make_matrix(5, synth.TAG_Z, Zq, d, torch.bfloat16, dev)
    W = synth.make_matrix(5, synth.TAG_W, L, d, torch.bfloat16, dev)
    ws = torch.empty(xc.mine_workspace(Zq, L, d, k, xc.XC_BF16), dtype=torch.uint8, device=dev)
    xc.mine_negatives(Z, W, k, workspace=ws)
    for lo, want in ((300, [0, 1, 0]), (10, [1, 0, 0]), (600, [0, 0, 1])):
        Zp = Z.clone()
        Zp[lo:lo + 50] = (Zp[lo:lo + 50].float() * 0.05).to(torch.bfloat16)
        xc.mine_negatives(Z, W, k, workspace=ws)                   # thresholds of the unchanged queries
        ids, sc = xc.mine_negatives(Zp, W, k, want_scores=True, workspace=ws, warm_margin=0.05)
        assert _fallback_flag(ws) == 1
        assert ws[:16].view(torch.int32).cpu().numpy()[1:4].tolist() == want
        ids_o, sc_o = orc.mine_negatives(f64(Zp), f64(W), k)
        check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o, f64(Zp), f64(W))


def test_mine_all_scores_equal_orders_by_id():
    dev = "cuda:0"
    W = torch.zeros((3000, 64), dtype=torch.bfloat16, device=dev)
    Z = synth.make_matrix(1, synth.TAG_Z, 70, 64, torch.bfloat16, dev)
    ids, sc = _run(Z, W, 20)
    assert (ids == np.arange(20)[None, :]).all()
    assert (sc == 0).all()


def test_mine_planted_rows_come_first():
    dev = "cuda:0"
    L, d, Zq, k = 20000, 128, 64, 10
    W = synth.make_matrix(2, synth.TAG_W, L, d, torch.bfloat16, dev)
    Z = synth.make_matrix(2, synth.TAG_Z, Zq, d, torch.bfloat16, dev)
    plant = (torch.arange(Zq) * 311 + 7) % L
    W[plant.to(dev)] = (Z.float() * 8.0).to(torch.bfloat16)       # <z, 8 z> dwarfs every random score
    ids, _ = _run(Z, W, k)
    assert (ids[:, 0] == plant.numpy()).all()


def test_mine_is_reproducible_run_to_run():
    dev = "cuda:0"
    W = synth.make_matrix(3, synth.TAG_W, 30000, 64, torch.bfloat16, dev)
    Z = synth.make_matrix(3, synth.TAG_Z, 300, 64, torch.bfloat16, dev)
    a = _run(Z, W, 64)
    b = _run(Z, W, 64)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_inference_topk_precision_on_planted_positives():
    """The same search serves prediction (top-5 labels of a query): queries are noisy copies of
    their label's row, precision@k of the GPU result equals the oracle's and is high."""
    dev = "cuda:0"
    L, d, Zq, k = 50000, 256, 400, 5
    W = synth.make_matrix(4, synth.TAG_W, L, d, torch.bfloat16, dev)
    noise = synth.make_matrix(4, synth.TAG_Z, Zq, d, torch.bfloat16, dev)
    truth = (np.arange(Zq) * 97 + 3) % L
    Z = (W[torch.as_tensor(truth, device=dev)].float() + 0.8 * noise.float()).to(torch.bfloat16)
    ids, sc = _run(Z, W, k)
    Z64, W64 = f64(Z), f64(W)
    ids_o, sc_o = orc.mine_negatives(Z64, W64, k)
    check_topk(ids, sc, ids_o, sc_o, Z64, W64)
    p1 = float((ids[:, 0] == truth).mean())
    p5 = float((ids == truth[:, None]).any(axis=1).mean())
    assert p1 == float((ids_o[:, 0] == truth).mean()) and p5 == float((ids_o == truth[:, None]).any(axis=1).mean())
    assert p1 > 0.9 and p5 >= p1


def _fallback_flag(ws):
    torch.cuda.synchronize()
    return int(ws[:4].view(torch.int32).item())


def test_warm_search_is_exact_whatever_the_workspace_holds():
    """The warm search starts from the thresholds left in the workspace; the result must equal the
    oracle's in every case: thresholds that still fit (one sweep), thresholds that a changed W
    has overtaken (the call repeats the full search), and a workspace that never saw a search."""
    import paper_2409_20156_amd as xc
    dev = "cuda:0"
    Zq, L, d, k = 300, 20000, 64, 50
    Z = synth.make_matrix(3, synth.TAG_Z, Zq, d, torch.bfloat16, dev)
    W = synth.make_matrix(3, synth.TAG_W, L, d, torch.bfloat16, dev)
    Z64 = f64(Z)
    ws = torch.empty(xc.mine_workspace(Zq, L, d, k, xc.XC_BF16), dtype=torch.uint8, device=dev)

    def check(Wc, ids, sc):
        ids_o, sc_o = orc.mine_negatives(Z64, f64(Wc), k)
        check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o, Z64, f64(Wc))

    # a workspace with arbitrary content: nothing to start from
    ws.random_(0, 255)
    ids, sc = xc.mine_negatives(Z, W, k, want_scores=True, workspace=ws, warm_margin=0.1)
    check(W, ids, sc)
    # same W again: the old k-th scores are exact thresholds, even with no margin
    ids, sc = xc.mine_negatives(Z, W, k, want_scores=True, workspace=ws, warm_margin=0.0)
    assert _fallback_flag(ws) == 0
    check(W, ids, sc)
    # a small drift of every row: the margin covers it
    W2 = (W.float() + 0.002 * synth.make_matrix(4, synth.TAG_W, L, d, torch.float32, dev)).to(torch.bfloat16)
    ids, sc = xc.mine_negatives(Z, W2, k, want_scores=True, workspace=ws, warm_margin=0.2)
    assert _fallback_flag(ws) == 0
    check(W2, ids, sc)
    # W shrunk to a tenth: every score falls far below its old threshold -> full search
    W3 = (W2.float() * 0.1).to(torch.bfloat16)
    ids, sc = xc.mine_negatives(Z, W3, k, want_scores=True, workspace=ws, warm_margin=0.05)
    assert _fallback_flag(ws) == 1
    check(W3, ids, sc)
    # only some queries overtaken (their embeddings shrunk): the full search is repeated for their
    # tile of 256 queries, the other tile keeps the result of the sweep
    ids, sc = xc.mine_negatives(Z, W3, k, want_scores=True, workspace=ws)
    Zp = Z.clone()
    Zp[10:60] = (Zp[10:60].float() * 0.05).to(torch.bfloat16)
    ids, sc = xc.mine_negatives(Zp, W3, k, want_scores=True, workspace=ws, warm_margin=0.05)
    assert _fallback_flag(ws) == 1
    flags = ws[:12].view(torch.int32).cpu().numpy()
    assert flags[1] == 1 and flags[2] == 0
    ids_o, sc_o = orc.mine_negatives(f64(Zp), f64(W3), k)
    check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o, f64(Zp), f64(W3))
    # a margin so wide that nearly every score passes: slow, still exact
    ids, sc = xc.mine_negatives(Z, W3, k, want_scores=True, workspace=ws, warm_margin=50.0)
    assert _fallback_flag(ws) == 0
    check(W3, ids, sc)
    # the cold call is unaffected by what the warm ones left
    ids, sc = xc.mine_negatives(Z, W, k, want_scores=True, workspace=ws)
    check(W, ids, sc)
