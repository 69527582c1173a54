"""Error behaviour of the library on a GPU machine: nothing is launched and nothing is written when
an argument is rejected, and the Python binding raises instead of falling back."""
import ctypes

import pytest
import torch

from paper_2409_20156_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_workspace_too_small_and_misaligned_pointers_are_rejected():
    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import binding
    lib = binding.load_library()
    Zq, L, d, k = 64, 1000, 64, 8
    W = synth.make_matrix(1, synth.TAG_W, L, d, torch.bfloat16, DEV)
    Z = synth.make_matrix(1, synth.TAG_Z, Zq, d, torch.bfloat16, DEV)
    need = xc.mine_workspace(Zq, L, d, k, xc.XC_BF16)
    ws = torch.zeros(need, dtype=torch.uint8, device=DEV)
    out = torch.full((Zq, k), -7, dtype=torch.int32, device=DEV)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.xc_mine_negatives(Z.data_ptr(), W.data_ptr(), Zq, L, d, k, xc.XC_BF16, out.data_ptr(), None,
                               ws.data_ptr(), need - 1, st)
    assert rc == -3                                              # XC_EWORKSPACE
    rc = lib.xc_mine_negatives(Z.data_ptr() + 2, W.data_ptr(), Zq, L, d, k, xc.XC_BF16, out.data_ptr(), None,
                               ws.data_ptr(), need, st)
    assert rc == -1                                              # misaligned Z
    rc = lib.xc_mine_negatives_warm(Z.data_ptr(), W.data_ptr(), Zq, L, d, k, xc.XC_BF16, ctypes.c_float(-0.5),
                                    out.data_ptr(), None, ws.data_ptr(), need, st)
    assert rc == -1                                              # a negative margin
    rc = lib.xc_mine_negatives_warm(Z.data_ptr(), W.data_ptr(), Zq, L, d, k, xc.XC_BF16, ctypes.c_float(float("nan")),
                                    out.data_ptr(), None, ws.data_ptr(), need, st)
    assert rc == -1
    torch.cuda.synchronize()
    assert (out == -7).all() and not ws.any()                    # nothing ran
    assert lib.xc_strerror(-3).decode().startswith("workspace")
    # the binding turns a status into an exception
    with pytest.raises(binding.XcError):
        xc.mine_negatives(Z, W, 0)
    with pytest.raises(ValueError):
        xc.mine_negatives(Z, W.float(), k)
    # ... and refuses host tensors: there is no CPU path
    with pytest.raises(Exception):
        xc.mine_negatives(Z.cpu(), W.cpu(), k)


def test_step_rejects_short_workspace_without_touching_w():
    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import binding
    lib = binding.load_library()
    B, L, d, k_p, n_neg = 8, 500, 64, 2, 12
    W = synth.make_matrix(2, synth.TAG_W, L, d, torch.float32, DEV)
    Z = synth.make_matrix(2, synth.TAG_Z, B, d, torch.float32, DEV)
    W0 = W.clone()
    pos = torch.zeros((B, k_p), dtype=torch.int32, device=DEV)
    neg = torch.ones((B, n_neg), dtype=torch.int32, device=DEV)
    logq = torch.zeros((B, n_neg), dtype=torch.float32, device=DEV)
    need = xc.step_workspace(B, d, k_p, n_neg, xc.XC_F32)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    loss = torch.zeros(1, device=DEV)
    dZ = torch.zeros((B, d), device=DEV)
    touched = torch.zeros(B * (k_p + n_neg), dtype=torch.int32, device=DEV)
    nt = torch.zeros(1, dtype=torch.int32, device=DEV)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.xc_step(Z.data_ptr(), W.data_ptr(), B, L, d, pos.data_ptr(), k_p, neg.data_ptr(), logq.data_ptr(),
                     n_neg, ctypes.c_float(0.1), 0, xc.XC_F32, loss.data_ptr(), dZ.data_ptr(), touched.data_ptr(),
                     nt.data_ptr(), None, ws.data_ptr(), need // 2, st)
    assert rc == -3
    rc = lib.xc_step(Z.data_ptr(), W.data_ptr(), B, L, d, pos.data_ptr(), k_p, neg.data_ptr(), logq.data_ptr(),
                     n_neg, ctypes.c_float(0.1), 5, xc.XC_F32, loss.data_ptr(), dZ.data_ptr(), touched.data_ptr(),
                     nt.data_ptr(), None, ws.data_ptr(), need, st)
    assert rc == -1                                              # unknown loss kind
    torch.cuda.synchronize()
    assert torch.equal(W, W0) and int(nt.item()) == 0
