"""Thin ctypes binding of libastra_xc.so: argument marshalling only.

Every function takes torch CUDA tensors, checks dtype / contiguity / device,
and passes raw device pointers plus the current HIP stream to the C entry point
of the same name.  Outputs and workspaces are allocated with torch.
"""
from __future__ import annotations

import ctypes
import os

import torch

XC_F32, XC_BF16 = 0, 1
XC_LOSS_BCE, XC_LOSS_SOFTMAX = 0, 1

_LIB = None
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libastra_xc.so")

_i64, _i32, _f32, _u64 = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_uint64
_ptr, _szp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)

_SIGNATURES = {
    "xc_strerror": (ctypes.c_char_p, [_i32]),
    "xc_last_hip_error": (_i32, []),
    "xc_version": (_i32, []),
    "xc_mine_workspace": (_i32, [_i64, _i64, _i32, _i32, _i32, _szp]),
    "xc_mine_negatives": (_i32, [_ptr, _ptr, _i64, _i64, _i32, _i32, _i32, _ptr, _ptr, _ptr,
                                 ctypes.c_size_t, _ptr]),
    "xc_mine_negatives_warm": (_i32, [_ptr, _ptr, _i64, _i64, _i32, _i32, _i32, ctypes.c_float, _ptr, _ptr, _ptr,
                                      ctypes.c_size_t, _ptr]),
    "xc_sample_negatives": (_i32, [_ptr, _i64, _i32, _i32, _i64, _u64, _ptr, _ptr, _ptr]),
    "xc_sample_negatives_mixture": (_i32, [ctypes.c_void_p, ctypes.c_void_p, _i64, _i32, _i32, _i32, _i64,
                                           ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "xc_sample_negatives_pps": (_i32, [ctypes.c_void_p, ctypes.c_void_p, _i64, _i32, _i32, _i32, _i64,
                                       ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "xc_step_workspace": (_i32, [_i64, _i32, _i32, _i32, _i32, _szp]),
    "xc_profile_enable": (_i32, [_i32]),
    "xc_profile_collect": (_i32, []),
    "xc_profile_get": (_i32, [_i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                              ctypes.POINTER(ctypes.c_int64)]),
    "xc_profile_reset": (_i32, []),
    "xc_copy_probe": (_i32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "xc_mfma_probe": (_i32, [ctypes.c_void_p, _i32, _i32, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]),
    "xc_step": (_i32, [_ptr, _ptr, _i64, _i64, _i32, _ptr, _i32, _ptr, _ptr, _i32, _f32, _i32, _i32,
                       _ptr, _ptr, _ptr, _ptr, _ptr, _ptr, ctypes.c_size_t, _ptr]),
    "xc_step_static": (_i32, [_ptr, _ptr, _i64, _i64, _i32, _ptr, _i32, _ptr, _ptr, _i32, _f32, _i32, _i32,
                              _ptr, _ptr, _ptr, _ptr, _ptr, _ptr]),
}
STATIC_SCRATCH_BYTES = 32 << 20


class XcError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load_library()
        msg = lib.xc_strerror(status).decode()
        if status == -4:
            msg += " hipError=%d" % lib.xc_last_hip_error()
        super().__init__("%s: %s (status %d)" % (where, msg, status))
        self.status = status


def load_library():
    """Load libastra_xc.so from the package directory; fail loudly if it is not built."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libastra_xc.so is not built: run `python -m paper_2409_20156_amd.build` "
                               "(or __graft_entry__.build())")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def exported_symbols():
    return sorted(_SIGNATURES)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return XC_F32
    if t.dtype == torch.bfloat16:
        return XC_BF16
    raise TypeError("Z and W must be float32 or bfloat16, got %s" % t.dtype)


def _dev(t: torch.Tensor, dtype=None, name="tensor"):
    if not t.is_cuda:
        raise RuntimeError("%s must live on the GPU: this library has no CPU path" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise XcError(status, where)


def mine_workspace(Zq: int, L: int, d: int, k_h: int, dtype_code: int) -> int:
    lib = load_library()
    n = ctypes.c_size_t(0)
    _check(lib.xc_mine_workspace(Zq, L, d, k_h, dtype_code, ctypes.byref(n)), "xc_mine_workspace")
    return n.value


def mine_negatives(Z: torch.Tensor, W: torch.Tensor, k_h: int, *, want_scores: bool = False,
                   workspace: torch.Tensor | None = None, out: torch.Tensor | None = None,
                   warm_margin: float | None = None):
    """shortlist int32 [Zq, k_h] (and fp32 scores if asked): exact top-k_h of Z W^T per row.

    warm_margin (relative, >= 0): start from the thresholds the previous search left in `workspace`
    (same result, usually less time); `workspace[:4]` viewed as int32 is 1 afterwards if the full
    search had to be repeated."""
    lib = load_library()
    code = _dtype_code(Z)
    if W.dtype != Z.dtype or Z.dim() != 2 or W.dim() != 2 or Z.shape[1] != W.shape[1]:
        raise ValueError("Z [Zq,d] and W [L,d] must share dtype and d")
    Zq, d = Z.shape
    L = W.shape[0]
    need = mine_workspace(Zq, L, d, k_h, code)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Z.device)
    if out is None:
        out = torch.empty((Zq, k_h), dtype=torch.int32, device=Z.device)
    scores = torch.empty((Zq, k_h), dtype=torch.float32, device=Z.device) if want_scores else None
    if warm_margin is None:
        _check(lib.xc_mine_negatives(_dev(Z, name="Z"), _dev(W, name="W"), Zq, L, d, k_h, code,
                                     _dev(out, torch.int32, "shortlist"),
                                     _dev(scores, torch.float32, "scores") if want_scores else None,
                                     _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()),
               "xc_mine_negatives")
    else:
        _check(lib.xc_mine_negatives_warm(_dev(Z, name="Z"), _dev(W, name="W"), Zq, L, d, k_h, code,
                                          float(warm_margin), _dev(out, torch.int32, "shortlist"),
                                          _dev(scores, torch.float32, "scores") if want_scores else None,
                                          _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()),
               "xc_mine_negatives_warm")
    return (out, scores) if want_scores else out


def sample_negatives(shortlist: torch.Tensor | None, k_h: int, k_r: int, L: int, seed: int, *,
                     B: int | None = None, device=None, neg: torch.Tensor | None = None,
                     logq: torch.Tensor | None = None):
    """neg int32 [B, k_h+k_r], logq fp32 [B, k_h+k_r]; shortlist None = warm-up phase."""
    lib = load_library()
    if shortlist is not None:
        if shortlist.dim() != 2 or shortlist.shape[1] != k_h:
            raise ValueError("shortlist must be [B, k_h]")
        B = shortlist.shape[0]
        device = shortlist.device
    elif B is None or device is None:
        raise ValueError("warm-up mode needs B and device")
    n = k_h + k_r
    if neg is None:
        neg = torch.empty((B, n), dtype=torch.int32, device=device)
    if logq is None:
        logq = torch.empty((B, n), dtype=torch.float32, device=device)
    _check(lib.xc_sample_negatives(_dev(shortlist, torch.int32, "shortlist") if shortlist is not None else None,
                                   B, k_h, k_r, L, seed & ((1 << 64) - 1),
                                   _dev(neg, torch.int32, "neg"), _dev(logq, torch.float32, "logq"), _stream()),
           "xc_sample_negatives")
    return neg, logq


def sample_negatives_mixture(shortlist: torch.Tensor, scores: torch.Tensor, k_h: int, k_r: int, L: int,
                             seed: int, *, neg: torch.Tensor | None = None, logq: torch.Tensor | None = None):
    """neg int32 [B, k_h+k_r], logq fp32: k_h draws proportional to the sigmoid of the stale scores over
    the [B, M] shortlist plus k_r uniform draws from [0, L)."""
    lib = load_library()
    if shortlist.dim() != 2 or scores.shape != shortlist.shape:
        raise ValueError("shortlist and scores must both be [B, M]")
    B, M = shortlist.shape
    n = k_h + k_r
    if neg is None:
        neg = torch.empty((B, n), dtype=torch.int32, device=shortlist.device)
    if logq is None:
        logq = torch.empty((B, n), dtype=torch.float32, device=shortlist.device)
    _check(lib.xc_sample_negatives_mixture(_dev(shortlist, torch.int32, "shortlist"),
                                           _dev(scores, torch.float32, "scores"), B, M, k_h, k_r, L,
                                           seed & ((1 << 64) - 1), _dev(neg, torch.int32, "neg"),
                                           _dev(logq, torch.float32, "logq"), _stream()),
           "xc_sample_negatives_mixture")
    return neg, logq


def sample_negatives_pps(shortlist: torch.Tensor, scores: torch.Tensor, k_h: int, k_r: int, L: int,
                         seed: int, *, neg: torch.Tensor | None = None, logq: torch.Tensor | None = None):
    """neg int32 [B, k_h+k_r], logq fp32: up to k_h slots of the [B, M] shortlist chosen without replacement with
    probability proportional to the sigmoid of the stale scores, the other slots uniform draws from [0, L)."""
    lib = load_library()
    if shortlist.dim() != 2 or scores.shape != shortlist.shape:
        raise ValueError("shortlist and scores must both be [B, M]")
    B, M = shortlist.shape
    n = k_h + k_r
    if neg is None:
        neg = torch.empty((B, n), dtype=torch.int32, device=shortlist.device)
    if logq is None:
        logq = torch.empty((B, n), dtype=torch.float32, device=shortlist.device)
    _check(lib.xc_sample_negatives_pps(_dev(shortlist, torch.int32, "shortlist"),
                                       _dev(scores, torch.float32, "scores"), B, M, k_h, k_r, L,
                                       seed & ((1 << 64) - 1), _dev(neg, torch.int32, "neg"),
                                       _dev(logq, torch.float32, "logq"), _stream()),
           "xc_sample_negatives_pps")
    return neg, logq


def step_workspace(B: int, d: int, k_p: int, n_neg: int, dtype_code: int) -> int:
    lib = load_library()
    n = ctypes.c_size_t(0)
    _check(lib.xc_step_workspace(B, d, k_p, n_neg, dtype_code, ctypes.byref(n)), "xc_step_workspace")
    return n.value


def xc_step_static(Z: torch.Tensor, W: torch.Tensor, pos: torch.Tensor, neg: torch.Tensor, logq: torch.Tensor,
                   lr: float, *, kind: int = XC_LOSS_BCE, out: dict) -> dict:
    """xc_step through the entry point that allocates nothing: temporaries live in the library's static
    device array, every output tensor comes from the caller in `out` (loss, dZ, touched, n_touched and
    optionally W_rows).  Raises XcError(-6) when the shape needs more than STATIC_SCRATCH_BYTES."""
    lib = load_library()
    code = _dtype_code(Z)
    if W.dtype != Z.dtype or Z.shape[1] != W.shape[1]:
        raise ValueError("Z [B,d] and W [L,d] must share dtype and d")
    B, d = Z.shape
    L = W.shape[0]
    k_p, n_neg = pos.shape[1], neg.shape[1]
    if pos.shape[0] != B or neg.shape[0] != B or tuple(logq.shape) != tuple(neg.shape):
        raise ValueError("pos [B,k_p], neg [B,n_neg], logq [B,n_neg] expected")
    rows = out.get("W_rows")
    _check(lib.xc_step_static(_dev(Z, name="Z"), _dev(W, name="W"), B, L, d,
                              _dev(pos, torch.int32, "pos") if k_p else None, k_p,
                              _dev(neg, torch.int32, "neg") if n_neg else None,
                              _dev(logq, torch.float32, "logq") if n_neg else None, n_neg,
                              float(lr), kind, code, _dev(out["loss"], torch.float32, "loss"),
                              _dev(out["dZ"], torch.float32, "dZ"), _dev(out["touched"], torch.int32, "touched"),
                              _dev(out["n_touched"], torch.int32, "n_touched"),
                              _dev(rows, W.dtype, "W_rows") if rows is not None else None, _stream()),
           "xc_step_static")
    return out


def xc_step(Z: torch.Tensor, W: torch.Tensor, pos: torch.Tensor, neg: torch.Tensor, logq: torch.Tensor,
            lr: float, *, kind: int = XC_LOSS_BCE, want_rows: bool = False,
            workspace: torch.Tensor | None = None, out: dict | None = None) -> dict:
    """One classifier step; W is updated in place.  Returns dict(loss [1], dZ [B,d] fp32,
    touched int32 [B*n] (first n_touched valid), n_touched int32 [1], W_rows or None)."""
    lib = load_library()
    code = _dtype_code(Z)
    if W.dtype != Z.dtype or Z.shape[1] != W.shape[1]:
        raise ValueError("Z [B,d] and W [L,d] must share dtype and d")
    B, d = Z.shape
    L = W.shape[0]
    k_p, n_neg = pos.shape[1], neg.shape[1]
    if pos.shape[0] != B or neg.shape[0] != B or tuple(logq.shape) != tuple(neg.shape):
        raise ValueError("pos [B,k_p], neg [B,n_neg], logq [B,n_neg] expected")
    P = B * (k_p + n_neg)
    need = step_workspace(B, d, k_p, n_neg, code)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Z.device)
    if out is None:
        out = {}
    dev = Z.device
    loss = out.get("loss") if out.get("loss") is not None else torch.empty(1, dtype=torch.float32, device=dev)
    dZ = out.get("dZ") if out.get("dZ") is not None else torch.empty((B, d), dtype=torch.float32, device=dev)
    touched = out.get("touched") if out.get("touched") is not None else torch.empty(P, dtype=torch.int32, device=dev)
    n_touched = out.get("n_touched") if out.get("n_touched") is not None else torch.empty(1, dtype=torch.int32, device=dev)
    rows = None
    if want_rows:
        rows = out.get("W_rows") if out.get("W_rows") is not None else torch.empty((P, d), dtype=W.dtype, device=dev)
    _check(lib.xc_step(_dev(Z, name="Z"), _dev(W, name="W"), B, L, d,
                       _dev(pos, torch.int32, "pos") if k_p else None, k_p,
                       _dev(neg, torch.int32, "neg") if n_neg else None,
                       _dev(logq, torch.float32, "logq") if n_neg else None, n_neg,
                       float(lr), kind, code, _dev(loss, torch.float32, "loss"), _dev(dZ, torch.float32, "dZ"),
                       _dev(touched, torch.int32, "touched"), _dev(n_touched, torch.int32, "n_touched"),
                       _dev(rows, W.dtype, "W_rows") if want_rows else None,
                       _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()),
           "xc_step")
    return {"loss": loss, "dZ": dZ, "touched": touched, "n_touched": n_touched, "W_rows": rows}


def profile_enable(on: bool) -> None:
    _check(load_library().xc_profile_enable(1 if on else 0), "xc_profile_enable")


def profile_reset() -> None:
    _check(load_library().xc_profile_reset(), "xc_profile_reset")


def profile_collect() -> dict:
    """Per-kernel {name: (total_ms, launches)} of the launches made while profiling was on."""
    lib = load_library()
    n = lib.xc_profile_collect()
    out = {}
    for i in range(n):
        name, ms, cnt = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_int64()
        _check(lib.xc_profile_get(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(cnt)), "xc_profile_get")
        out[name.value.decode()] = (ms.value, cnt.value)
    return out


def copy_probe(dst, src) -> None:
    """Launch the plain copy kernel over two equal-sized uint8 device tensors (counter calibration)."""
    if dst.numel() != src.numel():
        raise ValueError("copy_probe: sizes differ")
    _check(load_library().xc_copy_probe(_dev(dst, torch.uint8, "dst"), _dev(src, torch.uint8, "src"),
                                        src.numel(), _stream()), "xc_copy_probe")


def mfma_probe(iters: int, random_operands: bool) -> float:
    """Launch the register-resident MFMA loop once; returns the flop of the launch."""
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda:0")
    flop = ctypes.c_double()
    _check(load_library().xc_mfma_probe(_dev(out, torch.float32, "out"), int(iters), 1 if random_operands else 0,
                                        ctypes.byref(flop), _stream()), "xc_mfma_probe")
    return flop.value
