"""Outer loop of Alg. 1 over the three library calls (classifier only, fixed query pool).

Argument marshalling and the step counter only: warm-up steps with uniform negatives while
t < tau_s, then a refresh of the whole pool's shortlists every tau_r steps (xc_mine_negatives
with the current W) and hard + random steps (xc_sample_negatives, xc_step).  All buffers are
allocated once, before the first step.

With lag > 0 the refresh is asynchronous, as in the paper's pipeline: at a refresh step the
current W is copied to a snapshot, the search runs on a second stream (default priority) over
that snapshot while the training steps go on with the older shortlists, and the new shortlists
take over exactly `lag` steps later (the step stream waits for the search there), so the result
does not depend on timing.
"""
from __future__ import annotations

import torch

from . import binding as xc


class Schedule:
    def __init__(self, Z_pool: torch.Tensor, W: torch.Tensor, pos_pool: torch.Tensor, B: int, k_h: int,
                 k_r: int, tau_s: int, tau_r: int, lr: float, kind: int = xc.XC_LOSS_BCE, lag: int = 0,
                 warm_margin: float | None = None):
        if lag < 0 or (lag > 0 and lag > tau_r):
            raise ValueError("lag must lie in [0, tau_r]")
        self.Z, self.W, self.pos = Z_pool, W, pos_pool
        self.B, self.k_h, self.k_r, self.tau_s, self.tau_r, self.lr, self.kind = B, k_h, k_r, tau_s, tau_r, lr, kind
        self.lag = lag
        self.warm_margin = warm_margin                 # refreshes after the first start from the last thresholds
        self.searched = False
        self.full_repeats = torch.zeros(1, dtype=torch.int32, device=W.device)   # warm searches that had to be repeated in full
        dev = W.device
        pool, d = Z_pool.shape
        L = W.shape[0]
        self.pool, self.L = pool, L
        self.nbatch = max(1, pool // B)
        code = xc.XC_F32 if W.dtype == torch.float32 else xc.XC_BF16
        n_neg = k_h + k_r
        k_p = pos_pool.shape[1]
        self.mine_ws = torch.empty(xc.mine_workspace(pool, L, d, k_h, code), dtype=torch.uint8, device=dev)
        self.step_ws = torch.empty(xc.step_workspace(B, d, k_p, n_neg, code), dtype=torch.uint8, device=dev)
        self.shortlist = [torch.empty((pool, k_h), dtype=torch.int32, device=dev) for _ in range(2)]
        self.cur = -1                                  # index of the active shortlist buffer, -1 = none yet
        self.built = -1                                # index of the newest built (or being built) buffer
        self.pending = None                            # (activation step, buffer index, event) of a running search
        self.neg = torch.empty((B, n_neg), dtype=torch.int32, device=dev)
        self.logq = torch.empty((B, n_neg), dtype=torch.float32, device=dev)
        P = B * (k_p + n_neg)
        self.out = {"loss": torch.empty(1, dtype=torch.float32, device=dev),
                    "dZ": torch.empty((B, d), dtype=torch.float32, device=dev),
                    "touched": torch.empty(P, dtype=torch.int32, device=dev),
                    "n_touched": torch.empty(1, dtype=torch.int32, device=dev)}
        if lag > 0:
            self.W_snap = torch.empty_like(W)
            self.side = torch.cuda.Stream(device=dev)              # default priority
        self.t = 0
        self.refreshed = False                         # the last step() call started (lag>0) or did a refresh
        self.had_previous = False

    def previous_and_fresh(self):
        """(previous, newest) shortlist tensors after a refresh that had a predecessor, else None.
        With lag > 0 the caller must synchronise before reading the newest one."""
        if self.built < 0 or not self.had_previous:
            return None
        return self.shortlist[1 - self.built], self.shortlist[self.built]

    stale_and_fresh = previous_and_fresh

    def state_dict(self):
        """Everything a later `load_state_dict` needs to go on from here with the same results: the step
        counter, both shortlist buffers and which of them is active, built or waiting to take over, and a
        copy of W.  A search still running on the second stream is waited for first (its takeover step is kept),
        so the call synchronises.  The search thresholds are not part of it: the first refresh after a resume
        starts from scratch, which returns the same shortlists as one started from earlier thresholds."""
        if self.pending is not None:
            self.pending[2].synchronize()
        torch.cuda.synchronize(self.W.device)
        return {"t": self.t, "cur": self.cur, "built": self.built, "had_previous": self.had_previous,
                "pending": None if self.pending is None else (self.pending[0], self.pending[1]),
                "full_repeats": int(self.full_repeats.item()),
                "shortlist": [s.cpu().clone() for s in self.shortlist], "W": self.W.cpu().clone()}

    def load_state_dict(self, sd):
        """Back to the state `state_dict` saved (same pool, shapes and schedule parameters); W is overwritten."""
        if tuple(sd["W"].shape) != tuple(self.W.shape) or sd["W"].dtype != self.W.dtype:
            raise ValueError("the saved W does not fit this schedule")
        if any(tuple(a.shape) != tuple(b.shape) for a, b in zip(sd["shortlist"], self.shortlist)):
            raise ValueError("the saved shortlists do not fit this schedule")
        if self.pending is not None:
            self.pending[2].synchronize()
        self.W.copy_(sd["W"])
        for dst, src in zip(self.shortlist, sd["shortlist"]):
            dst.copy_(src)
        self.t, self.cur, self.built, self.had_previous = sd["t"], sd["cur"], sd["built"], sd["had_previous"]
        self.full_repeats.fill_(sd["full_repeats"])
        self.pending = None
        if sd["pending"] is not None:
            if self.lag == 0:
                raise ValueError("the saved state waits for an asynchronous search; this schedule has lag 0")
            done = torch.cuda.Event()
            done.record(torch.cuda.current_stream())           # the buffer is complete: nothing left to wait for
            self.pending = (sd["pending"][0], sd["pending"][1], done)
        self.searched = False
        self.refreshed = False
        torch.cuda.synchronize(self.W.device)

    def step(self, seed: int):
        t = self.t
        self.refreshed = False
        main = torch.cuda.current_stream()
        if self.pending is not None and self.pending[0] <= t:
            main.wait_event(self.pending[2])           # the search has to be finished from here on
            self.cur = self.pending[1]                 # (also before its snapshot and workspace are reused)
            self.pending = None
        if t >= self.tau_s and (t - self.tau_s) % self.tau_r == 0:
            nxt = 0 if self.built < 0 else 1 - self.built
            self.had_previous = self.built >= 0
            if self.lag == 0:
                warm = self.warm_margin if self.searched else None
                xc.mine_negatives(self.Z, self.W, self.k_h, workspace=self.mine_ws, out=self.shortlist[nxt],
                                  warm_margin=warm)
                if warm is not None:
                    self.full_repeats += self.mine_ws[:4].view(torch.int32)
                self.cur = nxt
            else:
                self.W_snap.copy_(self.W)                                      # on the step stream
                snap_done = torch.cuda.Event()
                snap_done.record(main)
                done = torch.cuda.Event()
                with torch.cuda.stream(self.side):
                    self.side.wait_event(snap_done)
                    warm = self.warm_margin if self.searched else None
                    xc.mine_negatives(self.Z, self.W_snap, self.k_h, workspace=self.mine_ws, out=self.shortlist[nxt],
                                      warm_margin=warm)
                    if warm is not None:
                        self.full_repeats += self.mine_ws[:4].view(torch.int32)
                    done.record(self.side)
                self.pending = (t + self.lag, nxt, done)
            self.built = nxt
            self.searched = True
            self.refreshed = True
        b = t % self.nbatch
        lo, hi = b * self.B, (b + 1) * self.B
        rows = self.shortlist[self.cur][lo:hi] if self.cur >= 0 else None
        xc.sample_negatives(rows, self.k_h, self.k_r, self.L, seed, B=self.B, device=self.W.device,
                            neg=self.neg, logq=self.logq)
        xc.xc_step(self.Z[lo:hi], self.W, self.pos[lo:hi], self.neg, self.logq, self.lr, kind=self.kind,
                   workspace=self.step_ws, out=self.out)
        self.t += 1
        return self.out
