"""Refresh-period sweep (the stale versus up-to-date hard negatives trade-off of Sec. 3.1):
throughput of the Alg. 1 loop and the overlap between consecutive shortlists, as a function
of the number of steps tau_r between two refreshes.

  python -m paper_2409_20156_amd.refresh_sweep [--workload c2] [--steps 100] [--taus 1,5,20,100]

For every tau_r the same synthetic job is run twice from the same initial W: once timed (no
host synchronisation inside the loop), once to measure, at every refresh after the first, the
mean over the pool's queries of |fresh shortlist & stale shortlist| / k_h.  One JSON line per
tau_r.  Inputs are the synthetic stand-ins of the benchmark (seeded); only the throughput and
the set overlap are reported, no accuracy.
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import synth
from .schedule import Schedule


def _job(wl, dev):
    W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, dev)
    Z = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, wl.pool, wl.d, wl.torch_dtype, dev)
    pos = synth.zipf_positives(synth.BASE_SEED, wl.pool, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
    Z = synth.add_positive_signal(Z, W, pos)
    return W, Z, torch.tensor(pos, device=dev)


def _overlap(stale, fresh):
    hit = (fresh[:, :, None] == stale[:, None, :]).any(dim=2)
    return float(hit.float().sum(dim=1).mean().item()) / fresh.shape[1]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--taus", default="1,5,20,100")
    ap.add_argument("--warm-margin", type=float, default=-1.0,
                    help="refreshes after the first start from the previous thresholds lowered by this relative margin (negative: full search)")
    ap.add_argument("--lag", type=int, default=0, help="steps a refresh runs beside the training steps before it takes over (0 = synchronous)")
    args = ap.parse_args()
    dev = "cuda:0"
    wl = synth.WORKLOADS[args.workload]
    seeds = [synth.step_seed(synth.BASE_SEED, wl.config_id, t) for t in range(args.steps)]
    for tau in [int(x) for x in args.taus.split(",")]:
        # timed run
        W, Z, pos = _job(wl, dev)
        sch = Schedule(Z, W, pos, wl.B, wl.k_h, wl.k_r, 0, tau, wl.lr, lag=min(args.lag, tau),
                       warm_margin=args.warm_margin if args.warm_margin >= 0 else None)
        sch.step(seeds[0])                                   # first refresh and step: warm-up, untimed
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(1, args.steps):
            sch.step(seeds[t])
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        full_repeats = int(sch.full_repeats.item())
        # overlap run (same trajectory: everything is deterministic)
        W, Z, pos = _job(wl, dev)
        sch = Schedule(Z, W, pos, wl.B, wl.k_h, wl.k_r, 0, tau, wl.lr, lag=min(args.lag, tau),
                       warm_margin=args.warm_margin if args.warm_margin >= 0 else None)
        overlaps = []
        for t in range(args.steps):
            sch.step(seeds[t])
            if sch.refreshed:
                pair = sch.previous_and_fresh()
                if pair is not None:
                    torch.cuda.synchronize()
                    overlaps.append(_overlap(*pair))
        torch.cuda.synchronize()
        n = args.steps - 1
        print(json.dumps({"workload": wl.name, "tau_r": tau, "lag": min(args.lag, tau), "steps": args.steps,
                          "refreshes_timed": sum(1 for t in range(1, args.steps) if t % tau == 0),
                          "steps_per_s": n / el, "queries_per_s": n * wl.B / el,
                          "mean_overlap_fresh_vs_stale": sum(overlaps) / len(overlaps) if overlaps else None,
                          "min_overlap": min(overlaps) if overlaps else None,
                          "warm_margin": args.warm_margin if args.warm_margin >= 0 else None,
                          "warm_searches_repeated_in_full": full_repeats}), flush=True)


if __name__ == "__main__":
    main()
