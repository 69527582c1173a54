#!/usr/bin/env python3
"""Throughput of the ASTRA classifier-layer hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
xc_sample_negatives + xc_step, plus, every `refresh` steps, xc_mine_negatives over
the whole query pool (the shortlist refresh of Alg. 1).  The default workload is
the second configuration of the baseline file (L=131072, d=768, bf16, B=512,
k_h=64, k_r=256, refresh every 20 steps, pool of 10240 queries).

Prints ONE JSON line.  `value` is queries/s over the timed region with all
inputs resident in HBM.  `roofline` describes the kernel that takes the most
time, timed per launch with HIP events on its own stream in a second pass over
the same steps (so the event records do not perturb `value`).  `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", help="tiny, c2, c3, c4 or c5")
    ap.add_argument("--pool", type=int, default=0, help="override the mined query pool size")
    ap.add_argument("--warm-margin", type=float, default=0.1,
                    help="refreshes after the first start from the thresholds of the one before, lowered by this "
                         "relative margin (xc_mine_negatives_warm: same shortlists); negative: every refresh is a full search")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch the library's plain copy kernel over this many MiB (three times), "
                         "for scaling hardware traffic counters in rocprofv3 --pmc runs")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="measured HBM bytes per launch from rocprofv3 --pmc runs, if present")
    return ap.parse_args()


class Job:
    """Device-resident state of one workload and the step function."""

    def __init__(self, wl, pool, device="cuda:0", warm_margin=None):
        import numpy as np
        import torch

        import paper_2409_20156_amd as xc
        from paper_2409_20156_amd import synth
        self.xc, self.torch, self.wl, self.synth = xc, torch, wl, synth
        self.dev = device
        self.pool = pool
        self.W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, device)
        self.Zpool = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, pool, wl.d, wl.torch_dtype, device)
        pos = synth.zipf_positives(synth.BASE_SEED, pool, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
        self.pos_np = pos
        self.pos = torch.tensor(pos, device=device)
        self.nbatch = max(1, pool // wl.B)
        code = xc.XC_F32 if wl.dtype == "f32" else xc.XC_BF16
        self.code = code
        n_neg = wl.k_h + wl.k_r
        self.mine_ws = torch.empty(xc.mine_workspace(pool, wl.L, wl.d, wl.k_h, code), dtype=torch.uint8, device=device)
        self.step_ws = torch.empty(xc.step_workspace(wl.B, wl.d, wl.k_p, n_neg, code), dtype=torch.uint8, device=device)
        self.shortlist = torch.empty((pool, wl.k_h), dtype=torch.int32, device=device)
        self.neg = torch.empty((wl.B, n_neg), dtype=torch.int32, device=device)
        self.logq = torch.empty((wl.B, n_neg), dtype=torch.float32, device=device)
        P = wl.B * (wl.k_p + n_neg)
        self.out = {"loss": torch.empty(1, dtype=torch.float32, device=device),
                    "dZ": torch.empty((wl.B, wl.d), dtype=torch.float32, device=device),
                    "touched": torch.empty(P, dtype=torch.int32, device=device),
                    "n_touched": torch.empty(1, dtype=torch.int32, device=device)}
        self.valid_pairs = [int((pos[b * wl.B:(b + 1) * wl.B] >= 0).sum()) + wl.B * n_neg
                            for b in range(self.nbatch)]
        self.t = 0
        self.mined = False
        self.warm_margin = warm_margin

    def mine(self):
        # every refresh after the first starts from the thresholds of the one before (same result)
        margin = self.warm_margin if self.mined else None
        self.xc.mine_negatives(self.Zpool, self.W, self.wl.k_h, workspace=self.mine_ws, out=self.shortlist,
                               warm_margin=margin)
        self.mined = True

    def step(self):
        wl, t = self.wl, self.t
        if (wl.refresh and t % wl.refresh == 0) or (not wl.refresh and t == 0):
            self.mine()
        b = t % self.nbatch
        lo, hi = b * wl.B, (b + 1) * wl.B
        seed = self.synth.step_seed(self.synth.BASE_SEED, wl.config_id, t)
        self.xc.sample_negatives(self.shortlist[lo:hi], wl.k_h, wl.k_r, wl.L, seed, neg=self.neg, logq=self.logq)
        self.xc.xc_step(self.Zpool[lo:hi], self.W, self.pos[lo:hi], self.neg, self.logq, wl.lr,
                        workspace=self.step_ws, out=self.out)
        self.t += 1
        return b


def cpu_baseline(wl, pool, budget_queries=None):
    """The oracle as it stands on a bounded sample of 10-20 s of CPU work: mining of
    `budget_queries` queries against all L labels (as many as keep the score matrix
    within 1 GiB, at most 1024; scaled to the pool), and sampling + step of the first
    `nb` queries of a batch (scaled to B)."""
    import numpy as np
    import torch

    from oracle import astra_oracle as orc
    from paper_2409_20156_amd import synth
    nb = min(wl.B, 512)
    if budget_queries is None:
        budget_queries = max(8, min(1024, (1 << 27) // wl.L))
    W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, "cpu").to(torch.float64).numpy()
    Z = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, max(nb, budget_queries), wl.d, wl.torch_dtype, "cpu").to(torch.float64).numpy()
    pos = synth.zipf_positives(synth.BASE_SEED, nb, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
    t0 = time.perf_counter()
    sl, _ = orc.mine_negatives(Z[:budget_queries], W, wl.k_h)
    t_mine_q = (time.perf_counter() - t0) / budget_queries
    sl_b = sl[:nb] if budget_queries >= nb else orc.mine_negatives(Z[:nb], W, wl.k_h)[0]
    t0 = time.perf_counter()
    neg, logq = orc.sample_negatives(sl_b, nb, wl.k_h, wl.k_r, wl.L, 1)
    orc.xc_step(Z[:nb], W, pos, neg, logq, wl.lr, storage=wl.dtype)
    t_step_q = (time.perf_counter() - t0) / nb
    refresh = wl.refresh if wl.refresh else wl.steps
    per_query = t_step_q + t_mine_q * pool / (refresh * wl.B)
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": 1.0 / per_query, "unit": "queries/s", "cores": cores, "kind": "oracle",
            "sample": "mining %d queries x all %d labels scaled to the pool of %d per %d steps; "
                      "sampling+step on %d queries scaled to B=%d; numpy float64 oracle, BLAS threads = cores"
                      % (budget_queries, wl.L, pool, refresh, nb, wl.B),
            "mine_s_per_query": t_mine_q, "step_s_per_query": t_step_q}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import binding, synth
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU")
    xc.load_library()
    wl = synth.WORKLOADS[args.workload]
    pool = args.pool or wl.pool
    job = Job(wl, pool, warm_margin=args.warm_margin if args.warm_margin >= 0 else None)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        job.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        job.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    value = wl.B * args.steps / elapsed
    # for comparison, the same number of steps with a full search at every refresh (untimed for `value`)
    full_search = None
    if job.warm_margin is not None and wl.refresh and not args.no_profile_pass:
        job.warm_margin = None
        t1 = time.perf_counter()
        for _ in range(args.steps):
            job.step()
        torch.cuda.synchronize()
        el1 = time.perf_counter() - t1
        full_search = {"value": wl.B * args.steps / el1, "ms_per_step": el1 * 1e3 / args.steps}
        job.warm_margin = args.warm_margin

    if args.copy_probe_mib:
        a = torch.randint(0, 255, (args.copy_probe_mib << 20,), dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(3):
            binding.copy_probe(b, a)
        torch.cuda.synchronize()
        del a, b

    # ---- second pass: the same number of steps with per-kernel HIP events --------------
    roofline, kernels, mines = None, {}, 0
    if not args.no_profile_pass:
        binding.profile_reset()
        binding.profile_enable(True)
        touched_sum, pairs_sum = 0, 0
        for _ in range(args.steps):
            if (wl.refresh and job.t % wl.refresh == 0) or (not wl.refresh and job.t == 0):
                mines += 1
            b = job.step()
            torch.cuda.synchronize()
            touched_sum += int(job.out["n_touched"].item())
            pairs_sum += job.valid_pairs[b]
        if mines == 0:
            # the schedule mined before the timed steps (one pass over the pool): one more pass here,
            # outside the timed region, so that the mining kernel of this workload is reported too
            job.mine()
            torch.cuda.synchronize()
            mines = 1
        binding.profile_enable(False)
        prof = binding.profile_collect()
        e = 2 if wl.dtype == "bf16" else 4
        row = wl.d * e
        for name, (ms, cnt) in prof.items():
            if cnt:
                kernels[name] = {"avg_us": ms * 1e3 / cnt, "launches": cnt, "total_ms": ms}
        models = {}
        if "mine_tile" in kernels:
            # one mining call sweeps the labels in several launches of the tile kernel (phases);
            # work and time are summed over the launches of the pass, i.e. a launch-time-weighted rate
            flops = 2.0 * wl.d * pool * wl.L * mines
            k = kernels["mine_tile"]
            models["mine_tile"] = {"bound": "mfma", "achieved": flops / (k["total_ms"] * 1e-3) / 1e12,
                                   "peak": PEAK_MFMA_TFLOPS[wl.dtype], "unit": "TFLOP/s",
                                   "launches_per_call": k["launches"] / max(mines, 1)}
        if "gather" in kernels:
            by = pairs_sum / args.steps * row
            k = kernels["gather"]
            models["gather"] = {"bound": "hbm", "achieved": by / (k["avg_us"] * 1e-6) / 1e9,
                                "peak": PEAK_HBM_GBS, "unit": "GB/s"}
        if "update" in kernels:
            by = 2.0 * touched_sum / args.steps * row
            k = kernels["update"]
            models["update"] = {"bound": "hbm", "achieved": by / (k["avg_us"] * 1e-6) / 1e9,
                                "peak": PEAK_HBM_GBS, "unit": "GB/s"}
        traffic = {}
        if os.path.exists(args.traffic_json):
            try:
                traffic = json.load(open(args.traffic_json)).get(wl.name, {})
            except Exception:
                traffic = {}
        for name, m in models.items():
            m["frac"] = m["achieved"] / m["peak"]
            t = traffic.get(name)
            m["traffic"] = t["bytes"] if t else None       # HBM bytes per launch (read + written)
            m["kernel"] = name
            m["avg_us"] = kernels[name]["avg_us"]
        if models:
            dominant = max(models, key=lambda n: kernels[n]["total_ms"])
            roofline = dict(models[dominant])
            roofline["others"] = {n: m for n, m in models.items() if n != dominant}

    result = {
        "metric": "queries/s through xc_step + mining",
        "value": value, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: L=%d d=%d %s B=%d k_p<=%d k_h=%d k_r=%d pool=%d refresh=%d"
                               % (wl.name, wl.L, wl.d, wl.dtype, wl.B, wl.k_p, wl.k_h, wl.k_r, pool, wl.refresh),
                   "loss": "bce",
                   "refresh_search": ("exact, warm start from the previous thresholds (margin %g)" % args.warm_margin)
                                     if args.warm_margin >= 0 else "exact, full search every time"},
        "roofline": roofline,
        "full_search_every_refresh": full_search,
        "kernels_us": {n: round(k["avg_us"], 2) for n, k in kernels.items()},
    }
    # ---- what the chip sustains on two trivial kernels (context for the fractions above) -----
    achievable = {}
    if not args.no_profile_pass:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for rnd in (0, 1):
            binding.mfma_probe(2000, bool(rnd))                     # warm-up
            ev[0].record()
            flop = sum(binding.mfma_probe(4000, bool(rnd)) for _ in range(5))
            ev[1].record()
            torch.cuda.synchronize()
            achievable["mfma_bf16_%s_operands_TFLOPs" % ("random" if rnd else "zero")] = flop / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        binding.copy_probe(b, a)
        ev[2].record()
        for _ in range(5):
            binding.copy_probe(b, a)
        ev[3].record()
        torch.cuda.synchronize()
        achievable["copy_GBs_read_plus_write"] = 5 * 2.0 * a.numel() / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9
        del a, b
    result["achievable"] = achievable

    if "mine_tile" in kernels:
        per_call_ms = (kernels["mine_tile"]["total_ms"] + kernels.get("mine_select", {"total_ms": 0})["total_ms"]) / max(mines, 1)
        result["mine_pairs_per_s"] = pool * wl.L / (per_call_ms * 1e-3)
        result["mine_ms_per_refresh"] = per_call_ms
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, pool)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
