#!/usr/bin/env python3
"""Throughput of the ASTRA classifier-layer hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
xc_sample_negatives + xc_step, plus the shortlist search of Alg. 1
(xc_mine_negatives over the whole query pool) whenever the schedule asks for one.
The timed region is the workload's scripted run: it starts with a search from
scratch and repeats the search every `refresh` steps (c2: every 20 steps, the
later ones started from the thresholds of the one before, same result), or, for
the workloads defined as "one mining pass plus N steps" (c3, c4, c5), once per N
steps.  So `value` always contains the mining the workload defines.

`--steps K` times exactly K steps of that schedule from its start (so one search
and K steps when K is below the search period); the share of search per step
then differs from the workload's, and the whole scripted run is timed too and
reported beside it (`scripted_run`).

The default workload is the largest configuration of the baseline file that fits
one GPU: c5 (L = 120 M labels, d = 256, bf16, about 61 GB of classifier rows,
B = 4096, one search over 16 384 queries plus 100 steps).  The smaller
configurations run after it and ride along under `other_workloads`.

Prints ONE JSON line.  `value` is queries/s over the timed region with all inputs
resident in HBM.  `roofline` describes the kernel that takes the most time of the
scripted run, timed with HIP events on its own stream in a second pass over the
same steps (so the event records do not perturb `value`); for the search it is
per call (the launches of one search summed), for the step kernels per launch.
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
HEADLINE = "c5"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0,
                    help="timed steps (default: the workload's scripted run, 100 for c5).  With another number the "
                         "timed region is that many steps of the schedule from its start, one search included, and "
                         "the whole scripted run is timed as well and reported under `scripted_run`")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE, help="tiny, c2, c3, c4 or c5")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads reported under other_workloads (default: c2,c3,c4 when the "
                         "headline workload runs with default steps; 'none' for none)")
    ap.add_argument("--pool", type=int, default=0, help="override the mined query pool size")
    ap.add_argument("--structured", action="store_true",
                    help="structured variant of the inputs: every query is pulled towards its first positive, so "
                         "searches return positives (masked in the step) and shortlists overlap")
    ap.add_argument("--no-structured-line", action="store_true",
                    help="do not add the structured-variant run of the headline workload under `structured`")
    ap.add_argument("--warm-margin", type=float, default=0.1,
                    help="searches after the first of a scripted run start from the thresholds of the one before, "
                         "lowered by this relative margin (xc_mine_negatives_warm: same shortlists); negative: "
                         "every search is a full search")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch the library's plain copy kernel over this many MiB (three times), "
                         "for scaling hardware traffic counters in rocprofv3 --pmc runs")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes per launch / per search from rocprofv3 --pmc runs (replayed, not measured here)")
    return ap.parse_args()


class Job:
    """Device-resident state of one workload and the step function."""

    def __init__(self, wl, pool, device="cuda:0", warm_margin=None, structured=False):
        import torch

        import paper_2409_20156_amd as xc
        from paper_2409_20156_amd import synth
        self.xc, self.torch, self.wl, self.synth = xc, torch, wl, synth
        self.dev = device
        self.pool = pool
        self.W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, wl.L, wl.d, wl.torch_dtype, device)
        self.Zpool = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, pool, wl.d, wl.torch_dtype, device)
        pos = synth.zipf_positives(synth.BASE_SEED, pool, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
        if structured:
            self.Zpool = synth.add_positive_signal(self.Zpool, self.W, pos)
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
        self.period = wl.refresh if wl.refresh else wl.steps      # steps between two searches
        self.warm_margin = warm_margin
        self.restart()

    def restart(self):
        """Back to the start of the scripted run (W keeps what the steps so far made of it)."""
        self.t = 0
        self.searches = {"cold": 0, "warm": 0}

    def mines_at(self, t):
        return t % self.period == 0

    def mine(self, t):
        # the first search of a scripted run is a search from scratch; the later ones of the same run start
        # from the thresholds of the one before (same result)
        cold = t % self.wl.steps == 0 or self.warm_margin is None
        self.xc.mine_negatives(self.Zpool, self.W, self.wl.k_h, workspace=self.mine_ws, out=self.shortlist,
                               warm_margin=None if cold else self.warm_margin)
        self.searches["cold" if cold else "warm"] += 1

    def step(self):
        wl, t = self.wl, self.t
        if self.mines_at(t):
            self.mine(t)
        b = t % self.nbatch
        lo, hi = b * wl.B, (b + 1) * wl.B
        seed = self.synth.step_seed(self.synth.BASE_SEED, wl.config_id, t)
        self.xc.sample_negatives(self.shortlist[lo:hi], wl.k_h, wl.k_r, wl.L, seed, neg=self.neg, logq=self.logq)
        self.xc.xc_step(self.Zpool[lo:hi], self.W, self.pos[lo:hi], self.neg, self.logq, wl.lr,
                        workspace=self.step_ws, out=self.out)
        self.t += 1
        return b


def cpu_baseline(wl, pool, steps_per_search):
    """The oracle as it stands on a bounded sample of about 10-30 s of CPU work, scaled to the timed region (one search per `steps_per_search` steps).

    Search: `nq` queries against the first `Ls` labels (all of them where the float64 matrix stays below
    about 4 GB, else a prefix whose rows are generated on the fly), scaled linearly to pool x L.
    Sampling + step: `nb` queries of a batch, scaled to B; for a label set too large to hold in float64
    the oracle gets the renumbered sub-problem with exactly the rows these pairs use."""
    import numpy as np
    import torch

    from oracle import astra_oracle as orc
    from paper_2409_20156_amd import synth
    nb = min(wl.B, 256 if wl.L * wl.d > (1 << 29) else 512)
    Ls = min(wl.L, (1 << 29) // wl.d)                               # at most 4 GiB of float64
    nq = max(8, min(1024, (1 << 27) // Ls))
    W = synth.make_matrix(synth.BASE_SEED, synth.TAG_W, Ls, wl.d, wl.torch_dtype, "cpu").to(torch.float64).numpy()
    Z = synth.make_matrix(synth.BASE_SEED, synth.TAG_Z, max(nb, nq), wl.d, wl.torch_dtype, "cpu").to(torch.float64).numpy()
    pos = synth.zipf_positives(synth.BASE_SEED, nb, wl.L, wl.zipf_s, wl.count_law, wl.k_p)
    t0 = time.perf_counter()
    sl, _ = orc.mine_negatives(Z[:nq], W, wl.k_h)
    t_mine_pair = (time.perf_counter() - t0) / (nq * Ls)             # seconds per (query, label)
    if Ls == wl.L:
        sl_b = sl[:nb] if nq >= nb else orc.mine_negatives(Z[:nb], W, wl.k_h)[0]
        t0 = time.perf_counter()
        neg, logq = orc.sample_negatives(sl_b, nb, wl.k_h, wl.k_r, wl.L, 1)
        orc.xc_step(Z[:nb], W, pos, neg, logq, wl.lr, storage=wl.dtype)
        t_step_q = (time.perf_counter() - t0) / nb
    else:
        # a shortlist over the whole label range (any distinct ids serve the timing), then the rows in use
        del W
        rng = np.random.default_rng(5)
        sl_b = np.stack([rng.choice(wl.L, size=wl.k_h, replace=False) for _ in range(nb)]).astype(np.int32)
        t0 = time.perf_counter()
        neg, logq = orc.sample_negatives(sl_b, nb, wl.k_h, wl.k_r, wl.L, 1)
        t_sample = time.perf_counter() - t0
        p64, n64 = pos.astype(np.int64), neg.astype(np.int64)
        used = np.unique(np.concatenate([p64[p64 >= 0], n64.reshape(-1)]))
        rows = synth.gaussian_rows_at(synth.BASE_SEED, synth.TAG_W, torch.as_tensor(used), wl.d,
                                      wl.torch_dtype).to(torch.float64).numpy()
        pos_c = np.where(p64 >= 0, np.searchsorted(used, np.maximum(p64, 0)), -1).astype(np.int32)
        neg_c = np.searchsorted(used, n64).astype(np.int32)
        t0 = time.perf_counter()
        orc.xc_step(Z[:nb], rows, pos_c, neg_c, logq, wl.lr, storage=wl.dtype)
        t_step_q = (t_sample + time.perf_counter() - t0) / nb
    period = steps_per_search                                          # as in the timed region of this run
    per_query = t_step_q + t_mine_pair * wl.L * pool / (period * wl.B)
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": 1.0 / per_query, "unit": "queries/s", "cores": cores, "kind": "oracle",
            "sample": "search: %d queries x the first %d of %d labels, scaled linearly to the pool of %d queries x all "
                      "labels, one search per %g steps as in this run's timed region (extrapolated); sampling + step: %d queries of a batch%s, "
                      "scaled to B=%d; numpy float64 oracle, BLAS threads = cores"
                      % (nq, Ls, wl.L, pool, period, nb,
                         "" if Ls == wl.L else " on the renumbered sub-problem holding the rows their pairs use", wl.B),
            "mine_s_per_query_label": t_mine_pair, "step_s_per_query": t_step_q}


def _traffic(path, wl_name):
    """Replayed, not measured in this run: bytes per launch (per search for the tile kernel) from the committed
    rocprofv3 --pmc summaries, with the commit that last changed the file."""
    if not os.path.exists(path):
        return {}, None
    try:
        data = json.load(open(path)).get(wl_name, {})
    except Exception:
        return {}, None
    commit = None
    try:
        commit = subprocess.run(["git", "-C", ROOT, "log", "-1", "--format=%h", "--", path], capture_output=True,
                                text=True, timeout=10).stdout.strip() or None
    except Exception:
        pass
    return data, {"file": os.path.relpath(path, ROOT), "commit": commit, "replayed": True}


def run_workload(args, name, steps=0, warmup=None, structured=False, profile_pass=True):
    """Warm-up, the timed scripted run, and (optionally) the same run again with per-kernel events."""
    import torch

    from paper_2409_20156_amd import binding, synth
    wl = synth.WORKLOADS[name]
    pool = args.pool or wl.pool
    K = steps or wl.steps
    W_ = args.warmup if warmup is None else warmup
    job = Job(wl, pool, warm_margin=args.warm_margin if args.warm_margin >= 0 else None, structured=structured)
    torch.cuda.synchronize()

    for _ in range(W_):                       # includes one search (step 0 of a scripted run)
        job.step()
    torch.cuda.synchronize()
    job.restart()
    t0 = time.perf_counter()
    for _ in range(K):
        job.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    res = {"workload": "%s: L=%d d=%d %s B=%d k_p<=%d k_h=%d k_r=%d pool=%d, one search per %d steps%s"
                       % (wl.name, wl.L, wl.d, wl.dtype, wl.B, wl.k_p, wl.k_h, wl.k_r, pool, job.period,
                          ", structured inputs" if structured else ""),
           "value": wl.B * K / elapsed, "unit": "queries/s", "steps": K, "warmup": W_,
           "ms_per_step": elapsed * 1e3 / K, "searches_in_timed_region": dict(job.searches)}

    kernels, roofline = {}, None
    if profile_pass:
        job.restart()
        binding.profile_reset()
        binding.profile_enable(True)
        touched_sum, pairs_sum, single_sum = 0, 0, 0
        stats = job.step_ws[:4].view(torch.int32)      # rows the gather updated itself (labels with one pair)
        for _ in range(K):
            b = job.step()
            torch.cuda.synchronize()
            touched_sum += int(job.out["n_touched"].item())
            single_sum += int(stats.item())
            pairs_sum += job.valid_pairs[b]
        binding.profile_enable(False)
        prof = binding.profile_collect()
        mines = job.searches["cold"] + job.searches["warm"]
        row = wl.d * (2 if wl.dtype == "bf16" else 4)
        for kname, (ms, cnt) in prof.items():
            if cnt:
                kernels[kname] = {"avg_us": ms * 1e3 / cnt, "launches": cnt, "total_ms": ms}
        traffic, source = _traffic(args.traffic_json, wl.name + ("_structured" if structured else ""))
        models = {}
        if "mine_tile" in kernels and mines:
            # one search sweeps the labels in several launches of the tile kernel; work and time are per search
            k = kernels["mine_tile"]
            ms_call = k["total_ms"] / mines
            t = traffic.get("mine_tile", {})
            models["mine_tile"] = {"bound": "mfma", "achieved": 2.0 * wl.d * pool * wl.L / (ms_call * 1e-3) / 1e12,
                                   "peak": PEAK_MFMA_TFLOPS[wl.dtype], "unit": "TFLOP/s", "per": "search",
                                   "ms": ms_call, "launches_per_search": k["launches"] / mines,
                                   "searches": dict(job.searches),
                                   "traffic": t.get("bytes_per_search"),
                                   "traffic_search_mode": t.get("search_mode"),
                                   "compulsory_bytes": (wl.L + pool) * row + pool * wl.k_h * 8}
        if "gather" in kernels:
            by = (pairs_sum + single_sum) / K * row        # every pair's row read, single-pair rows also written
            k = kernels["gather"]
            models["gather"] = {"bound": "hbm", "achieved": by / (k["avg_us"] * 1e-6) / 1e9, "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "per": "launch", "ms": k["avg_us"] * 1e-3,
                                "traffic": traffic.get("gather", {}).get("bytes"), "algorithmic_bytes": by}
        if "update" in kernels:
            by = 2.0 * (touched_sum - single_sum) / K * row     # rows of labels with several pairs: read and written
            k = kernels["update"]
            models["update"] = {"bound": "hbm", "achieved": by / (k["avg_us"] * 1e-6) / 1e9, "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "per": "launch", "ms": k["avg_us"] * 1e-3,
                                "traffic": traffic.get("update", {}).get("bytes"), "algorithmic_bytes": by}
        for kname, m in models.items():
            m["frac"] = m["achieved"] / m["peak"]
            m["kernel"] = kname
            m["traffic_source"] = source if m["traffic"] is not None else None
        if models:
            dominant = max(models, key=lambda n: kernels[n]["total_ms"])
            roofline = dict(models[dominant])
            roofline["others"] = {n: m for n, m in models.items() if n != dominant}
        if "mine_tile" in kernels and mines:
            per_call_ms = (kernels["mine_tile"]["total_ms"] + kernels.get("mine_select", {"total_ms": 0})["total_ms"]) / mines
            res["mine_pairs_per_s"] = pool * wl.L / (per_call_ms * 1e-3)
            res["mine_ms_per_search"] = per_call_ms
    if profile_pass:
        res["rows_per_step"] = {"touched": touched_sum / K, "updated_in_gather": single_sum / K}
        # the step as a whole against the memory roofline: every pair's row read once, every touched row written once
        # and, unless its label has a single pair, read once more
        step_us = sum(k["total_ms"] for n, k in kernels.items() if n not in ("mine_tile", "mine_select")) * 1e3 / K
        step_bytes = (pairs_sum + 2.0 * touched_sum - single_sum) / K * row
        res["step_hbm"] = {"algorithmic_bytes": step_bytes, "kernels_us": step_us,
                           "achieved_GBs": step_bytes / (step_us * 1e-6) / 1e9,
                           "frac_of_8TBs": step_bytes / (step_us * 1e-6) / 1e9 / PEAK_HBM_GBS}
    res["roofline"] = roofline
    res["kernels_us"] = {n: round(k["avg_us"], 2) for n, k in kernels.items()}
    if K != wl.steps:
        # the timed region above is the K steps that were asked for, with the searches the schedule puts there
        # (one at its start): a different share of search per step than the workload defines.  The workload's
        # whole scripted run, timed the same way, beside it:
        job.restart()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(wl.steps):
            job.step()
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        res["scripted_run"] = {"steps": wl.steps, "value": wl.B * wl.steps / el, "unit": "queries/s",
                               "ms_per_step": el * 1e3 / wl.steps, "searches": dict(job.searches)}
    del job
    torch.cuda.empty_cache()
    return wl, pool, res


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2409_20156_amd as xc
    from paper_2409_20156_amd import binding
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU")
    xc.load_library()

    wl, pool, head = run_workload(args, args.workload, steps=args.steps, structured=args.structured,
                                  profile_pass=not args.no_profile_pass)
    if args.copy_probe_mib:
        a = torch.randint(0, 255, (args.copy_probe_mib << 20,), dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(3):
            binding.copy_probe(b, a)
        torch.cuda.synchronize()
        del a, b

    result = {
        "metric": "queries/s through xc_step + mining",
        "value": head["value"], "unit": "queries/s", "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "loss": "bce",
                   "searches_in_timed_region": head["searches_in_timed_region"],
                   "search": "exact; the first of a scripted run from scratch" +
                             (", later ones from the previous thresholds (margin %g)" % args.warm_margin
                              if args.warm_margin >= 0 else ", every one from scratch")},
        "roofline": head["roofline"],
        "kernels_us": head["kernels_us"],
    }
    for k in ("mine_pairs_per_s", "mine_ms_per_search", "rows_per_step", "step_hbm", "scripted_run"):
        if k in head:
            result[k] = head[k]

    default_run = args.workload == HEADLINE and not args.pool and not args.structured
    if default_run and not args.no_structured_line and not args.no_profile_pass:
        # the structured variant of the same workload (queries pulled towards a positive), beside the i.i.d. run
        _, _, st = run_workload(args, args.workload, structured=True, profile_pass=True)
        result["structured"] = {k: st[k] for k in ("workload", "value", "ms_per_step", "mine_ms_per_search") if k in st}
        if st.get("roofline"):
            result["structured"]["mine_frac"] = (st["roofline"] if st["roofline"]["kernel"] == "mine_tile"
                                                 else st["roofline"]["others"].get("mine_tile", {})).get("frac")
    also = args.also
    if also is None:
        also = "c2,c3,c4" if default_run and not args.no_profile_pass else "none"
    others = {}
    for name in [n for n in also.split(",") if n and n != "none"]:
        _, _, r = run_workload(args, name, profile_pass=not args.no_profile_pass)
        others[name] = r
    if others:
        result["other_workloads"] = others

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

    if not args.no_cpu_baseline:
        n_search = sum(head["searches_in_timed_region"].values())
        result["cpu_baseline"] = cpu_baseline(wl, pool, head["steps"] / max(1, n_search))
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
