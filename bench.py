#!/usr/bin/env python3
"""Benchmark of the placement search hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
  kvp_score        S schedules of the workload (the dense part)
  kvp_delta_score  one proposed move on each of the first D schedules
  kvp_anneal       M moves on each of C chains (continuing one cooling schedule)
  kvp_best         exact re-score of every chain's best schedule + argmin
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

The default run goes through the four target configurations (Llama-3-8B-shaped,
long context, 70B-shaped GQA, batched serving), each at its own batch size, and
reports for each the scoring kernel's sustained rate (launched back to back),
its rate inside the whole step, the fraction of the HBM peak and the annealing
throughput.  The top-level `value`, `roofline` and `cpu_baseline` are those of
the largest configuration, batched serving (70.9 GB of placements per launch):
`value` is scored token-steps/s of kvp_score launched back to back.
`--workload NAME` runs one configuration only (and makes it the headline).
"""
import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK = 8.0e12          # MI355X HBM3E, bytes/s
GIB = 1 << 30
TARGETS = ["llama8b", "longctx", "gqa70b", "serving"]      # the headline is the last one
# HBM bytes per kvp_score launch (scoring kernel + finalize) from rocprofv3 FETCH_SIZE / WRITE_SIZE, each
# scaled by what the same counter reads for a device copy of 1 GiB; keyed by (workload, S, scorer that ran).
# Any other workload, batch size or kernel choice reports null.  Source: profiles/kvp_score_<workload>.md.
MEASURED_TRAFFIC = {("llama8b", 14564, "quad"): 4.514e9, ("longctx", 1024, "rowblock"): 9.432e9,
                    ("gqa70b", 512, "rowlane"): 11.776e9, ("serving", 512, "line"): 72.046e9}


def algorithmic_bytes(tr, S):
    """Bytes kvp_score has to move: every placement word once, the trace once
    per batch, 12 bytes of results per schedule."""
    Wd = tr.n_words
    return (S * tr.L * tr.N * Wd * 4 + tr.L * tr.N * tr.K * Wd * 4 + 3 * tr.N * Wd * 4 + tr.L * tr.N * 4
            + 12 * S)


def default_schedules(tr):
    per = tr.L * tr.N * tr.n_words * 4
    return max(tr.chains, math.ceil(4 * GIB / per))


def make_batch(tr, S, device, seed=1234):
    """S synthetic schedules on the GPU, [S][L][N][Wd] int32 words: about a
    quarter of the existing pages in HBM, independent bits (the scorer has no
    data-dependent branch).  Seeded torch generator."""
    import torch
    import workloads as W
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    per = tr.L * tr.N * tr.n_words
    alive = torch.from_numpy(W.pack_bits(tr.alive).view(np.int32)).to(device)        # [N][Wd]
    x = torch.empty((S, tr.L, tr.N, tr.n_words), dtype=torch.int32, device=device)
    chunk = max(1, (256 << 20) // (per * 4))
    lo, hi = -(2 ** 31), 2 ** 31 - 1
    for s0 in range(0, S, chunk):
        s1 = min(S, s0 + chunk)
        shape = (s1 - s0, tr.L, tr.N, tr.n_words)
        a = torch.randint(lo, hi, shape, dtype=torch.int32, device=device, generator=g)
        b = torch.randint(lo, hi, shape, dtype=torch.int32, device=device, generator=g)
        x[s0:s1] = a & b & alive
    return x


def upload(K, W, ctx, tr):
    prob = K.make_problem(tr.L, tr.N, tr.P, tr.K, tr.plane_bytes, tr.page_bytes, tr.token_bytes,
                          tr.bw_hbm, tr.bw_link, tr.bw_dram, tr.cap_pages)
    K.kvp_trace_upload(ctx, prob, W.pack_bits(tr.access), W.pack_bits(tr.alive), W.pack_bits(tr.persist),
                       W.pack_bits(tr.written))


def cpu_baseline(tr, X_sample, seconds):
    """The oracle as it stands, timed on the host cores on a bounded sample."""
    from concurrent.futures import ThreadPoolExecutor
    import oracle as O
    q = O.Problem(tr)
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1024")))
    t0 = time.perf_counter()
    O.cost(q, X_sample[0])
    t1 = time.perf_counter() - t0
    n = int(max(cores, min(len(X_sample) * 64, seconds / max(t1, 1e-6))))
    idx = [i % len(X_sample) for i in range(n)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(lambda i: O.cost(q, X_sample[i]), idx))
    wall = time.perf_counter() - t0
    out = {"value": n * tr.N / wall, "unit": "token-steps/s", "cores": cores, "kind": "oracle",
           "one_core_value": tr.N / t1,
           "sample": f"{n} schedule scorings of the {tr.name} workload ({len(X_sample)} distinct schedules drawn "
                     f"from the GPU batch), {n * t1:.0f} s of single-core work spread over {cores} threads"}
    # annealing: one chain per core, a short budget from the empty schedule
    mv = 1500 if tr.L * tr.P < 100000 else 150
    X0 = np.zeros(q.shape, np.uint8)
    t0 = time.perf_counter()
    O.anneal(q, range(cores), X0, threads=cores, seed=tr.seed, total_moves=mv)
    out["anneal_moves_per_s"] = cores * mv / (time.perf_counter() - t0)
    out["anneal_sample"] = f"{cores} chains x {mv} moves, one chain per thread (the initial scoring of each chain included)"
    return out


def run_workload(a, name, headline):
    """Times one configuration; returns its report (and, for the headline, the pieces of the top-level line)."""
    import torch
    import paper_2508_13231_amd as K
    import workloads as W

    dev = torch.device("cuda", 0)
    t_gen = time.perf_counter()
    tr = W.config(name, a.scale)
    t_gen = time.perf_counter() - t_gen
    S = a.schedules or default_schedules(tr)
    C = a.chains or tr.chains
    D = min(a.delta_batch, S)
    M = a.anneal_moves
    total = (a.steps + a.warmup) * M
    ctx = K.kvp_create(0)
    upload(K, W, ctx, tr)
    if a.score_kernel:
        K.kvp_set_score_kernel(ctx, a.score_kernel)
    d_x = make_batch(tr, S, dev)
    d_cost = torch.empty(S, dtype=torch.float64, device=dev)
    d_ex = torch.empty(S, dtype=torch.int32, device=dev)
    alg = algorithmic_bytes(tr, S)

    def timed(fn, reps):
        """Mean, median and minimum duration in ms of `reps` calls enqueued back to back."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        d = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)])
        return float(d.mean()), float(np.median(d)), float(d.min())

    score = lambda: K.kvp_score(ctx, d_x, S, d_cost, d_ex)
    if a.calibrate_copy:
        src = d_x.view(-1)[: GIB // 4]
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del dst
    # ---- kvp_score launched back to back: the sustained rate
    for _ in range(max(a.warmup, 1)):
        score()
    torch.cuda.synchronize()
    reps = max(a.steps, 3)
    sus_ms, sus_med, sus_min = timed(score, reps)
    kernel = K.SCORE_KERNEL_NAMES.get(K.kvp_score_kernel_used(ctx), "?")
    rep = {
        "workload": f"{tr.name} (scale {a.scale:g}): L={tr.L} N={tr.N} P={tr.P} K={tr.K} Wd={tr.n_words}, S={S} schedules "
                    f"({S * tr.L * tr.N * tr.n_words * 4 / GIB:.2f} GiB)",
        "schedules": S, "kernel": kernel, "bytes_per_launch": alg,
        "score_ms": sus_ms, "score_ms_median": sus_med, "score_ms_min": sus_min,
        "token_steps_per_s": S * tr.N / (sus_ms * 1e-3), "layer_steps_per_s": S * tr.N * tr.L / (sus_ms * 1e-3),
        "achieved_GBps": alg / (sus_ms * 1e-3) / 1e9, "frac": alg / (sus_ms * 1e-3) / HBM_PEAK,
        "traffic": None if a.score_kernel else MEASURED_TRAFFIC.get((name, S, kernel)),
        "trace_draw_s": t_gen,
    }
    if a.batch_sweep and name == "gqa70b":
        # the same kernel on batches that do not fill the last round of workgroups
        rep["batch_sweep"] = {}
        for S2 in (S, S + S // 8, S + S // 4):
            x2 = d_x if S2 == S else torch.cat([d_x, d_x[: S2 - S]])
            c2 = torch.empty(S2, dtype=torch.float64, device=dev)
            e2 = torch.empty(S2, dtype=torch.int32, device=dev)
            f = lambda: K.kvp_score(ctx, x2, S2, c2, e2)
            f(); torch.cuda.synchronize()
            ms = timed(f, reps)[0]
            rep["batch_sweep"][str(S2)] = {"score_ms": ms, "frac": algorithmic_bytes(tr, S2) / (ms * 1e-3) / HBM_PEAK}
            del x2, c2, e2
    step_ms = None
    if not a.score_only:
        # ---- the whole step: score, delta, anneal, best
        mv = W.random_moves(tr, D, seed=77)
        d_mv = torch.from_numpy(W.moves_to_records(mv).view(np.int32)).to(dev)
        d_dt = torch.empty(D, dtype=torch.float64, device=dev)
        d_ver = torch.empty(D, dtype=torch.int32, device=dev)
        # step counters and occupancy of the schedules that the moves are priced on: state that a search
        # keeps beside its schedules (the annealer updates its own with every accepted move), so they are
        # resident when the timed region starts, like the schedules themselves
        d_cnt = torch.empty((D, tr.L, tr.N, 4), dtype=torch.int32, device=dev)
        d_occ = torch.empty((D, tr.N), dtype=torch.int32, device=dev)
        K.kvp_score(ctx, d_x, D, d_cost[:D], d_ex[:D], d_cnt, d_occ)
        # every chain starts from the same admissible schedule: the capacity's worth of the most-read pages
        d_start = torch.empty((tr.L, tr.N, tr.n_words), dtype=torch.int32, device=dev)
        K.kvp_baseline(ctx, K.KVP_BASELINE_STATIC, d_start)
        shape_words = (tr.L, tr.N, tr.n_words)
        first = [True]

        def step(ev=None):
            def mark(i):
                if ev is not None:
                    ev[i].record()
            mark(0)
            K.kvp_score(ctx, d_x, S, d_cost, d_ex)
            mark(1)
            K.kvp_delta_score(ctx, d_x, D, d_mv, d_cnt, d_occ, d_dt, d_ver)
            mark(2)
            p = K.make_anneal_params(C, total, moves=M, seed=tr.seed,
                                     init_mode=K.KVP_INIT_BROADCAST if first[0] else K.KVP_INIT_CONTINUE)
            K.kvp_anneal(ctx, p, d_start if first[0] else None)
            first[0] = False
            mark(3)
            K.kvp_best(ctx)                                  # cost and chain of the winner; its schedule stays in HBM
            mark(4)

        for _ in range(a.warmup):
            step()
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(a.steps)]
        t0 = time.perf_counter()
        for i in range(a.steps):
            step(events[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ph = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in events])   # ms
        step_ms = wall * 1e3 / a.steps
        rep["phases_ms"] = {"score": float(ph[:, 0].mean()), "delta": float(ph[:, 1].mean()),
                            "anneal": float(ph[:, 2].mean()), "best": float(ph[:, 3].mean())}
        rep["step_ms"] = step_ms
        rep["interleaved_token_steps_per_s"] = S * tr.N / (float(ph[:, 0].mean()) * 1e-3)
        rep["interleaved_frac"] = alg / (float(ph[:, 0].mean()) * 1e-3) / HBM_PEAK
        rep["chains"], rep["moves_per_step"] = C, M
        rep["moves_per_s"] = C * M / (float(ph[:, 2].mean()) * 1e-3)
        rep["delta_moves_per_s"] = D / (float(ph[:, 1].mean()) * 1e-3)
        # once, outside the timed steps: the same call handing the winner's schedule to the host as well
        t0 = time.perf_counter()
        K.kvp_best(ctx, shape_words)
        rep["best_with_placement_to_host_ms"] = (time.perf_counter() - t0) * 1e3
        del d_mv, d_dt, d_ver, d_cnt, d_occ, d_start
    extra = {}
    if headline:
        extra["step_ms"] = step_ms if step_ms is not None else sus_ms
        if not a.no_cpu_baseline:
            samp = d_x[: min(2 if tr.L * tr.P > 100000 else 8, S)].cpu().numpy().view(np.uint32)
            K.kvp_destroy(ctx)
            ctx = None
            del d_x
            torch.cuda.empty_cache()
            extra["cpu_baseline"] = cpu_baseline(tr, W.unpack_bits(samp, tr.P), a.cpu_seconds)
    if ctx is not None:
        K.kvp_destroy(ctx)
    del d_cost, d_ex
    gc.collect()
    torch.cuda.empty_cache()
    return rep, extra


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="all",
                    help="all (the four target configurations, headline on serving) or one of tiny|llama8b|longctx|"
                         "serving|gqa70b|decode36k")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--schedules", type=int, default=0, help="S (default: the chains of the config, at least 4 GiB of placements)")
    ap.add_argument("--chains", type=int, default=0)
    ap.add_argument("--anneal-moves", type=int, default=2000, help="moves per chain per step")
    ap.add_argument("--delta-batch", type=int, default=16384)
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--score-only", action="store_true", help="time kvp_score alone (for profiling)")
    ap.add_argument("--no-batch-sweep", dest="batch_sweep", action="store_false",
                    help="skip the three batch sizes of the gqa70b workload")
    ap.add_argument("--score-kernel", type=int, default=0, help="kvp_set_score_kernel value (0 = auto)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain device copies of exactly 1 GiB, so that a counter run "
                         "(FETCH_SIZE / WRITE_SIZE) sees a kernel of known traffic to scale by")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU; chains and schedules shard trivially across GPUs "
              "but no multi-GPU path is built.  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    names = TARGETS if a.workload == "all" else [a.workload]
    reports = {}
    head = None
    for i, name in enumerate(names):
        rep, extra = run_workload(a, name, headline=i == len(names) - 1)
        reports[name] = rep
        print(f"bench: {name}: {rep['kernel']} {rep['score_ms']:.3f} ms, {rep['frac']:.3f} of peak", file=sys.stderr, flush=True)
        if extra:
            head = (name, rep, extra)
    name, rep, extra = head
    out = {
        "metric": "scored token-steps/s", "value": rep["token_steps_per_s"], "unit": "token-steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": extra["step_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32+f64",
        "data": "synthetic",
        "config": {"workload": rep["workload"] + ("" if a.score_only else
                                                  f", {rep.get('chains')} chains x {rep.get('moves_per_step')} moves per step, "
                                                  f"delta batch {min(a.delta_batch, rep['schedules'])}"),
                   "schedules": rep["schedules"], "value_is": "kvp_score launched back to back (sustained)"},
        "score_ms": rep["score_ms"], "score_ms_median": rep["score_ms_median"], "score_ms_min": rep["score_ms_min"],
        "layer_steps_per_s": rep["layer_steps_per_s"],
        "roofline": {"bound": "hbm", "achieved": rep["achieved_GBps"], "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": rep["frac"], "traffic": rep["traffic"],
                     "kernel": f"kvp_score ({rep['kernel']} scoring kernel + block-sum finalize)",
                     "bytes_per_launch": rep["bytes_per_launch"]},
        "configs": reports,
    }
    for k in ("phases_ms", "moves_per_s", "delta_moves_per_s", "interleaved_token_steps_per_s", "interleaved_frac"):
        if k in rep:
            out[k] = rep[k]
    if "cpu_baseline" in extra:
        out["cpu_baseline"] = extra["cpu_baseline"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
