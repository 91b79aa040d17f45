#!/usr/bin/env python3
"""Benchmark of the placement search hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
  kvp_score        S schedules of the workload (the dense part)
  kvp_delta_score  one proposed move on each of the first D schedules
  kvp_anneal       M moves on each of C chains (continuing one cooling schedule)
  kvp_best         exact re-score of every chain's best schedule + argmin
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

`value` is scored token-steps/s of kvp_score (S*N / its mean duration);
annealing throughput is reported next to it as `moves_per_s`.
"""
import argparse
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
# HBM bytes per kvp_score launch on the default workload with the default kernel, from rocprofv3
# FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB device copy (profiles/kvp_bench_llama8b.md).
# Any other workload, batch size or kernel choice reports null.
MEASURED_TRAFFIC = {("llama8b", 1.0, 14564): 4.514e9}


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
           "sample": f"{n} schedule scorings of the same workload ({len(X_sample)} distinct schedules drawn "
                     f"from the GPU batch), {n * t1:.0f} s of single-core work spread over {cores} threads"}
    # annealing: one chain per core, a short budget
    mv = 1500
    X0 = np.zeros(q.shape, np.uint8)
    t0 = time.perf_counter()
    O.anneal(q, range(cores), X0, threads=cores, seed=tr.seed, total_moves=mv)
    out["anneal_moves_per_s"] = cores * mv / (time.perf_counter() - t0)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama8b", help="tiny|llama8b|longctx|serving|gqa70b (the benchmark list), decode36k")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--schedules", type=int, default=0, help="S (default: >= 4 GiB of placements)")
    ap.add_argument("--chains", type=int, default=0)
    ap.add_argument("--anneal-moves", type=int, default=2000, help="moves per chain per step")
    ap.add_argument("--delta-batch", type=int, default=16384)
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--score-only", action="store_true", help="time kvp_score alone (for profiling)")
    ap.add_argument("--score-kernel", type=int, default=0, help="kvp_set_score_kernel value (0 = auto)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain device copies of exactly 1 GiB, so that a counter run "
                         "(FETCH_SIZE / WRITE_SIZE) sees a kernel of known traffic to scale by")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU; chains and schedules shard trivially across GPUs "
              "but no multi-GPU path is built.  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2508_13231_amd as K
    import workloads as W

    dev = torch.device("cuda", 0)
    tr = W.config(a.workload, a.scale)
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
    mv = W.random_moves(tr, D, seed=77)
    d_mv = torch.from_numpy(W.moves_to_records(mv).view(np.int32)).to(dev)
    d_dt = torch.empty(D, dtype=torch.float64, device=dev)
    d_ver = torch.empty(D, dtype=torch.int32, device=dev)
    # step counters and occupancy of the schedules that the moves are priced on: state that a search
    # keeps beside its schedules (the annealer updates its own with every accepted move), so they are
    # resident when the timed region starts, like the schedules themselves
    d_cnt = torch.empty((D, tr.L, tr.N, 4), dtype=torch.int32, device=dev)
    d_occ = torch.empty((D, tr.N), dtype=torch.int32, device=dev)
    if not a.score_only:
        # (in two launches of other sizes than the timed one, so that a profile lists them on rows of their own)
        h = D // 2
        for lo, hi in ((0, h), (h, D)):
            if hi > lo:
                K.kvp_score(ctx, d_x[lo:hi], hi - lo, d_cost[lo:hi], d_ex[lo:hi], d_cnt[lo:hi], d_occ[lo:hi])
    start = W.random_placements(tr, 1, seed=tr.seed, density=0.25)[0]
    d_start = torch.from_numpy(W.pack_bits(start).view(np.int32)).to(dev)
    shape_words = (tr.L, tr.N, tr.n_words)

    first = [True]

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        K.kvp_score(ctx, d_x, S, d_cost, d_ex)
        mark(1)
        if a.score_only:
            return
        K.kvp_delta_score(ctx, d_x, D, d_mv, d_cnt, d_occ, d_dt, d_ver)
        mark(2)
        p = K.make_anneal_params(C, total, moves=M, seed=tr.seed,
                                 init_mode=K.KVP_INIT_BROADCAST if first[0] else K.KVP_INIT_CONTINUE)
        K.kvp_anneal(ctx, p, d_start if first[0] else None)
        first[0] = False
        mark(3)
        K.kvp_best(ctx, shape_words)
        mark(4)

    if a.calibrate_copy:
        src = d_x.view(-1)[: GIB // 4]
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del dst
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    nev = 2 if a.score_only else 5
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(a.steps)]
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ph = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(nev - 1)] for e in events])   # ms
    score_ms = float(ph[:, 0].mean())
    alg = algorithmic_bytes(tr, S)
    achieved = alg / (score_ms * 1e-3)
    out = {
        "metric": "scored token-steps/s", "value": S * tr.N / (score_ms * 1e-3), "unit": "token-steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": wall * 1e3 / a.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32+f64",
        "data": "synthetic",
        "config": {"workload": f"{tr.name} (scale {a.scale:g}): L={tr.L} N={tr.N} P={tr.P} K={tr.K} "
                               f"Wd={tr.n_words}, S={S} schedules ({S * tr.L * tr.N * tr.n_words * 4 / GIB:.2f} GiB), "
                               f"{C} chains x {M} moves per step, delta batch {D}",
                   "schedules": S, "chains": C, "moves_per_step": M},
        "score_ms": score_ms, "score_ms_median": float(np.median(ph[:, 0])), "score_ms_min": float(ph[:, 0].min()),
        "layer_steps_per_s": S * tr.N * tr.L / (score_ms * 1e-3),
        "roofline": {"bound": "hbm", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK,
                     "traffic": None if a.score_kernel else MEASURED_TRAFFIC.get((a.workload, a.scale, S)),
                     "kernel": "kvp_score (score kernel + block-sum finalize)", "bytes_per_launch": alg},
    }
    if not a.score_only:
        out["phases_ms"] = {"score": score_ms, "delta": float(ph[:, 1].mean()), "anneal": float(ph[:, 2].mean()),
                            "best": float(ph[:, 3].mean())}
        out["moves_per_s"] = C * M / (float(ph[:, 2].mean()) * 1e-3)
        out["delta_moves_per_s"] = D / (float(ph[:, 1].mean()) * 1e-3)
    if not a.no_cpu_baseline and not a.score_only:
        samp = d_x[: min(8, S)].cpu().numpy().view(np.uint32)
        out["cpu_baseline"] = cpu_baseline(tr, W.unpack_bits(samp, tr.P), a.cpu_seconds)
    K.kvp_destroy(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
