#!/usr/bin/env python3
"""Placement strategies side by side on synthetic traces, in the manner of the
paper's evaluation (Sec. IV): tokens/s normalised to the static placement
across attention sparsity, tokens/s normalised to unlimited HBM and the HBM hit
rate under low and high variation of token importance.

    python -m paper_2508_13231_amd.report            # 4096-token prompt, 256 decode steps, 32 layers
    python -m paper_2508_13231_amd.report --quick    # a small shape, seconds
    python -m paper_2508_13231_amd.report --config longctx   # one of the benchmark workloads instead

Everything runs on the GPU through the library; the traces are synthetic (the
paper's are recorded attention of LLaMA-3.1-8B on NarrativeQA), so the numbers
show how the strategies relate on these traces, not the paper's figures.

Strategies (Sec. IV-A), all scored by kvp_score on the same token-level trace:
  unlimited   every entry in HBM, capacity ignored
  static      kvp_baseline FILL: entries stay where they were first written
  reactive    kvp_baseline RECENCY: the pool holds the most recently read entries
  page-16     pages of 16 tokens placed by the best (W, R) look-ahead policy, a
              page read whole when any of its tokens is needed
  page-16/t   the same placement unit, reads priced per token
  SA-guided   tokens placed by the best (W, R) policy (kvp_wr_search), refined by
              the direct search (kvp_anneal) started from it
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2508_13231_amd as K  # noqa: E402
import workloads as W  # noqa: E402


def token_trace(sparsity, phi, sigma, shape, seed):
    """One decoding sequence at token granularity: every step reads the top
    (1 - sparsity) share of the tokens by an AR(1) importance score, plus four
    sink tokens and the last eight."""
    L, N, prompt = shape
    return W.generate(W.Recipe("tok", L=L, N=N, page_tokens=1, prompt_lo=prompt, prompt_hi=prompt,
                               top_frac=1.0 - sparsity, sink_tokens=4, recent_tokens=8, phi=phi, sigma=sigma,
                               cap_frac=0.30, bw_hbm=4.0e12, bw_link=0.5e12, bw_dram=0.5e12, seed=seed))


class Session:
    """A trace resident on the GPU and the few calls the report needs."""

    def __init__(self, tr):
        import torch
        self.torch, self.tr = torch, tr
        self.dev = torch.device("cuda", 0)
        self.ctx = K.kvp_create(0)
        prob = K.make_problem(tr.L, tr.N, tr.P, tr.K, tr.plane_bytes, tr.page_bytes, tr.token_bytes,
                              tr.bw_hbm, tr.bw_link, tr.bw_dram, tr.cap_pages)
        K.kvp_trace_upload(self.ctx, prob, W.pack_bits(tr.access), W.pack_bits(tr.alive), W.pack_bits(tr.persist),
                           W.pack_bits(tr.written))
        self.shape = (tr.L, tr.N, tr.n_words)
        self.read_bytes = float(sum(int(tr.access[:, :, k, :].sum()) * tr.plane_bytes[k] for k in range(tr.K)))

    def close(self):
        K.kvp_destroy(self.ctx)

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def empty(self):
        return self.torch.empty(self.shape, dtype=self.torch.int32, device=self.dev)

    def measure(self, d_x):
        """(total latency, HBM hit rate, excess) of one schedule on the device."""
        t = self.torch
        cost = t.empty(1, dtype=t.float64, device=self.dev)
        ex = t.empty(1, dtype=t.int32, device=self.dev)
        cnt = t.empty((1, self.tr.L, self.tr.N, 4), dtype=t.int32, device=self.dev)
        K.kvp_score(self.ctx, d_x, 1, cost, ex, cnt)
        t.cuda.synchronize()
        hit = float(cnt[0, :, :, 0].sum(dtype=t.int64)) * K.kvp_plane_unit(self.ctx) / max(self.read_bytes, 1.0)
        return float(cost[0]), hit, int(ex[0]) & 0x7FFFFFFF

    def unlimited(self):
        x = np.broadcast_to(self.tr.alive[None], (self.tr.L, self.tr.N, self.tr.P)).copy()
        return self.measure(self.torch.from_numpy(W.pack_bits(x).view(np.int32)).to(self.dev))[:2]

    def baseline(self, kind):
        d = self.empty()
        K.kvp_baseline(self.ctx, kind, d)
        T, hit, ex = self.measure(d)
        assert ex == 0
        return T, hit

    def policy_search(self, w_max, refine_moves=0, chains=64, p0=0.005):
        """Best (W, R) look-ahead policy; optionally refined by the direct search from its schedule.
        The refinement starts cold (p0 = 0.005: few uphill moves are accepted): from a schedule this
        good, the paper's start temperature (p0 = 0.8) walks away from it and a budget of 1e5 moves per
        chain does not find the way back."""
        d = self.empty()
        res, _ = K.kvp_wr_search(self.ctx, w_max=w_max, total_moves=2000, n_levels=20, seed=1, stop_rel=0.0,
                                 c_min_frac=0.0, d_best_placement=d)
        T, hit, ex = self.measure(d)
        assert ex == 0 and T == res.best_T
        out = {"T": T, "hit": hit, "W": res.best_w, "R": res.best_r10 / 10, "placement": d}
        if refine_moves:
            p = K.make_anneal_params(chains, refine_moves, seed=7, init_mode=K.KVP_INIT_BROADCAST, p0=p0)
            K.kvp_anneal(self.ctx, p, d)
            cost, _, placement, _ = K.kvp_best(self.ctx, self.shape)
            if cost < T:
                d2 = self.torch.from_numpy(np.ascontiguousarray(placement).view(np.int32)).to(self.dev)
                T2, hit2, ex2 = self.measure(d2.reshape(self.shape))
                assert ex2 == 0 and T2 == cost
                out.update(T=T2, hit=hit2, refined=True)
        return out


def migrations_moved(tr, d_x, chains=16, proposals=400000):
    """The schedule d_x with its migrations moved into other layers' inference steps (kvp_refine_slots).  The
    capacity is counted after every inference step there, so it is first raised by what the schedule's pool
    exceeds it between two layers.  Returns (T, pages added to the capacity, seconds)."""
    import dataclasses
    import torch
    dev = d_x.device
    with Session(tr) as s:
        y0 = torch.zeros((1, tr.L, tr.N, tr.P), dtype=torch.uint8, device=dev)
        c, e = torch.empty(1, dtype=torch.float64, device=dev), torch.empty(1, dtype=torch.int32, device=dev)
        K.kvp_score_slots(s.ctx, d_x, y0, 1, c, e)
        torch.cuda.synchronize()
        over = int(e.item()) & 0x3FFFFFFF
    with Session(dataclasses.replace(tr, cap_pages=tr.cap_pages + over)) as s:
        t0 = time.perf_counter()
        d_y = torch.empty((chains, tr.L, tr.N, tr.P), dtype=torch.uint8, device=dev)
        p = K.make_anneal_params(chains, proposals, seed=2, init_mode=K.KVP_INIT_EMPTY)
        K.kvp_refine_slots(s.ctx, p, d_x, d_y)
        c, e = torch.empty(chains, dtype=torch.float64, device=dev), torch.empty(chains, dtype=torch.int32, device=dev)
        K.kvp_score_slots(s.ctx, d_x.unsqueeze(0).expand(chains, -1, -1, -1).contiguous(), d_y, chains, c, e)
        torch.cuda.synchronize()
        assert int(e.max().item()) == 0
        return float(c.min().item()), over, time.perf_counter() - t0


def evaluate(tok, w_max, refine_moves, chains):
    """Every strategy on one token-level trace: name -> (T, hit rate)."""
    rows = {}
    with Session(tok) as s:
        rows["unlimited"] = s.unlimited()
        rows["static"] = s.baseline(K.KVP_BASELINE_FILL)
        rows["reactive"] = s.baseline(K.KVP_BASELINE_RECENCY)
        r = s.policy_search(w_max, refine_moves, chains)
        rows["SA-guided"] = (r["T"], r["hit"])
        note = f"W={r['W']} R={r['R']:.1f}" + (" +direct" if r.get("refined") else "")
    for name, reads in (("page-16", "page"), ("page-16/t", "token")):
        with Session(W.regroup(tok, 16, reads)) as s:
            r = s.policy_search(w_max)
            rows[name] = (r["T"], r["hit"])
    return rows, note


ORDER = ["unlimited", "static", "reactive", "page-16", "page-16/t", "SA-guided"]


def config_row(name, w_max):
    """The named benchmark workload (pages as the trace has them): total decode latency of each
    strategy, the search refined by the workload's own chains and move budget."""
    tr = W.config(name)
    with Session(tr) as s:
        out = {"unlimited": s.unlimited(), "fill": s.baseline(K.KVP_BASELINE_FILL),
               "by frequency": s.baseline(K.KVP_BASELINE_STATIC), "recency": s.baseline(K.KVP_BASELINE_RECENCY)}
        t0 = time.perf_counter()
        r = s.policy_search(w_max)
        t1 = time.perf_counter()
        out[f"(W,R) policy, W={r['W']} R={r['R']:.1f} ({t1 - t0:.2f} s)"] = (r["T"], r["hit"])
        policy_x = r["placement"].clone()
        r2 = s.policy_search(w_max, refine_moves=tr.moves, chains=tr.chains)
        out[f"direct search from it, {tr.chains} chains x {tr.moves} moves, p0 = 0.005 ({time.perf_counter() - t1:.2f} s)"] = (r2["T"], r2["hit"])
        t2 = time.perf_counter()
        r3 = s.policy_search(w_max, refine_moves=tr.moves, chains=tr.chains, p0=0.8)
        out[f"the same with the paper's p0 = 0.8 ({time.perf_counter() - t2:.2f} s)"] = (r3["T"], r3["hit"])
    Tm, over, secs = migrations_moved(tr, policy_x)
    out[f"the policy's schedule, its migrations moved into other layers' steps (HBM for {over} pages more, the pool "
        f"counted after every inference step; 16 chains x 400000 proposals, {secs:.2f} s)"] = (Tm, r["hit"])
    print(f"{name}: L={tr.L} N={tr.N} P={tr.P} K={tr.K}, HBM for {tr.cap_pages} pages\n")
    print("| strategy | total decode latency T (s) | HBM hit rate |")
    print("|---|---|---|")
    for k, (T, hit) in out.items():
        print(f"| {k} | {T:.6e} | {hit:.1%} |")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--quick", action="store_true")
    ap.add_argument("--w-max", type=int, default=32)
    ap.add_argument("--refine-moves", type=int, default=20000, help="direct-search moves per chain (0: none)")
    ap.add_argument("--chains", type=int, default=64)
    ap.add_argument("--config", default=None, help="one of the benchmark workloads instead of the sweeps: "
                                                   "tiny | llama8b | longctx | serving | gqa70b")
    a = ap.parse_args()
    if a.config:
        config_row(a.config, a.w_max)
        return
    shape = (4, 64, 1024) if a.quick else (32, 256, 4096)
    print(f"shape: {shape[0]} layers, {shape[1]} decode steps, prompt of {shape[2]} tokens; HBM holds 30 % of the "
          f"entries; HBM : link : DRAM = 8 : 1 : 1\n")

    print("tokens/s normalised to the static placement, by attention sparsity (importance AR(1) 0.9 / 0.7)\n")
    print("| sparsity | " + " | ".join(ORDER) + " | best policy |")
    print("|---|" + "---|" * (len(ORDER) + 1))
    for sp in (0.5, 0.6, 0.7, 0.8, 0.9, 0.95):
        t0 = time.perf_counter()
        rows, note = evaluate(token_trace(sp, 0.9, 0.7, shape, seed=11), a.w_max, a.refine_moves, a.chains)
        base = rows["static"][0]
        print(f"| {sp:.0%} | " + " | ".join(f"{base / rows[k][0]:.2f}" for k in ORDER) + f" | {note} |", flush=True)
        print(f"  (sparsity {sp:.0%}: {time.perf_counter() - t0:.1f} s)", file=sys.stderr, flush=True)

    print("\ntokens/s normalised to unlimited HBM and HBM hit rate at 60 % sparsity, by variation of token importance\n")
    print("| variation | " + " | ".join(k for k in ORDER[1:]) + " |")
    print("|---|" + "---|" * (len(ORDER) - 1))
    for label, phi, sigma in (("low (AR(1) 0.99)", 0.99, 0.2), ("high (AR(1) 0.3)", 0.3, 1.0)):
        rows, note = evaluate(token_trace(0.6, phi, sigma, shape, seed=12), a.w_max, a.refine_moves, a.chains)
        unl = rows["unlimited"][0]
        print(f"| {label}: tokens/s | " + " | ".join(f"{unl / rows[k][0]:.2f}" for k in ORDER[1:]) + " |")
        print(f"| {label}: hit rate | " + " | ".join(f"{rows[k][1]:.0%}" for k in ORDER[1:]) + " |", flush=True)


if __name__ == "__main__":
    main()
