"""Differential tests over seeded random shapes: every scorer, the per-slot occupancy, the placement
generators, move pricing and both annealing walks against the CPU oracle, bit for bit.  The fixed cases
of test_gpu_parity.py aim at known boundaries; these look for the ones nobody thought of."""
import numpy as np
import pytest

import oracle as O
import workloads as W
from workloads.traces import Recipe, generate

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from gpu_util import Gpu
    return Gpu


def _random_trace(rng):
    kind = int(rng.integers(0, 3))
    seed = int(rng.integers(1 << 30))
    if kind == 0:       # unstructured: pages born, dying and re-used at random, several writes per step
        K = int(rng.integers(1, 5))
        pb = None if rng.random() < 0.5 else [int(x) * 4096 for x in rng.integers(1, 4, K)]
        return W.random_trace(seed, L=int(rng.choice([1, 2, 3, 5, 8, 24, 40])), N=int(rng.integers(1, 150)),
                              P=int(rng.integers(1, 700)), K=K, plane_bytes=pb, rebirth=bool(rng.random() < 0.7))
    if kind == 1:       # one decoding sequence: rows of 14 to 70 words
        pt = int(rng.choice([1, 2, 4, 8]))
        words = int(rng.integers(14, 70))
        return generate(Recipe("dec", L=int(rng.choice([2, 3, 4, 6, 8, 24, 40, 48, 80])), N=int(rng.integers(1, 140)),
                               page_tokens=pt, prompt_lo=words * 32 * pt, prompt_hi=words * 32 * pt,
                               K=int(rng.choice([1, 1, 2, 3, 8])), top_frac=0.15, sink_tokens=4, recent_tokens=8,
                               cap_frac=float(rng.choice([0.1, 0.3, 0.6])), seed=seed))
    pt = int(rng.choice([4, 16]))                                     # several sequences that end and are replaced
    return generate(Recipe("srv", L=int(rng.choice([2, 4, 8])), N=int(rng.integers(8, 100)), page_tokens=pt,
                           slots=int(rng.integers(2, 6)), prompt_lo=64, prompt_hi=int(rng.integers(128, 2000)),
                           top_frac=0.1, lifetime_mean=float(rng.choice([5.0, 30.0])), cap_frac=0.25, seed=seed))


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_everything_but_the_walk(G, seed):
    import torch
    import paper_2508_13231_amd as K
    from gpu_util import expected_counters
    rng = np.random.default_rng(1000 + seed)
    tr = _random_trace(rng)
    q = O.Problem(tr)
    X = np.concatenate([W.random_placements(tr, 3, seed=seed, density=0.4),
                        W.random_placements(tr, 2, seed=seed + 1, density=0.9, feasible=False)])
    want = [O.score(q, x) for x in X]
    for kernel in (0, 1, 2, 6, 9, 10, 11, 12, 13):                        # 0: the library's own choice
        with G(tr, score_kernel=kernel) as g:
            cost, ex, cnt, occ = g.score(X)
            for s, r in enumerate(want):
                assert cost[s] == r.cost and ex[s] == r.excess, (kernel, s)
                assert (occ[s] == r.occ).all() and (cnt[s].astype(np.uint64) == expected_counters(r, tr, g.unit)).all()
            if kernel:
                continue
            d = torch.full((len(X),), -1, dtype=torch.int32, device=g.dev)
            K.kvp_strict_excess(g.ctx, g.words(X), len(X), d)
            torch.cuda.synchronize()
            assert d.cpu().numpy().view(np.uint32).tolist() == [O.strict_excess(q, x) for x in X]
            if tr.L <= 24:                                                # pages migrating in steps of their choice
                Y = rng.integers(0, tr.L + (seed % 3 == 0), X.shape).astype(np.uint8)
                dc = torch.empty(len(X), dtype=torch.float64, device=g.dev)
                K.kvp_score_slots(g.ctx, g.words(X), g.to_dev(Y), len(X), dc, d)
                torch.cuda.synchronize()
                for s2 in range(len(X)):
                    r2 = O.score_slots(q, X[s2], Y[s2])
                    assert dc[s2].item() == r2.cost and d.cpu().numpy().view(np.uint32)[s2] == r2.excess, ("slots", s2)
            for kind, fn in ((K.KVP_BASELINE_STATIC, O.init_static_frequency), (K.KVP_BASELINE_RECENCY, O.init_recency),
                             (K.KVP_BASELINE_FILL, O.init_static_fill)):
                assert (g.baseline(kind) == fn(q).astype(bool)).all(), kind
            ws, rs = [1, int(rng.integers(1, 12)), 40], [10, int(rng.integers(0, 11)), 3]
            dp = torch.empty((3,) + g.shape_words, dtype=torch.int32, device=g.dev)
            K.kvp_wr_policy(g.ctx, ws, rs, dp)
            torch.cuda.synchronize()
            got = g.unpack(dp.cpu().numpy().view(np.uint32))
            for i in range(3):
                assert (got[i] == O.wr_policy(q, ws[i], rs[i]).astype(bool)).all(), (ws[i], rs[i])
            mv = W.random_moves(tr, len(X), seed=seed)
            dT, verdict = g.delta(X[:3], {k: v[:3] for k, v in mv.items()}, give_counters=True)
            for s in range(3):
                ov, od, _, _, _ = O.delta(q, X[s], {k: int(v[s]) for k, v in mv.items()})
                assert verdict[s] == ov and dT[s] == od, s


@pytest.mark.parametrize("seed", range(10))
def test_random_wide_single_sequence_every_scorer(G, seed):
    """One decoding sequence with rows of 66 to 260 words (the shapes of the segment-walking scorer),
    one to three tiles, up to six masked words at the end of a row and more."""
    import torch
    import paper_2508_13231_amd as K
    from gpu_util import expected_counters
    rng = np.random.default_rng(3000 + seed)
    pt = int(rng.choice([1, 2, 4, 8]))
    words = int(rng.integers(66, 260))
    tr = generate(Recipe("dec", L=int(rng.choice([2, 3, 4, 6, 8])), N=int(rng.integers(1, 200)), page_tokens=pt,
                         prompt_lo=words * 32 * pt, prompt_hi=words * 32 * pt, K=int(rng.choice([1, 1, 2, 3])),
                         top_frac=0.15, sink_tokens=4, recent_tokens=8, cap_frac=float(rng.choice([0.1, 0.3, 0.6])),
                         seed=int(rng.integers(1 << 30))))
    q = O.Problem(tr)
    X = np.concatenate([W.random_placements(tr, 5, seed=seed, density=0.4),
                        W.random_placements(tr, 2, seed=seed + 1, density=0.9, feasible=False)])
    want = [O.score(q, x) for x in X]
    used = set()
    for kernel in (0, 1, 2, 6, 9, 10, 11, 12, 13):
        with G(tr, score_kernel=kernel) as g:
            cost, ex, cnt, occ = g.score(X)
            used.add(K.kvp_score_kernel_used(g.ctx))
            for s, r in enumerate(want):
                assert cost[s] == r.cost and ex[s] == r.excess, (kernel, s)
                assert (occ[s] == r.occ).all() and (cnt[s].astype(np.uint64) == expected_counters(r, tr, g.unit)).all()
            if kernel == 0:
                d = torch.full((len(X),), -1, dtype=torch.int32, device=g.dev)
                K.kvp_strict_excess(g.ctx, g.words(X), len(X), d)
                torch.cuda.synchronize()
                assert d.cpu().numpy().view(np.uint32).tolist() == [O.strict_excess(q, x) for x in X]
    assert K.KVP_SCORE_LINE in used and K.KVP_SCORE_ROWS in used


@pytest.mark.parametrize("seed", range(16))
def test_random_shape_walks(G, seed):
    """Serial and four-per-round annealing both walk as the oracle does: same schedules, costs and tallies."""
    import paper_2508_13231_amd as K
    rng = np.random.default_rng(2000 + seed)
    if seed % 2:
        pt = int(rng.choice([1, 4, 16]))
        prompt = int(rng.integers(4, 60)) * pt * 8
        slots = 1 if seed % 4 == 1 else int(rng.integers(2, 5))
        tr = generate(Recipe("t", L=int(rng.choice([2, 4, 8])), N=int(rng.integers(4, 100)), page_tokens=pt, slots=slots,
                             prompt_lo=prompt // 2 + pt, prompt_hi=prompt + pt, K=int(rng.choice([1, 2, 8])), top_frac=0.15,
                             sink_tokens=4, recent_tokens=8, lifetime_mean=0.0 if slots == 1 else 20.0,
                             cap_frac=float(rng.choice([0.1, 0.3, 0.6])), seed=int(rng.integers(1 << 30))))
    else:
        tr = W.random_trace(int(rng.integers(1 << 30)), L=int(rng.choice([1, 2, 3, 5])), N=int(rng.integers(2, 90)),
                            P=int(rng.integers(2, 200)), K=int(rng.integers(1, 4)), rebirth=bool(rng.random() < 0.7))
    q = O.Problem(tr)
    total, chains = int(rng.choice([300, 1000, 2500])), 3
    max_len, sa_seed = int(rng.choice([1, 7, 63])), int(rng.integers(1 << 40))
    X0 = [np.zeros(q.shape, np.uint8), O.init_static_frequency(q), O.init_recency(q)][int(rng.integers(0, 3))]
    res, _ = O.anneal(q, range(chains), X0, seed=sa_seed, total_moves=total, max_len=max_len)
    for lookahead in (1, 4):
        with G(tr) as g:
            K.kvp_set_anneal_lookahead(g.ctx, lookahead)
            p = K.make_anneal_params(chains, total, seed=sa_seed, init_mode=K.KVP_INIT_BROADCAST, max_len=max_len)
            K.kvp_anneal(g.ctx, p, g.words(X0))
            _, _, _, cc = K.kvp_best(g.ctx, g.shape_words, chains)
            stats = K.kvp_chain_stats(g.ctx, chains)
            for c in range(chains):
                cur = g.unpack(K.kvp_chain_placement(g.ctx, c, 0, g.shape_words))
                assert (cur == res[c].X).all() and cc[c] == res[c].best_cost, (lookahead, c)
                assert stats[c].accepted == res[c].accepted and stats[c].null_moves == res[c].null_moves
    # the same under the capacity read at every inference step, from a start that fits every slot
    if O.strict_excess(q, X0) != 0:
        X0 = O.init_static_frequency(q)
    res, _ = O.anneal(q, range(chains), X0, seed=sa_seed, total_moves=total, max_len=max_len, per_slot=True)
    with G(tr) as g:
        K.kvp_set_capacity_mode(g.ctx, K.KVP_CAPACITY_PER_SLOT)
        p = K.make_anneal_params(chains, total, seed=sa_seed, init_mode=K.KVP_INIT_BROADCAST, max_len=max_len)
        K.kvp_anneal(g.ctx, p, g.words(X0))
        _, _, _, cc = K.kvp_best(g.ctx, g.shape_words, chains)
        stats = K.kvp_chain_stats(g.ctx, chains)
        for c in range(chains):
            cur = g.unpack(K.kvp_chain_placement(g.ctx, c, 0, g.shape_words))
            assert (cur == res[c].X).all() and cc[c] == res[c].best_cost, ("per slot", c)
            assert stats[c].accepted == res[c].accepted and stats[c].null_moves == res[c].null_moves
            assert O.strict_excess(q, cur) == 0
