"""Placements whose pages migrate in any inference step between their uses (a second plane Y of bytes): the
scorer and the annealing over Y against the oracle, bit for bit, through the C boundary."""
import dataclasses

import numpy as np
import pytest

import oracle as O
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from gpu_util import Gpu
    return Gpu


def _cases():
    from test_gpu_parity import CASES
    named = dict(CASES)
    yield "tiny", W.config("tiny")                                       # one layer: Y can only be 0
    yield "table1", named["table1"]
    yield "llama8b/8", W.config("llama8b", 0.125)
    yield "gqa70b/16", W.config("gqa70b", 0.0625)                        # 8 planes, 5 layers
    yield "serving/16", W.config("serving", 0.0625)                      # sequences that end and are replaced
    yield "tok-p16", named["tok-p16"]                                    # five weight planes
    yield "rand-tiles", named["rand-tiles"]                              # pages born, dying, re-used
    yield "rand-L16", named["rand-L16"]
    yield "rand-L70", W.random_trace(41, L=70, N=24, P=50, K=2)          # more layers than lanes: ranges of up to 69 steps
    yield "rand-wide", W.random_trace(43, L=4, N=300, P=8000, K=1)       # 300 000 schedule words: the list of migrating pages is scanned in 293 blocks


CASES = list(_cases())


def _score_slots_gpu(g, X, Y):
    import torch
    import paper_2508_13231_amd as K
    S = len(X)
    d_y = g.to_dev(np.ascontiguousarray(Y, dtype=np.uint8))
    d_cost = torch.full((S,), -1.0, dtype=torch.float64, device=g.dev)
    d_ex = torch.full((S,), -1, dtype=torch.int32, device=g.dev)
    K.kvp_score_slots(g.ctx, g.words(X), d_y, S, d_cost, d_ex)
    torch.cuda.synchronize()
    return d_cost.cpu().numpy(), d_ex.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("name,tr", CASES, ids=[c[0] for c in CASES])
def test_score_slots_matches_oracle_bit_for_bit(G, name, tr):
    rng = np.random.default_rng(len(name))
    q = O.Problem(tr)
    X = np.concatenate([W.random_placements(tr, 3, seed=5, density=0.4),
                        W.random_placements(tr, 2, seed=6, density=0.9, feasible=False)])
    X[4] |= 1                                                            # bits on pages that do not exist, too
    Y = rng.integers(0, tr.L, X.shape).astype(np.uint8)
    Y[0] = 0                                                             # every page in its own step
    Y[3] = rng.integers(0, 256, X.shape[1:]).astype(np.uint8)            # values out of range among them
    want = [O.score_slots(q, x, y) for x, y in zip(X, Y)]
    with G(tr) as g:
        cost, ex = _score_slots_gpu(g, X, Y)
        for s, r in enumerate(want):
            assert cost[s] == r.cost and ex[s] == r.excess, (name, s, cost[s], r.cost, hex(ex[s]), hex(r.excess))
        # Y = 0 is the schedule of kvp_score, and its pool is the one of kvp_strict_excess
        plain = g.score(X[:1], counters=False)
        assert cost[0] == plain[0][0]
    if tr.L > 1:
        zero = np.zeros_like(X[1])
        assert any((want[s].slot_t != O.score_slots(q, X[s], zero).slot_t).any() for s in (1, 2)), "Y changed nothing: nothing tested"
        assert (want[3].excess & 0x40000000) != 0


def _walk_start(q, tr, seed):
    """A placement that migrates and fits every inference step: where a walk under the per-slot capacity ends."""
    X0 = O.init_static_frequency(q)
    return O.anneal_chain(q, 0, X0, seed=seed, total_moves=2500, n_levels=10, max_len=15, per_slot=True).X


@pytest.mark.parametrize("name,tr", [c for c in CASES if c[0] in ("table1", "llama8b/8", "gqa70b/16", "serving/16", "rand-tiles", "rand-L70", "rand-wide")],
                         ids=lambda v: v if isinstance(v, str) else "")
def test_refine_slots_walks_like_the_oracle(G, name, tr):
    import torch
    import paper_2508_13231_amd as K
    if name == "rand-tiles":
        tr = dataclasses.replace(tr, cap_pages=20)
    if name == "rand-L70":
        tr = dataclasses.replace(tr, cap_pages=200)                   # a pool that fills: moves get blocked
    q = O.Problem(tr)
    if name == "rand-wide":
        # where a walk that counts the pool per token step ends (the oracle's per-slot walk takes minutes here),
        # and a pool just large enough for it at every inference step
        X = O.anneal_chain(q, 0, O.init_static_frequency(q), seed=3, total_moves=2500, n_levels=10).X
        tr = dataclasses.replace(tr, cap_pages=int(O.score_slots(q, X, np.zeros_like(X)).pool.max()))
        q = O.Problem(tr)
    else:
        X = _walk_start(q, tr, 3)
    chains, total = 3, 4000
    want = [O.refine_slots(q, c, X, np.zeros_like(X), seed=77, total_moves=total, n_levels=10) for c in range(chains)]
    assert sum(r.accepted for r in want) > 10, "nothing migrates in this start: nothing tested"
    with G(tr) as g:
        d_x = g.words(X[None])[0].contiguous()
        d_y = torch.full((chains,) + X.shape, 255, dtype=torch.uint8, device=g.dev)
        p = K.make_anneal_params(chains, total, seed=77, n_levels=10, init_mode=K.KVP_INIT_EMPTY)
        stats = K.kvp_refine_slots(g.ctx, p, d_x, d_y)
        Yg = d_y.cpu().numpy()
        for c in range(chains):
            assert (Yg[c] == want[c].Y).all(), (name, c)
            assert stats[c].t_cur == want[c].T_cur and stats[c].t_best == want[c].T_best and stats[c].c0 == want[c].C0
            assert (stats[c].accepted, stats[c].uphill, stats[c].null_moves, stats[c].clipped, stats[c].improved) == \
                   (want[c].accepted, want[c].uphill, want[c].null_moves, want[c].clipped, want[c].improved)
            assert stats[c].moves_done == total
        # the final schedules fit every inference step, and their running cost is their cost
        cost, ex = _score_slots_gpu(g, np.broadcast_to(X, (chains,) + X.shape), Yg)
        assert (ex == 0).all()
        for c in range(chains):
            assert cost[c] == O.score_slots(q, X, Yg[c]).cost
            assert stats[c].t_cur == pytest.approx(cost[c], rel=1e-12)
            assert cost[c] <= O.cost(q, X) * (1 + 1e-12) or want[c].uphill > 0
        # carried on from given starts: the second half of a schedule twice as long, started where the first ended
        p2 = K.make_anneal_params(chains, total, moves=1000, seed=78, n_levels=10, init_mode=K.KVP_INIT_GIVEN)
        stats2 = K.kvp_refine_slots(g.ctx, p2, d_x, d_y)
        for c in range(chains):
            w2 = O.refine_slots(q, c, X, Yg[c], seed=78, total_moves=total, n_levels=10, move_end=1000)
            assert (d_y[c].cpu().numpy() == w2.Y).all() and stats2[c].t_cur == w2.T_cur and stats2[c].accepted == w2.accepted


def test_refine_slots_refuses_bad_starts_and_arguments(G):
    import torch
    import paper_2508_13231_amd as K
    tr = W.config("llama8b", 0.125)
    q = O.Problem(tr)
    # a placement that fits every token step as a whole and overfills an inference step in between
    bad = O.anneal(q, range(1), O.init_static_frequency(q), seed=5, total_moves=2500)[0][0].X
    assert O.score(q, bad).excess == 0 and O.strict_excess(q, bad) > 0
    good = _walk_start(q, tr, 3)
    with G(tr) as g:
        d_y = torch.zeros((2,) + good.shape, dtype=torch.uint8, device=g.dev)
        p = K.make_anneal_params(2, 100, seed=1, init_mode=K.KVP_INIT_EMPTY)
        with pytest.raises(K.KvpError) as e:
            K.kvp_refine_slots(g.ctx, p, g.words(bad[None])[0].contiguous(), d_y)
        assert e.value.code == K.KVP_EINFEASIBLE
        d_y[1, 0, 1, :] = tr.L                                          # a Y out of range on some migrating page
        Yh = d_y.cpu().numpy()
        pg = K.make_anneal_params(2, 100, seed=1, init_mode=K.KVP_INIT_GIVEN)
        if O.score_slots(q, good, Yh[1]).excess & 0x40000000:
            with pytest.raises(K.KvpError) as e:
                K.kvp_refine_slots(g.ctx, pg, g.words(good[None])[0].contiguous(), d_y)
            assert e.value.code == K.KVP_EINFEASIBLE
        for kw in (dict(moves=101), dict(init_mode=K.KVP_INIT_CONTINUE), dict(p0=1.0)):
            pb = K.make_anneal_params(2, 100, seed=1, **{"init_mode": K.KVP_INIT_EMPTY, **kw})
            with pytest.raises(K.KvpError) as e:
                K.kvp_refine_slots(g.ctx, pb, g.words(good[None])[0].contiguous(), d_y)
            assert e.value.code == K.KVP_EINVAL


@pytest.mark.timeout(600)
def test_full_size_slots_on_config_1(G):
    """Config 1 at its full size: sampled schedules of a batch against the oracle, and sampled chains of a walk."""
    import torch
    import paper_2508_13231_amd as K
    from test_gpu_parity import _full_trace
    tr, q = _full_trace("llama8b")
    rng = np.random.default_rng(4)
    S = 64
    X = W.random_placements(tr, S, seed=9, density=0.3, feasible=False)
    Y = rng.integers(0, tr.L, X.shape).astype(np.uint8)
    with G(tr) as g:
        cost, ex = _score_slots_gpu(g, X, Y)
        for s in (0, 1, 31, 63):
            r = O.score_slots(q, X[s], Y[s])
            assert cost[s] == r.cost and ex[s] == r.excess, s
    # a placement with many migrations (where a walk that counts the pool per token step ends), and a pool just
    # large enough for it at every inference step: moves that need room are blocked now and then
    X0 = O.anneal_chain(q, 0, O.init_static_frequency(q), seed=3, total_moves=30000, n_levels=20).X
    tr = dataclasses.replace(tr, cap_pages=int(O.score_slots(q, X0, np.zeros_like(X0)).pool.max()))
    q = O.Problem(tr)
    with G(tr) as g:
        chains, total, moves = 256, 100000, 30000
        d_y = torch.empty((chains,) + X0.shape, dtype=torch.uint8, device=g.dev)
        p = K.make_anneal_params(chains, total, moves=moves, seed=tr.seed, init_mode=K.KVP_INIT_EMPTY)
        stats = K.kvp_refine_slots(g.ctx, p, g.words(X0[None])[0].contiguous(), d_y)
        for c in (0, 100, 255):
            w = O.refine_slots(q, c, X0, np.zeros_like(X0), seed=tr.seed, total_moves=total, move_end=moves)
            assert (d_y[c].cpu().numpy() == w.Y).all() and stats[c].t_cur == w.T_cur, c
            assert (stats[c].accepted, stats[c].null_moves, stats[c].clipped) == (w.accepted, w.null_moves, w.clipped)
