"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Each test is chosen so that a plausible
slip in the oracle (a dropped term of Eq. 3/4, a swapped bandwidth, a wrong
neighbour in the migration term, a different summation tree) fails it.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
import workloads as W
from workloads.traces import Trace


def _frac(s):
    a, b = s.split("/")
    return Fraction(a) / Fraction(b)


def _mini(L=1, N=1, P=1, K=1, bw=(4.9e12, 900e9, 500e9), cap=10**6, plane_bytes=None,
          page_bytes=65536, token_bytes=4096):
    z = lambda *s: np.zeros(s, np.uint8)
    return Trace("mini", L, N, P, K, z(L, N, K, P), z(N, P), z(N, P), z(N, P),
                 plane_bytes or [page_bytes // K] * K, page_bytes, token_bytes, bw[0], bw[1], bw[2], cap)


# ---------------------------------------------------------------- Eqs. 2-4 --
def test_step_time_hand_cases(golden_dir):
    rows = 0
    for line in open(os.path.join(golden_dir, "step_time_cases.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        bh, bk, bd = map(float, line[:3])
        b6 = list(map(int, line[3:9]))
        want = float(_frac(line[9]))
        got = O.step_time(_mini(bw=(bh, bk, bd)), b6)
        # the oracle multiplies by a rounded reciprocal: two roundings
        assert got == pytest.approx(want, rel=4e-16, abs=0.0), (line, got, want)
        rows += 1
    assert rows >= 12


def test_step_time_is_max_of_tiers_and_monotone():
    tr = _mini()
    rng = np.random.default_rng(0)
    for _ in range(200):
        b = rng.integers(0, 1 << 24, 6).astype(np.uint64)
        t = O.step_time(tr, b)
        th = float(b[0] + b[2] + b[4] + b[5]) / tr.bw_hbm
        assert t >= th * (1 - 1e-15)
        for i in range(6):                      # more traffic of any kind never helps
            b2 = b.copy(); b2[i] += 4096
            assert O.step_time(tr, b2) >= t


# ------------------------------------------------------------------- csum --
def test_csum_tree_shape_by_hand():
    B = 2.0 ** 53                                # B + 1 rounds back to B (ties to even)
    v = np.zeros(64); v[0] = B; v[32] = 1.0; v[16] = -B
    # fold 32: v0 = B+1 -> B ; fold 16: v0 = B + (-B) = 0.  A left-to-right sum gives 1.
    assert O.csum(v) == 0.0
    v = np.zeros(64); v[0] = B; v[1] = 1.0; v[33] = 1.0
    # fold 32: v1 = 2 ; ... ; fold 1: v0 = B + 2 exactly.  Left-to-right: B+1 -> B, +1 -> B.
    assert O.csum(v) == B + 2.0
    v = np.zeros(64); v[0] = B; v[63] = 1.0; v[31] = 1.0
    # fold 32: v31 = 2; it reaches v0 only at the last fold: B + 2
    assert O.csum(v) == B + 2.0


def test_csum_blocks_are_added_in_order_and_padded():
    B = 2.0 ** 53
    v = np.zeros(130); v[0] = B; v[64] = 1.0; v[128] = 1.0; v[129] = 1.0
    # block sums B, 1, 2 ; (B + 1) -> B ; B + 2 exact
    assert O.csum(v) == B + 2.0
    v = np.zeros(130); v[0] = B; v[64] = 1.0; v[65] = 1.0; v[128] = 1.0
    # block sums B, 2, 1 ; B + 2 exact ; (B+2) + 1 -> tie -> even mantissa = B + 4
    assert O.csum(v) == B + 4.0
    assert O.csum(np.zeros(0)) == 0.0
    assert O.csum(np.array([3.25])) == 3.25


def test_csum_close_to_exact_sum():
    rng = np.random.default_rng(1)
    for m in (1, 63, 64, 65, 1000, 8192):
        v = rng.random(m) * 1e-6
        assert O.csum(v) == pytest.approx(math.fsum(v), rel=1e-13)
    v = rng.integers(0, 1000, 4096).astype(np.float64)      # integers: every order is exact
    assert O.csum(v) == float(v.sum())


# ------------------------------------------------------------------ Philox --
def test_philox_known_answers(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        w = line.split("#")[0].split()
        if not w:
            continue
        x = [int(t, 16) for t in w]
        assert list(O.philox4x32_10(x[0:4], x[4:6])) == x[6:10]
        n += 1
    assert n == 3


# ------------------------------------------------- the sets of Eqs. 3 and 4 --
def _hand_instance():
    tr = _mini(L=1, N=3, P=4, plane_bytes=[100], page_bytes=1000, token_bytes=10, cap=1,
               bw=(1000.0, 100.0, 50.0))
    tr.alive[:] = [[1, 1, 0, 0], [1, 1, 1, 0], [1, 0, 1, 1]]       # page 1 dies, pages 2, 3 are born
    tr.persist[:] = [[0, 0, 0, 0], [1, 1, 0, 0], [1, 0, 1, 0]]
    tr.written[:] = [[0, 1, 0, 0], [0, 0, 1, 0], [0, 0, 0, 1]]
    tr.access[0, :, 0, :] = [[1, 1, 0, 0], [1, 0, 1, 0], [0, 0, 1, 1]]
    X = np.array([[[1, 0, 0, 0], [0, 1, 1, 0], [1, 1, 0, 1]]], np.uint8)   # bit (n=2,p=1) is on a dead page
    return tr, X


def test_step_bytes_hand_instance():
    tr, X = _hand_instance()
    s = O.score(tr, X)
    #                 hr   er   hw  ew   mi    mo
    want = [[100, 100, 0, 10, 0, 0],          # n=0: no migration at the first step
            [100, 100, 10, 0, 1000, 1000],    # p0 leaves, p1 enters, p2 is born in HBM for free
            [100, 100, 10, 0, 1000, 1000]]    # p0 returns, p2 leaves, p3 born; dead bit ignored
    assert s.step_bytes[0].tolist() == want
    assert s.occ.tolist() == [1, 2, 2]
    assert s.excess == (1 | 0x80000000)
    # Eq. 3/4 by hand with B_h=1000, B_k=100, B_d=50:
    t0 = max(100 / 1000, 100 / 50 + max(10 / 100, 0, 10 / 50))
    t1 = max(2110 / 1000, 100 / 50 + max(1000 / 100, 1000 / 100, 2000 / 50))
    assert s.step_t[0].tolist() == pytest.approx([t0, t1, t1], rel=1e-15)
    assert s.cost == pytest.approx(t0 + 2 * t1, rel=1e-15)


def test_total_is_summed_in_execution_order():
    # Eq. 1 summed in the order the steps run, g = n*L + l.  With unit bandwidths
    # a step's latency is its byte count, so t = [2^53, 1, 0, 1] in that order:
    # the tree adds (t0 + t2) + (t1 + t3) = 2^53 + 2 exactly, while the layer-major
    # order [2^53, 0, 1, 1] would give (2^53 + 1 -> 2^53) + 1 -> 2^53.
    tr = _mini(L=2, N=2, P=1, K=2, bw=(1.0, 1.0, 1.0), plane_bytes=[2 ** 53, 1], token_bytes=0)
    tr.alive[:] = 1
    tr.access[0, 0, 0, 0] = 1
    tr.access[1, 0, 1, 0] = 1
    tr.access[1, 1, 1, 0] = 1
    s = O.score(tr, np.zeros((2, 2, 1), np.uint8))
    assert s.step_t.tolist() == [[2.0 ** 53, 0.0], [1.0, 1.0]]
    assert s.cost == 2.0 ** 53 + 2.0


# ------------------------------------------------------------ closed forms --
@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("table1", 1.0), ("llama8b", 0.125),
                                        ("serving", 0.06), ("gqa70b", 0.04)])
def test_closed_forms_all_hbm_and_all_dram(name, scale):
    tr = W.config(name, scale)
    pb = np.array(tr.plane_bytes, dtype=np.int64)
    acc_b = (tr.access.astype(np.int64).sum(axis=3) * pb[None, None, :]).sum(axis=2)   # [L][N]
    wr_b = tr.written.astype(np.int64).sum(axis=1) * tr.token_bytes                     # [N]
    allx = np.broadcast_to(tr.alive[None], (tr.L, tr.N, tr.P)).copy()
    s = O.score(tr, allx)
    # every page in HBM: nothing off-package, no migration: t = (reads + write)/B_h
    want = math.fsum(((acc_b + wr_b[None]) / tr.bw_hbm).ravel())
    assert s.cost == pytest.approx(want, rel=1e-13)
    assert (s.step_bytes[..., 1] == 0).all() and (s.step_bytes[..., 3:] == 0).all()
    assert s.occ.tolist() == (tr.L * tr.alive.sum(axis=1)).tolist()
    # nothing in HBM: t = reads/min{B_k,B_d} + max(write/B_k, write/B_d)
    e = O.score(tr, np.zeros_like(allx))
    bmin = min(tr.bw_link, tr.bw_dram)
    want = math.fsum((acc_b / bmin + wr_b[None] / bmin).ravel())
    assert e.cost == pytest.approx(want, rel=1e-13)
    assert e.excess == 0 and (e.occ == 0).all()
    # any schedule: both tiers working flat out bound a step from below
    lb = (acc_b + wr_b[None]) / (tr.bw_hbm + bmin)
    for X in W.random_placements(tr, 3, seed=7):
        r = O.score(tr, X)
        assert (r.step_t >= lb * (1 - 1e-12)).all()
        assert r.feasible
        hr, er, hw, ew = (r.step_bytes[..., i].astype(np.int64) for i in range(4))
        assert (hr + er == acc_b).all() and (hw + ew == wr_b[None]).all()


def test_score_ignores_dead_bits_and_reports_excess():
    tr = W.config("table1")
    X = W.random_placements(tr, 1, seed=3)[0]
    a = O.score(tr, X)
    Y = X | (1 - tr.alive[None])                   # set every dead bit
    b = O.score(tr, Y)
    assert b.cost == a.cost and (b.occ == a.occ).all()
    assert b.excess == (a.excess | 0x80000000)
    full = O.score(tr, np.ones_like(X))
    assert (full.excess & 0x7FFFFFFF) == int(tr.L * tr.alive.sum(axis=1).max() - tr.cap_pages)


def test_single_step_optimum_is_the_balanced_split():
    # One step, P pages all read, equal sizes: with h pages in HBM the latency is
    # max(h b/B_h, (P-h) b/B_e).  The best h follows from that formula alone.
    P, b = 12, 65536
    tr = _mini(L=1, N=1, P=P, bw=(4.0e12, 0.5e12, 0.5e12), cap=P, page_bytes=b, token_bytes=0)
    tr.alive[:] = 1
    tr.access[:] = 1
    want = min(max(Fraction(h * b, 4 * 10**12), Fraction((P - h) * b, 5 * 10**11)) for h in range(P + 1))
    best, X, nf = O.brute_force(tr)
    assert nf == 2 ** P
    assert best == pytest.approx(float(want), rel=1e-15)
    assert int(X.sum()) == 11          # 11 b/4e12 = 1.80e-7 > 1 b/5e11 = 1.31e-7; h = 10 gives 2.62e-7


# -------------------------------------------------------------- brute force --
def _micro(seed, L=2, N=3, P=3, **kw):
    return W.random_trace(seed, L, N, P, **kw)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_bruteforce_optimum_is_monotone_in_capacity_and_bounded(seed):
    tr = _micro(seed)
    pb = tr.plane_bytes[0]
    acc_b = tr.access.astype(np.int64).sum(axis=(2, 3)) * pb
    wr_b = tr.written.astype(np.int64).sum(axis=1) * tr.token_bytes
    lb = float(((acc_b + wr_b[None]) / (tr.bw_hbm + min(tr.bw_link, tr.bw_dram))).sum())
    prev = None
    for cap in range(0, int(tr.L * tr.alive.sum(axis=1).max()) + 1):
        tr.cap_pages = cap
        best, X, nf = O.brute_force(tr)
        s = O.score(tr, X)
        assert s.cost == best and s.feasible
        assert best >= lb * (1 - 1e-12)
        if cap == 0:                                    # only the empty schedule is feasible
            assert nf == 1 and best == O.cost(tr, np.zeros_like(X))
        if prev is not None:
            assert best <= prev and nf >= prev_nf
        prev, prev_nf = best, nf
        for init in (O.init_static_frequency(tr), O.init_recency(tr)):
            si = O.score(tr, init)
            assert si.feasible and si.cost >= best


# ------------------------------------------------------------------- moves --
def _move(op, l, p, n1, ln, l2=0, q=0, d=0):
    return dict(op=op, layer=l, page=p, n1=n1, len=ln, layer2=l2, page2=q, dsel=d)


def _move_instance():
    tr = _mini(L=2, N=8, P=2, cap=2)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[:] = 1
    X = np.zeros((2, 8, 2), np.uint8)
    X[0, :, 0] = [0, 0, 0, 1, 1, 0, 0, 0]
    X[0, :, 1] = [1, 1, 0, 0, 0, 0, 0, 0]
    X[1, :, 0] = [0, 0, 1, 1, 1, 1, 0, 0]
    return tr, X          # occupancy 1 1 1 2 2 1 0 0, capacity 2


HAND_MOVES = [
    # move, verdict, steps flipped on (layer,page), steps flipped on the victim, base
    (_move(0, 0, 0, 1, 5), 0, [1, 2, 5], [], 1),            # SET to 1 skips steps already set
    (_move(0, 1, 1, 2, 4), 1, [2], [], 2),                  # clipped at the full step 3
    (_move(0, 1, 1, 3, 2), 2, [], [], 3),                   # starts on a full step: null
    (_move(0, 1, 0, 3, 63), 0, [3, 4, 5], [], 3),           # SET to 0 runs to the end of the trace
    (_move(1, 1, 1, 2, 4, 0, 0), 0, [2, 3, 4, 5], [3, 4], 2),   # SWAP evicts the victim only where full
    (_move(1, 1, 1, 3, 2, 0, 1), 2, [], [], 3),             # victim absent on the full steps: null
    (_move(1, 0, 0, 3, 1, 1, 0), 0, [3], [], 3),            # SWAP on a set bit acts as SET to 0
    (_move(2, 0, 0, 0, 10, 0, 0, 0), 0, [1, 2], [], 1),     # SHIFT: rising edge at 3, two steps earlier
    (_move(2, 0, 0, 0, 10, 0, 0, 2), 0, [3], [], 1),        # ... one step later
    (_move(2, 0, 0, 0, 10, 0, 0, 3), 0, [3, 4], [], 1),     # ... two steps later
    (_move(2, 1, 0, 3, 5, 0, 0, 3), 0, [6, 7], [], 4),      # falling edge at 6 moved two steps later
    (_move(2, 1, 0, 3, 5, 0, 0, 1), 0, [5], [], 4),         # falling edge one step earlier
    (_move(2, 1, 0, 3, 2, 0, 0, 1), 2, [], [], 3),          # no edge within (3, 5]
    (_move(2, 1, 1, 0, 63, 0, 0, 0), 2, [], [], 0),         # constant timeline: null
    (_move(0, 0, 0, 8, 1), 2, [], [], 0),                   # malformed record: null
]


@pytest.mark.parametrize("mv,verdict,f1,f2,base", HAND_MOVES)
def test_moves_by_hand(mv, verdict, f1, f2, base):
    tr, X = _move_instance()
    v, dT, b, g1, g2 = O.delta(tr, X, mv)
    assert v == verdict
    assert np.nonzero(g1)[0].tolist() == f1 and np.nonzero(g2)[0].tolist() == f2
    if v != 2:
        assert b == base


def test_shift_respects_capacity_and_span_start():
    tr, X = _move_instance()
    X[1, :, 1] = [0, 0, 0, 0, 0, 1, 1, 0]          # occupancy 1 1 1 2 2 2 1 0
    v, _, _, f1, _ = O.delta(tr, X, _move(2, 1, 1, 2, 6, 0, 0, 0))     # edge at 5, wants steps 4, 3: both full
    assert v == 2 and not f1.any()
    v, _, _, f1, _ = O.delta(tr, X, _move(2, 1, 1, 2, 6, 0, 0, 3))     # same edge two steps later: 5, 6 cleared
    assert v == 0 and np.nonzero(f1)[0].tolist() == [5, 6]
    v, _, b, f1, _ = O.delta(tr, X, _move(2, 1, 1, 5, 6, 0, 0, 3))     # falling edge at 7, two later: the trace ends
    assert v == 0 and np.nonzero(f1)[0].tolist() == [7] and b == 5


@pytest.mark.parametrize("seed", range(6))
def test_moves_keep_schedules_feasible_and_delta_matches_rescoring(seed):
    tr = W.random_trace(100 + seed, L=3, N=40, P=21, K=2 if seed % 2 else 1,
                        plane_bytes=[4096, 61440] if seed % 2 else None)
    X = W.random_placements(tr, 1, seed=seed, density=0.45)[0]
    base = O.score(tr, X)
    assert base.feasible
    mv = W.random_moves(tr, 400, seed=seed, max_len=63 if seed % 3 else 7)
    kinds = set()
    for i in range(400):
        m = {k: int(v[i]) for k, v in mv.items()}
        v, dT, b, f1, f2 = O.delta(tr, X, m)
        kinds.add((m["op"], v))
        if v == 2:
            assert dT == 0.0 and not f1.any() and not f2.any()
            continue
        Y, _ = O.apply_move(tr, X, m)
        after = O.score(tr, Y)
        assert after.feasible and not (after.excess >> 31)
        # the window sum equals the difference of the two totals up to rounding
        assert dT == pytest.approx(after.cost - base.cost, rel=1e-9, abs=1e-12 * base.cost)
        # edits stay on the two timelines and inside the 64-step window
        diff = np.argwhere(Y != X)
        for l, n, p in diff:
            assert (l, p) in ((m["layer"], m["page"]), (m["layer2"], m["page2"]))
            assert b <= n < b + 64
        if f2.any():                                    # a victim is only taken on full steps
            assert (base.occ[f2.astype(bool)] == tr.cap_pages).all()
            assert (after.occ[f2.astype(bool)] == tr.cap_pages).all()
    assert {(0, 0), (1, 0), (2, 0)} <= kinds and any(v == 1 for _, v in kinds)


# --------------------------------------------------------------- annealing --
def test_anneal_reaches_the_exhaustive_optimum_on_micro_instances():
    hit = 0
    for seed in range(4):
        tr = _micro(10 + seed, L=2, N=3, P=3)
        tr.cap_pages = 3
        best, _, _ = O.brute_force(tr)
        X0 = np.zeros((tr.L, tr.N, tr.P), np.uint8)
        res, bi = O.anneal(tr, range(8), X0, seed=seed, total_moves=4000, max_len=3)
        r = res[bi]
        assert r.best_cost >= best * (1 - 1e-15)          # nothing beats the optimum
        assert O.score(tr, r.best_X).feasible
        hit += r.best_cost == best
    assert hit >= 3


def test_anneal_invariants_on_tiny_config():
    tr = W.config("tiny")
    q = O.Problem(tr)
    starts = {"static": O.init_static_frequency(q), "recency": O.init_recency(q),
              "empty": np.zeros(q.shape, np.uint8)}
    for name, X0 in starts.items():
        c0 = O.score(q, X0)
        assert c0.feasible
        r = O.anneal_chain(q, 3, X0, seed=0, total_moves=3000)
        fin = O.score(q, r.X)
        bst = O.score(q, r.best_X)
        assert fin.feasible and bst.feasible
        assert r.best_cost == bst.cost <= c0.cost                  # never worse than its start
        assert r.T_best == pytest.approx(bst.cost, rel=1e-9)       # running value only drifts by rounding
        assert r.T_cur == pytest.approx(fin.cost, rel=1e-9)
        assert r.accepted > 0 and r.C0 >= 0
        if name != "empty":
            assert r.uphill > 0                                     # p0 = 0.8: uphill moves are taken early
    # same seed, same chain: identical; another chain id: a different walk
    a = O.anneal_chain(q, 3, starts["empty"], seed=0, total_moves=3000)
    b = O.anneal_chain(q, 3, starts["empty"], seed=0, total_moves=3000)
    c = O.anneal_chain(q, 4, starts["empty"], seed=0, total_moves=3000)
    assert (a.X == b.X).all() and a.T_cur == b.T_cur
    assert not (a.X == c.X).all()
    # stopping and resuming continues the same walk (counter-based draws)
    h = O.anneal_chain(q, 3, starts["empty"], seed=0, total_moves=3000, move_end=1234)
    h2 = O.anneal_chain(q, 3, None, seed=0, total_moves=3000, move_begin=1234, resume=h)
    assert (h2.X == a.X).all() and h2.T_cur == a.T_cur and (h2.best_X == a.best_X).all()


def test_initial_temperature_gives_the_target_uphill_acceptance():
    # C0 = mean uphill dT / (-ln p0) (Sec. III-B: p0 = 0.8).  Held at that
    # temperature (alpha = 1) a walk accepts uphill proposals at a rate of at
    # least about p0: E[exp(-dT/C0)] >= exp(-E[dT]/C0) = p0 by convexity.
    tr = W.config("tiny")
    X0 = O.init_static_frequency(tr)
    for p0, lo, hi in ((0.8, 0.72, 0.97), (0.3, 0.22, 0.75)):
        r = O.anneal_chain(tr, 0, X0, seed=5, total_moves=600, alpha=1.0, p0=p0)
        assert r.C0 > 0 and r.state.uphill_seen > 100
        assert lo <= r.uphill / r.state.uphill_seen <= hi
    cold = O.anneal_chain(tr, 0, X0, seed=5, total_moves=600, alpha=1e-9, n_levels=600)
    assert cold.uphill <= 2                      # frozen after the first move: pure descent


def test_static_and_recency_placements_by_hand():
    tr = _mini(L=1, N=4, P=3, cap=1)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[0, :, 0, :] = [[1, 0, 0], [0, 1, 0], [0, 1, 0], [0, 0, 1]]
    st = O.init_static_frequency(tr)
    assert st[0].tolist() == [[0, 1, 0]] * 4                   # page 1 is read twice
    rc = O.init_recency(tr)
    # before step 0 nothing was read: lowest index; then the page read one step earlier
    assert rc[0].tolist() == [[1, 0, 0], [1, 0, 0], [0, 1, 0], [0, 1, 0]]


def test_static_fill_by_hand():
    # two layers, three page slots, room for three pages.  Step 0: pages 0 and 1 exist in both layers and take
    # the places in the order (l0,p0) (l0,p1) (l1,p0); (l1,p1) stays outside for good.  Step 1: page 2 is
    # born: no room.  Step 2: slot 0 is re-used by new data: both old entries leave (one place was taken,
    # (l0,p0)), the new (l0,p0) takes it again, and with (l1,p0) gone one more place is free for (l1,p0) new.
    tr = _mini(L=2, N=4, P=3, cap=3)
    tr.alive[:] = [[1, 1, 0], [1, 1, 1], [1, 1, 1], [0, 1, 1]]
    tr.persist[:] = [[0, 0, 0], [1, 1, 0], [0, 1, 1], [0, 1, 1]]
    X = O.init_static_fill(tr)
    assert X[0].tolist() == [[1, 1, 0], [1, 1, 0], [1, 1, 0], [0, 1, 0]]
    assert X[1].tolist() == [[1, 0, 0], [1, 0, 0], [1, 0, 0], [0, 0, 0]]


@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("llama8b", 0.25), ("serving", 0.0625)])
def test_static_fill_never_migrates_and_fills_what_fits(name, scale):
    tr = W.config(name, scale)
    X = O.init_static_fill(tr)
    r = O.score(tr, X)
    assert r.feasible
    assert not (X & ~tr.alive[None]).any()
    assert int(r.step_bytes[..., 4].sum()) == 0 and int(r.step_bytes[..., 5].sum()) == 0     # nothing moves in or out
    occ = X.sum(axis=(0, 2))
    # a page outside HBM while there is room can only be one that was born when there was none
    born = tr.alive.astype(bool) & ~tr.persist.astype(bool)
    born[0] = tr.alive[0].astype(bool)
    for n in range(tr.N):
        if occ[n] < tr.cap_pages:
            assert not (born[n][None] & ~X[:, n].astype(bool)).any()
    # with room for everything, everything that exists is inside
    import dataclasses
    assert (O.init_static_fill(dataclasses.replace(tr, cap_pages=tr.L * tr.P)) == np.broadcast_to(tr.alive[None], X.shape)).all()


# ---- occupancy counted after every (step, layer) slot ----

def test_strict_excess_by_hand():
    # two layers, one page each, room for one.  Step 0: layer 1 holds its page.  Step 1: layer 0 takes its page in at
    # slot (1,0), while layer 1 gives its page up only at slot (1,1): two pages in between, one too many, although
    # every token step as a whole holds one page.
    tr = _mini(L=2, N=2, P=1, cap=1)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    X = np.zeros((2, 2, 1), np.uint8)
    X[1, 0, 0] = 1
    X[0, 1, 0] = 1
    assert O.score(tr, X).excess == 0 and O.strict_excess(tr, X) == 1
    # the other way round the page leaves first: no overshoot
    Y = np.zeros((2, 2, 1), np.uint8)
    Y[0, 0, 0] = 1
    Y[1, 1, 0] = 1
    assert O.score(tr, Y).excess == 0 and O.strict_excess(tr, Y) == 0
    # a page of layer 1 that does not persist into step 1 is gone before slot (1,0)
    tr.persist[1, 0] = 0
    assert O.strict_excess(tr, X) == 0
    # a bit on a page that does not exist takes no room: page 1 of two is never alive
    t2 = _mini(L=2, N=2, P=2, cap=1)
    t2.alive[:, 0] = 1
    t2.persist[1, 0] = 1
    Z = np.zeros((2, 2, 2), np.uint8)
    Z[0, :, 0] = 1                                                     # layer 0 keeps its page: the pool is full
    assert O.strict_excess(t2, Z) == 0
    Z[1, :, 1] = 1                                                     # stray bits of layer 1
    assert O.strict_excess(t2, Z) == 0


@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("llama8b", 0.25), ("serving", 0.0625), ("gqa70b", 0.0625)])
def test_strict_excess_bounds(name, scale):
    tr = W.config(name, scale)
    q = O.Problem(tr)
    # placements that never migrate fill the pool monotonically inside a step: slot by slot is step by step
    for X in (O.init_static_fill(q), O.init_static_frequency(q)):
        assert O.strict_excess(q, X) == O.score(q, X).excess == 0
    # any schedule: never less than the per-step count; at most one layer's swing more
    for X in W.random_placements(tr, 3, seed=4, density=0.5, feasible=False):
        per_step = O.score(q, X).excess & 0x7FFFFFFF
        strict = O.strict_excess(q, X)
        occ_l = (X & tr.alive[None]).sum(axis=2)                       # [L][N]
        assert per_step <= strict <= per_step + int(occ_l.sum(axis=0).max())
    # the last slot of a step is the step: with one layer the two counts agree
    if tr.L == 1:
        X = W.random_placements(tr, 1, seed=5, density=0.9, feasible=False)[0]
        assert O.strict_excess(q, X) == O.score(q, X).excess & 0x7FFFFFFF


# ---- the capacity at every inference step (Eq. 5 with the decision tuple S(n, l) of Sec. III-A) ----

def _slot_table_by_simulation(tr, X):
    """The pool after every slot, counted from scratch: numpy, no code shared with the oracle."""
    L, N, P = X.shape
    cur = np.zeros((L, P), bool)
    tab = np.zeros((N, L), np.int64)
    for n in range(N):
        keep = tr.persist[n].astype(bool) if n > 0 else np.zeros(P, bool)
        cur &= keep[None]
        for l in range(L):
            cur[l] = X[l, n].astype(bool) & tr.alive[n].astype(bool)
            tab[n, l] = cur.sum()
    return tab


def test_slot_occupancy_by_hand():
    tr = _mini(L=2, N=2, P=1, cap=1)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    X = np.zeros((2, 2, 1), np.uint8)
    X[1, 0, 0] = 1
    X[0, 1, 0] = 1                                   # layer 0 takes its page before layer 1 lets go
    assert O.slot_occupancy(tr, X).tolist() == [[0, 1], [2, 1]]
    Y = np.zeros((2, 2, 1), np.uint8)
    Y[0, 0, 0] = 1
    Y[1, 1, 0] = 1                                   # layer 0 lets go before layer 1 takes
    assert O.slot_occupancy(tr, Y).tolist() == [[1, 1], [0, 1]]
    tr.persist[1, 0] = 0                             # the page is replaced at step 1: gone before slot (1, 0)
    assert O.slot_occupancy(tr, X).tolist() == [[0, 1], [1, 1]]


@pytest.mark.parametrize("seed", range(5))
def test_slot_occupancy_against_simulation_and_the_two_excess_counts(seed):
    tr = W.random_trace(300 + seed, L=[1, 2, 3, 5, 4][seed], N=17, P=23, K=1, rebirth=True)
    for X in W.random_placements(tr, 4, seed=seed, density=0.5, feasible=False):
        tab = O.slot_occupancy(tr, X)
        assert (tab == _slot_table_by_simulation(tr, X)).all()
        assert (tab[:, -1] == O.score(tr, X).occ).all()                      # the last slot of a step is the step
        assert max(int(tab.max()) - tr.cap_pages, 0) == O.strict_excess(tr, X)


def _one_page_per_layer(L, N, cap=1):
    tr = _mini(L=L, N=N, P=1, cap=cap)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[:] = 1
    return tr


def test_per_slot_moves_by_hand():
    # two layers, one page each, room for one; layer 1 holds its page at step 0 only.
    # slots: step 0 [0 1], step 1 [1 0] (layer 1 lets go at slot (1,1)), step 2 [0 0]
    tr = _one_page_per_layer(2, 3)
    X = np.zeros((2, 3, 1), np.uint8)
    X[1, 0, 0] = 1
    assert O.slot_occupancy(tr, X).tolist() == [[0, 1], [1, 0], [0, 0]]
    # layer 0 in at step 1: the step as a whole has room, slot (1,0) has not
    assert O.resolve(tr, X, _move(0, 0, 0, 1, 1))[0] == 0
    v, f1, f2, _ = O.resolve(tr, X, _move(0, 0, 0, 1, 1), per_slot=True)
    assert v == 2 and not f1.any()
    # layer 1 in at steps 1 and 2: slot (1,1) has room, and so has (2,0), where the page is still held
    v, f1, f2, _ = O.resolve(tr, X, _move(0, 1, 0, 1, 2), per_slot=True)
    assert v == 0 and f1.tolist() == [0, 1, 1] and not f2.any()
    # layer 0 in at step 2: nothing is held there
    v, f1, f2, _ = O.resolve(tr, X, _move(0, 0, 0, 2, 1), per_slot=True)
    assert v == 0 and f1.tolist() == [0, 0, 1]
    # layer 0 in at step 0: slot (0,1) would hold two
    v, f1, f2, _ = O.resolve(tr, X, _move(0, 0, 0, 0, 1), per_slot=True)
    assert v == 2
    # a run that starts on a free slot stops at the blocked one: steps 2.. of layer 0 from step 2 only
    X2 = X.copy(); X2[1, 2, 0] = 1                   # layer 1 back in at step 2: slots step 2 [0 1]
    v, f1, f2, _ = O.resolve(tr, X2, _move(0, 0, 0, 1, 2), per_slot=True)
    assert v == 2                                     # step 1 blocked at once: nothing flips


def test_per_slot_eviction_by_hand():
    # three layers, one page each, room for one
    tr = _one_page_per_layer(3, 2)
    X = np.zeros((3, 2, 1), np.uint8)
    X[2, :, 0] = 1                                   # the last layer holds its page throughout
    assert O.slot_occupancy(tr, X).tolist() == [[0, 0, 1], [1, 1, 1]]
    mv = _move(1, 0, 0, 1, 1, 2, 0)                  # layer 0 in at step 1, evicting layer 2's page
    v, f1, f2, _ = O.resolve(tr, X, mv)
    assert v == 0 and f1.tolist() == [0, 1] and f2.tolist() == [0, 1]      # the step as a whole: one in, one out
    v, f1, f2, _ = O.resolve(tr, X, mv, per_slot=True)
    assert v == 2 and not f1.any() and not f2.any()  # slots (1,0), (1,1) would hold both: the victim leaves too late
    Y = np.zeros((3, 2, 1), np.uint8)
    Y[0, :, 0] = 1                                   # now the first layer holds its page
    assert O.slot_occupancy(tr, Y).tolist() == [[1, 1, 1], [1, 1, 1]]
    v, f1, f2, _ = O.resolve(tr, Y, _move(1, 2, 0, 1, 1, 0, 0), per_slot=True)
    assert v == 0 and f1.tolist() == [0, 1] and f2.tolist() == [0, 1]      # the victim leaves at slot (1,0), first
    # the same at step 0: layer 2's page would still be held at slot (1,0), where layer 0 takes its page back
    assert O.resolve(tr, Y, _move(1, 2, 0, 0, 1, 0, 0))[0] == 0
    assert O.resolve(tr, Y, _move(1, 2, 0, 0, 1, 0, 0), per_slot=True)[0] == 2
    # unless layer 2's page is replaced at step 1 and so does not carry over
    tr.persist[1, 0] = 0
    v, f1, f2, _ = O.resolve(tr, Y, _move(1, 2, 0, 0, 1, 0, 0), per_slot=True)
    assert v == 0 and f1.tolist() == [1, 0] and f2.tolist() == [1, 0]


def test_per_slot_eviction_relief_by_hand():
    # victim in the page's own layer: it leaves in the very slot in which the page comes
    tr = _mini(L=1, N=1, P=2, cap=1)
    tr.alive[:] = 1
    X = np.zeros((1, 1, 2), np.uint8)
    X[0, 0, 0] = 1
    v, f1, f2, _ = O.resolve(tr, X, _move(1, 0, 1, 0, 1, 0, 0), per_slot=True)
    assert v == 0 and f1.tolist() == [1] and f2.tolist() == [1]
    # a victim that is replaced at the next step frees nothing there: it would have been gone anyway.
    # Two layers, two pages, room for one; page 0 carries over into step 1, page 1 holds new data at step 1.
    t2 = _mini(L=2, N=2, P=2, cap=1)
    t2.alive[:] = 1
    t2.persist[1, 0] = 1
    X = np.zeros((2, 2, 2), np.uint8)
    X[1, 0, 1] = 1                                   # step 0: layer 1 holds page 1 (the victim)
    X[0, 1, 1] = 1                                   # step 1: layer 0 holds page 1
    assert O.slot_occupancy(t2, X).tolist() == [[0, 1], [1, 1]]
    mv = _move(1, 1, 0, 0, 1, 1, 1)                  # layer 1: page 0 in at step 0 for page 1
    assert O.resolve(t2, X, mv)[0] == 0              # each step as a whole holds one page
    v, f1, f2, _ = O.resolve(t2, X, mv, per_slot=True)
    assert v == 2 and not f1.any()                   # page 0 of layer 1 would still be held at slot (1,0)
    Y = X.copy(); Y[1, 0, 1] = 0; Y[1, 0, 0] = 1
    assert O.score(t2, Y).excess == 0 and O.strict_excess(t2, Y) == 1
    t2.persist[1, 1] = 1                             # if page 1 carried over too, its leaving would free slot (1,0)...
    assert O.slot_occupancy(t2, X).tolist() == [[0, 1], [2, 1]]       # ...but then the start itself overfills it
    X[0, 1, 1] = 0; X[0, 1, 0] = 1                   # layer 0 holds page 0 at step 1 instead: slots [[0 1] [2 1]] still
    X[1, 0, 1] = 1
    t2.cap_pages = 2
    # room for two.  Without the eviction slot (1,0) would hold three (layer 0's page, and pages 0 and 1 of
    # layer 1 carried over); with it the victim's leaving frees that slot as well: two
    v, f1, f2, _ = O.resolve(t2, X, mv, per_slot=True)
    assert v == 0 and f1.tolist() == [1, 0] and f2.tolist() == [1, 0]
    Y = X.copy(); Y[1, 0, 1] = 0; Y[1, 0, 0] = 1
    assert O.slot_occupancy(t2, Y).tolist() == [[0, 1], [2, 1]]


def _all_moves(tr, rng, count):
    for _ in range(count):
        yield _move(int(rng.integers(0, 3)), int(rng.integers(tr.L)), int(rng.integers(tr.P)), int(rng.integers(tr.N)),
                    int(rng.integers(1, 6)), int(rng.integers(tr.L)), int(rng.integers(tr.P)), int(rng.integers(4)))


@pytest.mark.parametrize("seed", range(6))
def test_per_slot_moves_never_overfill_a_slot_and_single_bits_match_brute_force(seed):
    rng = np.random.default_rng(seed)
    tr = W.random_trace(400 + seed, L=[2, 3, 4][seed % 3], N=9, P=7, K=1, rebirth=bool(seed % 2))
    tr.cap_pages = int(rng.integers(1, 6))
    X = np.zeros((tr.L, tr.N, tr.P), np.uint8)
    applied = blocked = 0
    for mv in _all_moves(tr, rng, 1500):
        assert O.strict_excess(tr, X) == 0
        v, f1, f2, _ = O.resolve(tr, X, mv, per_slot=True)
        l, p, n1 = mv["layer"], mv["page"], mv["n1"]
        if mv["op"] == 0 and mv["len"] == 1 and tr.alive[n1, p] and not X[l, n1, p]:
            Y = X.copy(); Y[l, n1, p] = 1                # one bit set: allowed exactly when no slot overflows
            assert (v == 0) == (O.strict_excess(tr, Y) == 0)
            blocked += v != 0
        if v == 2:
            continue
        Y = X.copy()
        Y[l, :, p] ^= f1
        Y[mv["layer2"], :, mv["page2"]] ^= f2
        assert O.strict_excess(tr, Y) == 0, mv
        assert not (Y & ~tr.alive[None]).any()
        if rng.random() < 0.7:
            X = Y; applied += 1
    assert applied > 100 and blocked > 0


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_per_slot_optimum_is_no_better_than_per_step_optimum_by_brute_force(seed):
    tr = W.random_trace(500 + seed, L=2, N=3, P=2, K=1, rebirth=False)
    tr.alive[:] = 1; tr.persist[1:] = 1                  # 12 bits: every schedule is enumerated
    tr.cap_pages = 1 + seed % 2
    best_step, _, _ = O.brute_force(tr)
    best_slot, n_slot, n_step = math.inf, 0, 0
    for code in range(1 << 12):
        X = np.array([(code >> i) & 1 for i in range(12)], np.uint8).reshape(2, 3, 2)
        sc = O.score(tr, X)
        if sc.excess:
            assert O.strict_excess(tr, X) > 0            # a full step is a full slot
            continue
        n_step += 1
        if O.strict_excess(tr, X) == 0:
            n_slot += 1
            best_slot = min(best_slot, sc.cost)
    assert 0 < n_slot < n_step                           # the slot reading really forbids some schedules
    assert best_slot >= best_step
    # the walk under the slot reading stays inside its set and cannot beat its optimum
    r = O.anneal_chain(tr, 0, np.zeros((2, 3, 2), np.uint8), seed=seed, total_moves=400, n_levels=10, max_len=3, per_slot=True)
    assert O.strict_excess(tr, r.best_X) == 0 and O.strict_excess(tr, r.X) == 0
    assert r.best_cost >= best_slot


@pytest.mark.parametrize("seed", range(4))
def test_per_slot_walk_keeps_every_slot_within_capacity(seed):
    tr = W.random_trace(600 + seed, L=3, N=30, P=19, K=1, rebirth=True)
    X0 = [np.zeros((tr.L, tr.N, tr.P), np.uint8), O.init_static_frequency(tr)][seed % 2]
    a = O.anneal_chain(tr, seed, X0, seed=11 + seed, total_moves=1500, n_levels=10, max_len=7, per_slot=True)
    b = O.anneal_chain(tr, seed, X0, seed=11 + seed, total_moves=1500, n_levels=10, max_len=7)
    assert O.strict_excess(tr, a.X) == 0 and O.strict_excess(tr, a.best_X) == 0
    assert a.accepted > 50 and a.best_cost <= O.cost(tr, X0) and (seed % 2 or a.best_cost < O.cost(tr, X0))
    assert a.T_cur == pytest.approx(O.cost(tr, a.X), rel=1e-12)
    assert (a.X != b.X).any()                            # the two readings walk apart
    # a start that overfills a slot is refused, though every step as a whole fits
    t2 = _one_page_per_layer(2, 2)
    bad = np.zeros((2, 2, 1), np.uint8); bad[1, 0, 0] = 1; bad[0, 1, 0] = 1
    O.anneal_chain(t2, 0, bad, seed=1, total_moves=10, n_levels=1)
    with pytest.raises(ValueError):
        O.anneal_chain(t2, 0, bad, seed=1, total_moves=10, n_levels=1, per_slot=True)


# ---- migration in any inference step (Sec. III-A: S(n, l) places all KV data; the bytes are charged where they move) ----

def _slot_instance():
    # two layers, one page each.  Layer 0 keeps its page in HBM and reads it at step 1; layer 1's page comes in for step 1.
    # B_h = 8, B_k = 2, B_d = 4 bytes/s; a page and a read are 8 bytes.
    tr = _mini(L=2, N=2, P=1, bw=(8.0, 2.0, 4.0), cap=2, page_bytes=8, token_bytes=8)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[0, 1, 0, 0] = 1
    X = np.zeros((2, 2, 1), np.uint8)
    X[0, :, 0] = 1
    X[1, 1, 0] = 1
    return tr, X


def test_slot_score_by_hand():
    tr, X = _slot_instance()
    Y = np.zeros_like(X)
    # in its own step (1,1), step 3 of 4: step 2 reads 8 bytes of HBM (8/8 = 1 s); step 3 moves 8 bytes in:
    # t^h = 1, t^e = max(0, 8/2, 8/4) = 4
    s0 = O.score_slots(tr, X, Y)
    assert s0.slot_t.tolist() == [0.0, 0.0, 1.0, 4.0] and s0.cost == 5.0
    assert s0.pool.tolist() == [1, 1, 1, 2] and s0.excess == 0
    assert O.slot_bytes(tr, X, Y, 3).tolist() == [0, 0, 0, 0, 8, 0] and O.slot_bytes(tr, X, Y, 2).tolist() == [8, 0, 0, 0, 0, 0]
    # one step earlier, in layer 0's step (1,0): t^h = (8 + 8)/8 = 2, t^e = 4: the HBM read hides under the transfer
    Y[1, 1, 0] = 1
    s1 = O.score_slots(tr, X, Y)
    assert s1.slot_t.tolist() == [0.0, 0.0, 4.0, 0.0] and s1.cost == 4.0
    assert s1.pool.tolist() == [1, 1, 2, 2] and s1.excess == 0          # the page takes its room one step earlier
    assert O.slot_bytes(tr, X, Y, 2).tolist() == [8, 0, 0, 0, 8, 0] and O.slot_bytes(tr, X, Y, 3).tolist() == [0] * 6
    tr.cap_pages = 1
    assert O.score_slots(tr, X, Y).excess == 1 and O.score_slots(tr, X, np.zeros_like(X)).excess == 1
    # Y is looked at only where a page migrates, and must name one of the L steps up to the page's own
    Y[:] = 0; Y[0, 1, 0] = 1; Y[1, 0, 0] = 1
    assert O.score_slots(tr, X, Y).slot_t.tolist() == s0.slot_t.tolist()
    Y[1, 1, 0] = 2
    bad = O.score_slots(tr, X, Y)
    assert bad.excess & 0x40000000 and bad.slot_t.tolist() == s0.slot_t.tolist()
    # a page that leaves: layer 1 holds its page at step 0 only.  Leaving one step earlier frees the room earlier
    Z = np.zeros((2, 2, 1), np.uint8); Z[1, 0, 0] = 1
    tr.cap_pages = 2
    Y[:] = 0
    assert O.score_slots(tr, Z, Y).pool.tolist() == [0, 1, 1, 0]
    assert O.slot_bytes(tr, Z, Y, 3).tolist() == [0, 0, 0, 0, 0, 8]
    Y[1, 1, 0] = 1
    assert O.score_slots(tr, Z, Y).pool.tolist() == [0, 1, 0, 0]
    assert O.slot_bytes(tr, Z, Y, 2).tolist() == [0, 8, 0, 0, 0, 8]                     # layer 0's read now comes from DRAM


def _pool_by_simulation(tr, X, Y):
    """The pool after every inference step, page by page: numpy, no code shared with the oracle."""
    L, N, P = X.shape
    alive, persist = tr.alive.astype(bool), tr.persist.astype(bool)
    x = X.astype(bool) & alive[None]
    pool = np.zeros(N * L, np.int64)
    # when does page (l, p) take the value it has at its step n: at its own step, or Y steps earlier if it migrates
    since = np.zeros((L, N, P), np.int64)
    for l in range(L):
        for n in range(N):
            since[l, n] = n * L + l
            if n > 0:
                mig = persist[n] & (x[l, n] != x[l, n - 1])
                y = np.where(Y[l, n] > L - 1, 0, Y[l, n]).astype(np.int64)
                since[l, n] -= np.where(mig, y, 0)
    for g in range(N * L):
        n0 = g // L
        cnt = 0
        for l in range(L):
            for p in range(P):
                # the newest step of the page whose value has taken effect by g
                m = n0 + 1 if n0 + 1 < N and since[l, n0 + 1, p] <= g and persist[n0 + 1, p] else n0
                if m == n0 and since[l, n0, p] > g:
                    # its own step of this token step is still to come: the value of the step before, if it carried over
                    cnt += bool(n0 > 0 and persist[n0, p] and x[l, n0 - 1, p])
                else:
                    cnt += bool(x[l, m, p])
        pool[g] = cnt
    return pool


@pytest.mark.parametrize("seed", range(6))
def test_slot_score_against_the_per_layer_score_and_a_simulation(seed):
    rng = np.random.default_rng(seed)
    tr = W.random_trace(700 + seed, L=[1, 2, 3, 4, 5, 3][seed], N=11, P=13, K=1 + seed % 2, rebirth=bool(seed % 2))
    L = tr.L
    for X in W.random_placements(tr, 3, seed=seed, density=0.5, feasible=False):
        Y0 = np.zeros_like(X)
        s0, ref = O.score_slots(tr, X, Y0), O.score(tr, X)
        # every page in its own step: the schedule of Eqs. 1-5 as scored before, and the pool of the per-slot count
        assert s0.cost == ref.cost and (s0.slot_t.reshape(tr.N, L) == ref.step_t.T).all()
        assert (s0.pool.reshape(tr.N, L) == O.slot_occupancy(tr, X)).all()
        assert (s0.excess & 0x3FFFFFFF) == O.strict_excess(tr, X)
        Y = rng.integers(0, L, X.shape).astype(np.uint8)
        s1 = O.score_slots(tr, X, Y)
        assert (s1.pool == _pool_by_simulation(tr, X, Y)).all()
        # bytes are moved, not made: every kind of volume sums to what it was
        b0 = np.array([O.slot_bytes(tr, X, Y0, g) for g in range(tr.N * L)]).sum(axis=0)
        b1 = np.array([O.slot_bytes(tr, X, Y, g) for g in range(tr.N * L)]).sum(axis=0)
        assert (b0 == b1).all() and b0[4] + b0[5] > 0
        # reads and writes stay in their steps
        for g in range(tr.N * L):
            assert (O.slot_bytes(tr, X, Y, g)[:4] == O.slot_bytes(tr, X, Y0, g)[:4]).all()
        assert s1.cost == O.csum(s1.slot_t)


def test_slot_refinement_by_hand_and_against_enumeration():
    # the hand instance: one page migrates, two steps to choose from; the walk must find the cheaper one
    tr, X = _slot_instance()
    r = O.refine_slots(tr, 0, X, np.zeros_like(X), seed=3, total_moves=200, n_levels=5)
    assert r.Y[1, 1, 0] == 1 and r.T_best == 4.0 and O.score_slots(tr, X, r.Y).cost == 4.0
    tr.cap_pages = 1                                            # the start already overfills: refused
    with pytest.raises(ValueError):
        O.refine_slots(tr, 0, X, np.zeros_like(X), seed=3, total_moves=10, n_levels=1)
    # a micro instance, all assignments enumerated
    tr = W.random_trace(811, L=3, N=3, P=2, K=1, rebirth=False)
    tr.alive[:] = 1; tr.persist[1:] = 1
    tr.cap_pages = 4
    X = None
    for cand in W.random_placements(tr, 60, seed=2, density=0.5):
        mig = (cand[:, 1:] != cand[:, :-1]).sum()
        if 3 <= mig <= 5 and O.strict_excess(tr, cand) == 0:
            X = cand; break
    assert X is not None
    where = np.argwhere(X[:, 1:] != X[:, :-1])
    best, n_ok = math.inf, 0
    for code in range(3 ** len(where)):
        Y = np.zeros_like(X)
        c = code
        for (l, n, p) in where:
            Y[l, n + 1, p] = c % 3; c //= 3
        sc = O.score_slots(tr, X, Y)
        if sc.excess == 0:
            n_ok += 1; best = min(best, sc.cost)
    assert n_ok >= 2 and best <= O.score(tr, X).cost
    r = O.refine_slots(tr, 1, X, np.zeros_like(X), seed=5, total_moves=3000, n_levels=20)
    final = O.score_slots(tr, X, r.Y)
    assert final.excess == 0 and best <= final.cost <= O.score(tr, X).cost
    assert r.T_cur == pytest.approx(final.cost, rel=1e-12) and r.T_best >= best * (1 - 1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_slot_refinement_stays_feasible_and_in_slices(seed):
    tr = W.random_trace(900 + seed, L=4, N=20, P=17, K=1, rebirth=True)
    q = O.Problem(tr)
    X = O.anneal_chain(q, 0, np.zeros(q.shape, np.uint8), seed=seed, total_moves=1500, n_levels=10, max_len=7, per_slot=True).X
    tr2 = tr
    r = O.refine_slots(q, seed, X, np.zeros_like(X), seed=20 + seed, total_moves=4000, n_levels=10)
    sc = O.score_slots(q, X, r.Y)
    assert sc.excess == 0 and r.accepted > 20 and r.T_cur == pytest.approx(sc.cost, rel=1e-12)
    assert r.T_best <= O.cost(q, X)
    a = O.refine_slots(q, seed, X, np.zeros_like(X), seed=20 + seed, total_moves=4000, n_levels=10, move_end=1700)
    b = O.refine_slots(q, seed, X, None, seed=20 + seed, total_moves=4000, n_levels=10, move_begin=1700, resume=a)
    assert (b.Y == r.Y).all() and b.T_cur == r.T_cur and b.accepted == r.accepted and b.null_moves == r.null_moves
    if seed == 0:                                               # a tight pool blocks moves that would need room
        tight = O.Problem(tr2.__class__(**{**tr2.__dict__, "cap_pages": int(O.score_slots(q, X, np.zeros_like(X)).pool.max())}))
        rt = O.refine_slots(tight, seed, X, np.zeros_like(X), seed=20 + seed, total_moves=4000, n_levels=10)
        assert rt.clipped > 0 and O.score_slots(tight, X, rt.Y).excess == 0


# ---- token-granular reads inside pages: the plane encoding against the token-level definition ----

def _token_trace(seed=9):
    return W.generate(W.Recipe("tok", L=3, N=40, page_tokens=1, prompt_lo=200, prompt_hi=200, top_frac=0.3,
                               sink_tokens=4, recent_tokens=8, cap_frac=0.3, seed=seed))


@pytest.mark.parametrize("pt", [4, 16])
def test_token_granular_reads_cost_what_their_tokens_cost(pt):
    """A page placement scored on the regrouped trace moves, in reads and writes of every step, exactly the
    bytes that the same placement moves token by token; reading whole pages moves at least as much."""
    tok = _token_trace()
    pg, whole = W.regroup(tok, pt, "token"), W.regroup(tok, pt, "page")
    assert pg.K == pt.bit_length() and pg.plane_bytes == [tok.token_bytes << k for k in range(pg.K)]
    assert pg.page_bytes == pt * tok.token_bytes and pg.cap_pages == tok.cap_pages // pt
    touched = (np.add.reduceat(np.pad(tok.access[:, :, 0, :], ((0, 0), (0, 0), (0, pg.P * pt - tok.P))),
                               np.arange(0, pg.P * pt, pt), axis=-1) > 0)
    for x in W.random_placements(pg, 3, seed=3, density=0.4):
        xt = np.repeat(x, pt, axis=-1)[..., :tok.P] & tok.alive[None]
        a, b, w = O.score(pg, x).step_bytes, O.score(tok, xt).step_bytes, O.score(whole, x).step_bytes
        assert (a[..., :4] == b[..., :4]).all()                       # hr, er, hw, ew
        assert (a[..., 0] + a[..., 1] == tok.token_bytes * tok.access[:, :, 0, :].sum(axis=-1)).all()
        assert (w[..., 0] + w[..., 1] == pg.page_bytes * touched.sum(axis=-1)).all()
        assert (w[..., 0] >= a[..., 0]).all() and (w[..., 1] >= a[..., 1]).all()
        assert (w[..., 2:] == a[..., 2:]).all()                       # writes and migration do not depend on the read model


# ---- the (W, R) look-ahead policy and its search (Sec. III-B), pinned to the reading stated in the oracle ----

def _wr_mini():
    tr = _mini(L=1, N=4, P=4, cap=2)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[0, :, 0, :] = [[1, 1, 0, 0], [0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 0, 1]]
    return tr


def test_wr_policy_by_hand():
    tr = _wr_mini()
    # W = 2, R = 1.  n=0: reads in steps 0,1 are (1,2,1,0): ranking 1,0,2: wanted {1,0}, both come in.
    # n=1: (0,1,2,1): wanted {2,1}; 2 comes in, the pool is full: the unwanted page 0 leaves.
    # n=2: (0,0,1,2): wanted {3,2}; 3 comes in, 1 leaves.  n=3: wanted {3}: nothing to do.
    assert O.wr_policy(tr, 2, 10)[0].tolist() == [[1, 1, 0, 0], [0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 1, 1]]
    # R = 0.5: of the two qualified pages at n=0 only round(0.5 * 2) = 1 comes in, the better ranked (page 1);
    # n=1: one qualified, round(0.5) = 1 (half rounds up): page 2, no eviction needed
    assert O.wr_policy(tr, 2, 5)[0].tolist() == [[0, 1, 0, 0], [0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 1, 1]]
    # R = 0.4: round(0.8) = 1 at n=0 (page 1), round(0.4) = 0 at n=1; at n=2 pages 3 and 2 are qualified:
    # round(0.8) = 1, page 3, and there is room for it
    assert O.wr_policy(tr, 2, 4)[0].tolist() == [[0, 1, 0, 0], [0, 1, 0, 0], [0, 1, 0, 1], [0, 1, 0, 1]]
    # W = 1 only sees the current step: ties to the lower page
    assert O.wr_policy(tr, 1, 10)[0].tolist() == [[1, 1, 0, 0], [0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 1, 1]]
    # R = 0: nothing ever migrates
    assert not O.wr_policy(tr, 3, 0).any()


def test_wr_policy_forgets_pages_that_stop_persisting_and_counts_planes():
    tr = _wr_mini()
    tr.persist[2, 1] = 0                                         # page 1 is re-used at step 2
    got = O.wr_policy(tr, 4, 10)[0].tolist()
    # n=0: reads ahead (1,2,2,2): ranking 1,2,3,0: pool {1,2}; n=1: (0,1,2,2): ranking 2,3,1: wanted {2,3}: 3 in, 1 out
    # n=2: page 1 would have left anyway; (0,0,1,2): pool {2,3} stays
    assert got == [[0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 1, 1], [0, 0, 1, 1]]
    tr2 = _mini(L=2, N=2, P=2, K=2, cap=1)
    tr2.alive[:] = 1
    tr2.persist[1:] = 1
    tr2.access[0, 0, :, 0] = [1, 0]                              # (layer 0, page 0): one plane reads it
    tr2.access[1, 0, :, 1] = [1, 1]                              # (layer 1, page 1): both planes read it
    X = O.wr_policy(tr2, 1, 10)
    assert X[:, 0, :].tolist() == [[0, 0], [0, 1]]              # the pool is shared by the layers: frequency 2 beats 1
    assert X[:, 1, :].tolist() == [[0, 0], [0, 1]]              # nothing is read at step 1: the pool stays


def _wr_rows(rows, cap=2):
    tr = _mini(L=1, N=len(rows), P=len(rows[0]), cap=cap)
    tr.alive[:] = 1
    tr.persist[1:] = 1
    tr.access[0, :, 0, :] = rows
    return tr


def test_wr_policy_evictions_by_hand():
    """Who leaves a full pool, and how many: three instances worked by hand from the stated reading."""
    # W = 1, R = 0.5, room for 2.  n=0: only page 2 is read: it comes in (round(0.5) = 1).  n=1: reads (1,1,0,1):
    # wanted {0,1}, one of the two qualified comes in (page 0), there is room.  n=2: wanted {1} comes in, the pool
    # {0,2} is full: ONE page leaves, both candidates are unread, so the lower index, page 0.
    assert O.wr_policy(_wr_rows([[0, 0, 1, 0], [1, 1, 0, 1], [0, 1, 0, 0]]), 1, 5)[0].tolist() == \
        [[0, 0, 1, 0], [1, 0, 1, 0], [0, 1, 1, 0]]
    # W = 1, R = 1.  n=0: reads (1,0,1,1): wanted {0,2} come in.  n=1: every page is read once: ranking 0,1,2,3, wanted
    # {0,1}; page 1 comes in and the unwanted page 2 leaves -- not the wanted page 0, which is read as often and has
    # the lower index.  n=2: wanted {1,2}: 2 in, 0 out.
    assert O.wr_policy(_wr_rows([[1, 0, 1, 1], [1, 1, 1, 1], [0, 1, 1, 0]]), 1, 10)[0].tolist() == \
        [[1, 0, 1, 0], [1, 1, 0, 0], [0, 1, 1, 0]]
    # W = 2, R = 0.5.  n=0: reads over steps 0,1 are (0,1,2,1): wanted {2,1}, one comes in: page 2.  n=1: steps 1,2:
    # (1,1,1,2): ranking 3,0,1,2: wanted {3,0}, page 3 comes in, there is room.  n=2: only step 2 is left: (1,1,0,1):
    # wanted {0,1}, page 0 comes in; of the unwanted pool pages 2 (unread) and 3 (read once) the LEAST read leaves.
    assert O.wr_policy(_wr_rows([[0, 1, 1, 0], [0, 0, 1, 1], [1, 1, 0, 1]]), 2, 5)[0].tolist() == \
        [[0, 0, 1, 0], [0, 0, 1, 1], [1, 0, 0, 1]]
    # a slot re-used by new data at step 1 (it exists before and after, but does not persist): the old entry leaves
    # the pool, and the new one is not read, so it stays outside
    tr = _wr_rows([[1, 1], [0, 1]])
    tr.persist[1, 0] = 0
    assert O.wr_policy(tr, 1, 10)[0].tolist() == [[1, 1], [0, 1]]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_wr_policy_invariants(seed):
    tr = W.random_trace(100 + seed, L=2, N=12, P=9, K=2, cap_pages=5)
    q = O.Problem(tr)
    for Wn in (1, 3, 12, 40):
        for r10 in (0, 3, 10):
            X = O.wr_policy(tr, Wn, r10).astype(bool)
            assert not (X & ~tr.alive.astype(bool)[None]).any()          # only existing pages
            assert X.sum(axis=(0, 2)).max() <= tr.cap_pages               # the shared pool is never overfull
            assert O.score(q, X).excess == 0
            if r10 == 0:
                assert not X.any()
    # capacity for everything and R = 1: whatever is read within the window is in HBM when it is read
    big = W.random_trace(100 + seed, L=2, N=12, P=9, K=2, cap_pages=2 * 9)
    X = O.wr_policy(big, 2, 10).astype(bool)
    read_now = big.access.astype(bool).any(axis=2)                        # [L][N][P]
    assert not (read_now & ~X).any()


def test_wr_search_walks_the_grid_as_stated():
    tr = W.config("tiny")
    q = O.Problem(tr)
    res, tab = O.wr_search(tr, w_max=12, total_moves=300, n_levels=10, seed=7, stop_rel=0.0, c_min_frac=0.0)
    known = tab >= 0
    assert res.stop_reason == 0 and res.proposals == 300 and res.evaluated == known.sum()
    assert res.best_T == tab[known].min() and tab[res.best_w - 1, res.best_r10] == res.best_T
    assert tab[res.cur_w - 1, res.cur_r10] == res.cur_T
    # every table entry is the score of the policy's schedule
    for w, r in [(res.best_w, res.best_r10), (1, 5), (res.cur_w, res.cur_r10)]:
        assert tab[w - 1, r] == O.score(q, O.wr_policy(tr, w, r)).cost
    # start temperature: an average uphill proposal from the start is accepted with probability p0
    assert res.c0 > 0
    # the paper's stop rules end the walk early: no 0.1 % improvement over a level
    res2, _ = O.wr_search(tr, w_max=12, total_moves=3000, n_levels=10, seed=7)
    assert res2.stop_reason in (1, 2) and res2.proposals < 3000
    # the search over placements themselves does at least as well from the same start
    best = O.wr_policy(tr, res.best_w, res.best_r10)
    out, _ = O.anneal(tr, chains=[0], X0=best, total_moves=3000, seed=1)
    assert out[0].T_best <= res.best_T


# ---- replica exchange between chains (parallel tempering; an extension, not in the paper) ---------

def test_exchange_by_hand():
    # the colder chain holds the worse schedule: (1/1 - 1/2)(10 - 8) = 1 > 0, they always trade
    C, C0, n = O.exchange_step(3, 0, [10.0, 8.0], [1.0, 2.0], [1.5, 2.5])
    assert (list(C), list(C0), n) == ([2.0, 1.0], [2.5, 1.5], 1)
    # odd rounds pair (1, 2), (3, 4), ...: chain 0 and, with four chains, chain 3 sit out
    C, C0, n = O.exchange_step(3, 1, [0.0, 9.0, 1.0, 0.0], [7.0, 1.0, 4.0, 9.0], [7.0, 1.0, 4.0, 9.0])
    assert (list(C), n) == ([7.0, 4.0, 1.0, 9.0], 1)
    # equal costs or equal temperatures: exponent 0, the trade is accepted (and changes nothing that matters)
    assert O.exchange_step(3, 0, [5.0, 5.0], [1.0, 2.0], [1.0, 2.0])[2] == 1
    assert list(O.exchange_step(3, 0, [5.0, 6.0], [2.0, 2.0], [1.0, 3.0])[1]) == [3.0, 1.0]
    # a temperature that is not positive: the pair is left alone
    C, C0, n = O.exchange_step(3, 0, [10.0, 8.0], [0.0, 2.0], [0.0, 2.0])
    assert (list(C), n) == ([0.0, 2.0], 0)
    # a single chain, and the last chain of an odd count in an even round
    assert O.exchange_step(3, 0, [1.0], [1.0], [1.0])[2] == 0
    assert list(O.exchange_step(3, 0, [9.0, 1.0, 5.0], [1.0, 2.0, 3.0], [1.0, 2.0, 3.0])[0]) == [2.0, 1.0, 3.0]


def test_exchange_accepts_with_the_metropolis_probability():
    # the colder chain holds the better schedule: exponent (1/1 - 1/2)(8 - 10) = -1, traded with probability 1/e
    rounds = 20000
    k = sum(O.exchange_step(11, 2 * r, [8.0, 10.0], [1.0, 2.0], [1.0, 2.0])[2] for r in range(rounds))
    p = math.exp(-1.0)
    assert abs(k / rounds - p) < 4.0 * math.sqrt(p * (1 - p) / rounds)
    # the same by the position of the pair instead of the round
    n = 4000
    T = np.tile([8.0, 10.0], n)
    C = np.tile([1.0, 2.0], n)
    k = O.exchange_step(12, 0, T, C, C)[2]
    assert abs(k / n - p) < 4.0 * math.sqrt(p * (1 - p) / n)


def test_exchange_draw_is_the_stated_philox_block():
    seed, rnd, a = 0x1234_5678_9ABC_DEF0, (5 << 32) | 6, 2
    r = O.philox4x32_10([rnd & 0xFFFFFFFF, rnd >> 32, a, 16], [seed & 0xFFFFFFFF, seed >> 32])
    u = ((int(r[0]) << 20 | int(r[1]) >> 12) + 0.5) * 2.0 ** -52
    # chains 2 and 3 with temperatures 1 and 2 and cost gap g: exponent -g / 2; trade iff u < exp(-g / 2)
    g = -2.0 * math.log(u)
    for gap, want in ((g * (1 - 1e-9), 1), (g * (1 + 1e-9), 0)):
        T = [0.0, 0.0, 1.0, 1.0 + gap]
        assert O.exchange_step(seed, rnd, T, [1.0, 1.0, 1.0, 2.0], [1.0, 1.0, 1.0, 2.0])[2] == 1 + want
        # (the pair (0, 1) has equal costs and always trades)


@pytest.mark.parametrize("seed", [0, 1])
def test_exchange_keeps_the_ladder_and_feeds_the_next_slice(seed):
    tr = W.config("tiny")
    kw = dict(seed=seed, total_moves=4000, n_levels=10)
    X0 = O.init_static_frequency(O.Problem(tr))
    res = [O.anneal_chain(tr, c, X0, move_end=1000, **kw) for c in range(5)]       # calibrates, then the first moves
    O.temper(res, [1.0, 2.0, 4.0, 8.0, 16.0])
    ladder = sorted(r.state.C for r in res)
    level0 = res[0].state.level
    assert all(r.state.C0 == r.C0 for r in res)
    traded = 0
    for rnd in range(1, 4):
        before = sorted((r.state.C, r.state.C0) for r in res)
        traded += O.exchange(res, seed, rnd)
        assert sorted((r.state.C, r.state.C0) for r in res) == before             # temperatures move, none is lost
        res = [O.anneal_chain(tr, r.chain, None, move_begin=1000 * rnd, move_end=1000 * (rnd + 1), resume=r, **kw)
               for r in res]
    assert traded > 0
    # every chain cooled by the same factor: what they hold is still the ladder times alpha^level
    level = res[0].state.level
    assert all(r.state.level == level for r in res)
    want = []
    for c in ladder:
        for _ in range(level - level0):
            c = c * 0.9
        want.append(c)
    assert sorted(r.state.C for r in res) == want
    for r in res:
        assert O.score(O.Problem(tr), r.X).excess == 0 and r.T_best <= O.cost(O.Problem(tr), X0)


# ---- the two proposal generators (Sec. III-B: three operators with shares 0.4, 0.4, 0.2; window
# ---- steps -2, -1, +1, +2; ratio steps -0.1, +0.1) ------------------------------------------------

def _within(k, n, p, sigmas=4.0):
    return abs(k / n - p) < sigmas * math.sqrt(p * (1 - p) / n)


def test_draw_move_decoded_by_hand_from_the_published_block():
    # Seed 0, chain 0, move 0, stream 0: block 0 of the proposal is Philox4x32-10 of counter 0 under
    # key 0, the first published vector: 6627e8d5 e169c58d bc57ac4c 9b00dbd8.
    #   word 0 = 1713891541 = 0.39905 * 2^32, below 0.4 * 2^32 (floor 1717986918): the first operator
    #   word 1 / 2^32 = 0.880520: layer floor(0.880520 * 32)  = floor(28.18)  = 28
    #   word 2 / 2^32 = 0.735713: page  floor(0.735713 * 272) = floor(200.11) = 200
    #   word 3 / 2^32 = 0.605482: step  floor(0.605482 * 256) = floor(155.003) = 155
    tr = _mini(L=32, N=256, P=272)
    m, _ = O.draw_moves(tr, 0, 0, 1, seed=0)
    assert (m["op"][0], m["layer"][0], m["page"][0], m["n1"][0]) == (0, 28, 200, 155)
    # the shares are cumulative: with 0.39 for the first operator the same word (0.39905) falls to the
    # second, and with 0.39 + 0.009 for the first two to the third
    assert O.draw_moves(tr, 0, 0, 1, seed=0, op_prob=(0.39, 0.41, 0.2))[0]["op"][0] == 1
    assert O.draw_moves(tr, 0, 0, 1, seed=0, op_prob=(0.39, 0.009, 0.601))[0]["op"][0] == 2
    # another shape, the same block: floor(0.880520 * 80) = 70, floor(0.735713 * 1040) = 765,
    # floor(0.605482 * 2048) = 1240
    m, _ = O.draw_moves(_mini(L=80, N=2048, P=1040), 0, 0, 1, seed=0)
    assert (m["layer"][0], m["page"][0], m["n1"][0]) == (70, 765, 1240)
    # the third published vector as (move, chain, stream) = counter and seed = key
    ctr, key = [0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0]
    blk = [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]
    m, _ = O.draw_moves(tr, ctr[2], ctr[0] | ctr[1] << 32, 1, seed=key[0] | key[1] << 32, stream0=ctr[3])
    # 0xd16cfe09 / 2^32 = 0.818: beyond 0.4 + 0.4, the third operator
    assert (m["op"][0], m["layer"][0], m["page"][0], m["n1"][0]) == (
        2, blk[1] * 32 >> 32, blk[2] * 272 >> 32, blk[3] * 256 >> 32) == (2, 18, 85, 36)


def test_draw_slot_move_decoded_by_hand_from_the_published_blocks():
    # The proposal of the annealing over migration steps is one block.  Seed 0, chain 0, move 0, stream 0: counter 0
    # under key 0, the first published vector 6627e8d5 e169c58d bc57ac4c 9b00dbd8.
    #   word 0 / 2^32 = 0.399045: migrating page floor(0.399045 * 1000) = 399
    #   word 1 / 2^32 = 0.880520: new Y floor(0.880520 * 32) = 28
    #   u = ((bc57ac4c << 20 | 9b00dbd8 >> 12) + 1/2) 2^-52 = 0.7357...
    idx, y, u = O.draw_slot_moves(0, 0, 1, seed=0, stream=0, M=1000, L=32)
    assert (idx[0], y[0]) == (399, 28)
    assert u[0] == ((0xbc57ac4c << 20 | 0x9b00dbd8 >> 12) + 0.5) * 2.0 ** -52 and 0.7357 < u[0] < 0.7358
    idx, y, _ = O.draw_slot_moves(0, 0, 1, seed=0, stream=0, M=3, L=1)
    assert (idx[0], y[0]) == (1, 0)                                      # floor(0.399 * 3) = 1; one layer: Y = 0
    # the third published vector as (move, chain, stream) = counter and seed = key
    ctr, key = [0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0]
    blk = [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]
    idx, y, u = O.draw_slot_moves(ctr[2], ctr[0] | ctr[1] << 32, 1, seed=key[0] | key[1] << 32, stream=ctr[3], M=77777, L=80)
    # 0xd16cfe09 / 2^32 = 0.818069: floor(0.818069 * 77777) = floor(63626.98) = 63626; 0x94fdcceb / 2^32 = 0.581998: 46
    assert (idx[0], y[0]) == (blk[0] * 77777 >> 32, blk[1] * 80 >> 32) == (63626, 46)
    assert u[0] == ((blk[2] << 20 | blk[3] >> 12) + 0.5) * 2.0 ** -52
    # consecutive proposals are consecutive counters: the index and Y are uniform, and not tied to each other
    idx, y, u = O.draw_slot_moves(3, 0, 60000, seed=99, stream=32, M=10, L=4)
    for v in range(10):
        assert _within(int((idx == v).sum()), 60000, 0.1)
    for v in range(4):
        assert _within(int((y == v).sum()), 60000, 0.25)
    assert _within(int(((idx == 3) & (y == 2)).sum()), 60000, 0.025) and _within(int((u < 0.3).sum()), 60000, 0.3)
    first, _, _ = O.draw_slot_moves(3, 0, 5, seed=99, stream=40, M=10, L=4)
    assert first.tolist() != idx[:5].tolist()                            # the calibration draws from a stream of its own


def test_slot_refinement_proposes_migrating_pages_only():
    # every proposal names a page that migrates, so the null moves are those whose drawn Y is the old one: about 1 in L
    tr = W.random_trace(950, L=4, N=20, P=17, K=1, rebirth=True)
    q = O.Problem(tr)
    X = O.anneal_chain(q, 0, np.zeros(q.shape, np.uint8), seed=1, total_moves=1500, n_levels=10, max_len=7, per_slot=True).X
    r = O.refine_slots(q, 0, X, np.zeros_like(X), seed=4, total_moves=8000, n_levels=10)
    assert _within(r.null_moves - r.clipped, 8000 - r.clipped, 0.25, sigmas=6.0)
    # only bytes of migrating pages are ever written, and in the order (layer, step, page) the first migrating page
    # is the one that proposal index 0 names
    mig = (X[:, 1:] != X[:, :-1]) & tr.persist[None, 1:].astype(bool) & (tr.alive[None, 1:].astype(bool) | tr.alive[None, :-1].astype(bool))
    assert not (r.Y[:, 1:][~mig]).any() and not r.Y[:, 0].any()
    assert r.Y.any()


def test_draw_move_second_and_third_block_feed_span_victim_direction_and_u():
    tr = _mini(L=7, N=50, P=90)
    seed, chain, mi = 0x0123_4567_89AB_CDEF, 5, (3 << 32) | 17
    m, u = O.draw_moves(tr, chain, mi, 1, seed=seed, stream0=8, max_len=11)
    key = [seed & 0xFFFFFFFF, seed >> 32]
    b = [int(x) for x in O.philox4x32_10([mi & 0xFFFFFFFF, mi >> 32, chain, 9], key)]
    c = [int(x) for x in O.philox4x32_10([mi & 0xFFFFFFFF, mi >> 32, chain, 10], key)]
    assert (m["len"][0], m["layer2"][0], m["page2"][0], m["dsel"][0]) == (
        1 + (b[0] * 11 >> 32), b[1] * 7 >> 32, b[2] * 90 >> 32, b[3] >> 30)
    assert u[0] == ((c[0] << 20 | c[1] >> 12) + 0.5) * 2.0 ** -52


def test_draw_move_frequencies():
    n = 200_000
    L, N, P, max_len = 5, 12, 37, 9
    m, u = O.draw_moves(_mini(L=L, N=N, P=P), 3, 0, n, seed=77, max_len=max_len)
    # the three operators at 0.4, 0.4, 0.2 (Sec. III-B)
    for op, p in ((0, 0.4), (1, 0.4), (2, 0.2)):
        assert _within((m["op"] == op).sum(), n, p), op
    # every index uniform on exactly its range
    for name, size in (("layer", L), ("page", P), ("n1", N), ("layer2", L), ("page2", P), ("dsel", 4)):
        cnt = np.bincount(m[name], minlength=size)
        assert len(cnt) == size and all(_within(k, n, 1.0 / size) for k in cnt), name
    # spans 1 .. max_len, each equally often
    cnt = np.bincount(m["len"], minlength=max_len + 1)
    assert len(cnt) == max_len + 1 and cnt[0] == 0 and all(_within(k, n, 1.0 / max_len) for k in cnt[1:])
    # the acceptance draw: inside (0, 1), mean 1/2, variance 1/12, every decile equally often
    assert u.min() > 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4.0 * math.sqrt(1 / 12 / n) and abs(u.var() - 1 / 12) < 0.002
    assert all(_within(k, n, 0.1) for k in np.bincount((u * 10).astype(int), minlength=10))
    # fields do not lean on each other: operator against direction, span against step, page against victim
    for a, b, sa, sb in (("op", "dsel", 3, 4), ("len", "n1", max_len + 1, N), ("layer", "layer2", L, L)):
        joint = np.zeros((sa, sb))
        np.add.at(joint, (m[a], m[b]), 1)
        pa, pb = joint.sum(1) / n, joint.sum(0) / n
        for i in range(sa):
            for j in range(sb):
                if pa[i] * pb[j] > 0:
                    assert _within(joint[i, j], n, pa[i] * pb[j], 4.5), (a, b, i, j)
    # other shares are honoured as given
    m2, _ = O.draw_moves(_mini(L=L, N=N, P=P), 0, 0, 50_000, seed=5, op_prob=(0.1, 0.6, 0.3))
    for op, p in ((0, 0.1), (1, 0.6), (2, 0.3)):
        assert _within((m2["op"] == op).sum(), 50_000, p), op
    # a proposal depends on (seed, chain, move) only and differs between chains and between moves
    again, _ = O.draw_moves(_mini(L=L, N=N, P=P), 3, 1000, 50, seed=77, max_len=max_len)
    assert all((again[k] == m[k][1000:1050]).all() for k in again)
    other, _ = O.draw_moves(_mini(L=L, N=N, P=P), 4, 0, 50, seed=77, max_len=max_len)
    assert any((other[k] != m[k][:50]).any() for k in other)


def test_wr_propose_decoded_by_hand_from_the_published_block():
    # Proposal 0 on stream 0 under seed 0 is the first published vector 6627e8d5 e169c58d bc57ac4c 9b00dbd8:
    #   word 0 / 2^32 = 0.39905 < 0.4: a window move; top two bits of word 1 (0xe...) = 3: the last of
    #   (-2, -1, +1, +2); top bit of word 2 (0xb...) = 1: ratio up, used only by a ratio or diagonal move
    u_want = (0x9b00dbd8 + 0.5) / 2.0 ** 32
    ok, w2, r2, u = O.wr_proposals(5, 5, 0, 1, seed=0, stream=0)
    assert (ok[0], w2[0], r2[0], u[0]) == (1, 7, 5, u_want)
    ok, w2, r2, _ = O.wr_proposals(5, 5, 0, 1, seed=0, stream=0, op_prob=(0.39, 0.41, 0.2))     # a ratio move
    assert (ok[0], w2[0], r2[0]) == (1, 5, 6)
    ok, w2, r2, _ = O.wr_proposals(5, 5, 0, 1, seed=0, stream=0, op_prob=(0.39, 0.009, 0.601))  # diagonal
    assert (ok[0], w2[0], r2[0]) == (1, 7, 6)
    # proposals that leave 1 <= W <= w_max or 0 <= R <= 1 are refused
    assert O.wr_proposals(5, 5, 0, 1, seed=0, stream=0, w_max=6)[0][0] == 0
    assert O.wr_proposals(5, 5, 0, 1, seed=0, stream=0, w_max=7)[0][0] == 1
    assert O.wr_proposals(5, 10, 0, 1, seed=0, stream=0, op_prob=(0.39, 0.41, 0.2))[0][0] == 0


def test_wr_propose_frequencies():
    n = 200_000
    ok, w2, r2, u = O.wr_proposals(50, 5, 0, n, seed=9)
    assert ok.all()
    dw, dr = w2 - 50, r2 - 5
    # step sets: window by -2, -1, +1, +2 (never 0 on its own), ratio by one tenth up or down
    assert set(np.unique(dw)) == {-2, -1, 0, 1, 2} and set(np.unique(dr)) == {-1, 0, 1}
    window, ratio, diag = (dw != 0) & (dr == 0), (dw == 0) & (dr != 0), (dw != 0) & (dr != 0)
    assert not ((dw == 0) & (dr == 0)).any()
    for sel, p in ((window, 0.4), (ratio, 0.4), (diag, 0.2)):
        assert _within(sel.sum(), n, p)
    # the steps of each kind equally often, alone and in a diagonal move
    for sel in (window, diag):
        k = sel.sum()
        assert all(_within((dw[sel] == d).sum(), k, 0.25) for d in (-2, -1, 1, 2))
    for sel in (ratio, diag):
        assert _within((dr[sel] == 1).sum(), sel.sum(), 0.5)
    k = diag.sum()
    for d in (-2, -1, 1, 2):
        for e in (-1, 1):
            assert _within(((dw == d) & (dr == e)).sum(), k, 0.125, 4.5)
    assert u.min() > 0.0 and u.max() < 1.0 and abs(u.mean() - 0.5) < 4.0 * math.sqrt(1 / 12 / n)
    # u does not lean on the kind of move
    for sel in (window, ratio, diag):
        assert abs(u[sel].mean() - 0.5) < 4.5 * math.sqrt(1 / 12 / sel.sum())
    # at the edge of the grid exactly the proposals that would leave it are refused
    ok, w2, r2, _ = O.wr_proposals(1, 0, 0, 50_000, seed=10, w_max=2)
    ok50 = O.wr_proposals(50, 5, 0, 50_000, seed=10)
    dw, dr = ok50[1] - 50, ok50[2] - 5
    assert ((ok == 1) == ((dw >= 0) & (dw <= 1) & (dr >= 0))).all()
    assert (w2[ok == 1] == 1 + dw[ok == 1]).all() and (r2[ok == 1] == dr[ok == 1]).all()


def _flat_table(w_max, value):
    return np.full((w_max, 11), float(value))


def test_wr_search_on_given_cost_tables_by_hand():
    tr = W.config("tiny")      # the table is given in full, so the trace is never looked at
    # (a) every state costs the same: each proposal inside the grid has dT = 0 and is accepted, no proposal is
    # uphill so the start temperature is 0, and the best cost does not improve over the first level: the
    # stagnation rule (Sec. III-B: less than 0.1 % over a level) ends the walk there
    res, tab = O.wr_search(tr, w_max=40, total_moves=1000, n_levels=10, seed=3, w0=20, r10_0=5,
                           table=_flat_table(40, 2.5))
    assert (res.stop_reason, res.levels_done, res.proposals, res.c0) == (1, 1, 100, 0.0)
    assert res.accepted == res.proposals - res.out_of_range and res.evaluated == 0
    assert (res.best_w, res.best_r10, res.best_T, res.cur_T) == (20, 5, 2.5, 2.5)
    # (b) the start costs 1, every other state 2: each calibration proposal is uphill by exactly 1, so the
    # start temperature is 1 / (-ln 0.8) and a first uphill move is accepted with probability 0.8; with the
    # stagnation rule off the walk cools by 0.9 per level until 0.9^k < c_min_frac = 0.5, i.e. k = 7
    # (0.9^6 = 0.531, 0.9^7 = 0.478), and stops there for the temperature
    t = _flat_table(40, 2.0)
    t[19, 5] = 1.0
    res, _ = O.wr_search(tr, w_max=40, total_moves=1000, n_levels=10, seed=3, w0=20, r10_0=5, stop_rel=0.0,
                         c_min_frac=0.5, table=t)
    assert res.c0 == 1.0 / -math.log(0.8)
    assert (res.stop_reason, res.levels_done, res.proposals) == (2, 7, 700)
    assert (res.best_w, res.best_r10, res.best_T) == (20, 5, 1.0)
    # ... and with both rules off the budget ends it
    res, _ = O.wr_search(tr, w_max=40, total_moves=1000, n_levels=10, seed=3, w0=20, r10_0=5, stop_rel=0.0,
                         c_min_frac=0.0, table=t.copy())
    assert (res.stop_reason, res.levels_done, res.proposals) == (0, 9, 1000)
    # (c) the Metropolis rule at the start temperature: over many seeds, the first proposal (always uphill by
    # 1) is accepted 8 times in 10
    acc = sum(O.wr_search(tr, w_max=40, total_moves=1, n_levels=1, seed=s, w0=20, r10_0=5, stop_rel=0.0,
                          c_min_frac=0.0, table=t.copy())[0].accepted for s in range(6000))
    assert _within(acc, 6000, 0.8)
    # (d) a slope with the start at its top corner: no proposal inside the grid is uphill (c0 = 0), the walk
    # is a pure descent, so the current state is the best one and costs what the table says
    w_max = 30
    t = np.array([[1000.0 - (w + 1) - r for r in range(11)] for w in range(w_max)])
    res, _ = O.wr_search(tr, w_max=w_max, total_moves=60, n_levels=1, seed=4, w0=1, r10_0=0, stop_rel=0.0,
                         c_min_frac=0.0, table=t.copy())
    assert res.c0 == 0.0 and res.stop_reason == 0 and res.proposals == 60
    assert (res.best_w, res.best_r10) == (res.cur_w, res.cur_r10) and res.best_T == res.cur_T
    assert res.cur_T == t[res.cur_w - 1, res.cur_r10] and res.cur_T < 1000.0 - 1
    # accepted moves are exactly the proposals inside the grid that do not go up; each lowers W + R by 0..3
    assert 0 < res.accepted <= res.proposals - res.out_of_range
    assert 1000.0 - res.cur_T - 1 <= 3 * res.accepted
