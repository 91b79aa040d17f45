"""ctypes front end of the CPU oracle (oracle/kvp_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
cpu_baseline leg call this; the GPU library never does and shares nothing with
it.  Every array that goes in or out is one byte per boolean.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvp_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liborc.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]


SANITIZE_FLAGS = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
_LIB_SAN = os.path.join(_HERE, "_build", "liborc_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle.  sanitize=True builds a second library with AddressSanitizer and
    UBSan (any finding aborts); a process loads it with libasan preloaded and
    KVP_ORACLE_SANITIZE=1 in its environment."""
    out = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(out), exist_ok=True)
        tmp = out + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", *CFLAGS, *(SANITIZE_FLAGS if sanitize else []), "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, out)
    return out


class _Problem(C.Structure):
    _fields_ = [("L", C.c_int32), ("N", C.c_int32), ("P", C.c_int32), ("K", C.c_int32),
                ("access", C.c_void_p), ("alive", C.c_void_p), ("persist", C.c_void_p),
                ("written", C.c_void_p), ("plane_bytes", C.c_uint64 * 8),
                ("page_bytes", C.c_uint64), ("token_bytes", C.c_uint64),
                ("bw_hbm", C.c_double), ("bw_link", C.c_double), ("bw_dram", C.c_double),
                ("cap_pages", C.c_uint64)]


class _Move(C.Structure):
    _fields_ = [(k, C.c_uint32) for k in ("op", "layer", "page", "n1", "len", "layer2", "page2", "dsel")]


class _SAParams(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("total_moves", C.c_uint64), ("move_begin", C.c_uint64),
                ("move_end", C.c_uint64), ("n_levels", C.c_uint32), ("max_len", C.c_uint32),
                ("p0", C.c_double), ("alpha", C.c_double), ("op_prob", C.c_double * 3), ("per_slot", C.c_uint32)]


class _SAState(C.Structure):
    _fields_ = [("T_cur", C.c_double), ("T_best", C.c_double), ("C0", C.c_double), ("C", C.c_double),
                ("level", C.c_uint32), ("accepted", C.c_uint64), ("uphill", C.c_uint64),
                ("null_moves", C.c_uint64), ("clipped", C.c_uint64), ("improved", C.c_uint64),
                ("uphill_seen", C.c_uint64)]


class _WRParams(C.Structure):
    _fields_ = [("w_max", C.c_uint32), ("w0", C.c_uint32), ("r10_0", C.c_uint32), ("n_levels", C.c_uint32),
                ("seed", C.c_uint64), ("total_moves", C.c_uint64), ("p0", C.c_double), ("alpha", C.c_double),
                ("op_prob", C.c_double * 3), ("stop_rel", C.c_double), ("c_min_frac", C.c_double)]


class WRResult(C.Structure):
    _fields_ = [("best_w", C.c_uint32), ("best_r10", C.c_uint32), ("cur_w", C.c_uint32), ("cur_r10", C.c_uint32),
                ("levels_done", C.c_uint32), ("stop_reason", C.c_uint32), ("proposals", C.c_uint64),
                ("accepted", C.c_uint64), ("out_of_range", C.c_uint64), ("evaluated", C.c_uint64),
                ("best_T", C.c_double), ("cur_T", C.c_double), ("c0", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build(sanitize=os.environ.get("KVP_ORACLE_SANITIZE") == "1"))
        L.orc_csum.restype = C.c_double
        L.orc_csum.argtypes = [C.c_void_p, C.c_size_t]
        L.orc_step_time.restype = C.c_double
        L.orc_step_time.argtypes = [C.POINTER(_Problem), C.c_void_p]
        L.orc_score.restype = C.c_double
        L.orc_score.argtypes = [C.POINTER(_Problem), C.c_void_p, C.POINTER(C.c_uint32), C.c_void_p,
                                C.c_void_p, C.c_void_p]
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_delta.restype = C.c_int
        L.orc_delta.argtypes = [C.POINTER(_Problem), C.c_void_p, C.POINTER(_Move), C.POINTER(C.c_double),
                                C.POINTER(C.c_int), C.c_void_p, C.c_void_p]
        L.orc_resolve.restype = C.c_int
        L.orc_resolve.argtypes = [C.POINTER(_Problem), C.c_void_p, C.c_void_p, C.POINTER(_Move),
                                  C.c_void_p, C.c_void_p, C.POINTER(C.c_int)]
        L.orc_resolve_strict.restype = C.c_int
        L.orc_resolve_strict.argtypes = L.orc_resolve.argtypes
        L.orc_slot_occupancy.restype = None
        L.orc_slot_occupancy.argtypes = [C.POINTER(_Problem), C.c_void_p, C.c_void_p]
        L.orc_score_slots.restype = C.c_double
        L.orc_score_slots.argtypes = [C.POINTER(_Problem), C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32), C.c_void_p,
                                      C.c_void_p]
        L.orc_slot_bytes.restype = None
        L.orc_slot_bytes.argtypes = [C.POINTER(_Problem), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.orc_draw_slot_move.restype = None
        L.orc_draw_slot_move.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                         C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_double)]
        L.orc_refine_slots.restype = C.c_int
        L.orc_refine_slots.argtypes = [C.POINTER(_Problem), C.POINTER(_SAParams), C.c_uint32, C.c_void_p, C.c_void_p,
                                       C.POINTER(_SAState)]
        L.orc_init_static_frequency.argtypes = [C.POINTER(_Problem), C.c_void_p]
        L.orc_init_recency.argtypes = [C.POINTER(_Problem), C.c_void_p]
        L.orc_init_static_fill.argtypes = [C.POINTER(_Problem), C.c_void_p]
        L.orc_strict_excess.restype = C.c_uint32
        L.orc_strict_excess.argtypes = [C.POINTER(_Problem), C.c_void_p]
        L.orc_bruteforce.restype = C.c_int
        L.orc_bruteforce.argtypes = [C.POINTER(_Problem), C.POINTER(C.c_double), C.c_void_p,
                                     C.POINTER(C.c_uint64)]
        L.orc_anneal_chain.restype = C.c_int
        L.orc_anneal_chain.argtypes = [C.POINTER(_Problem), C.POINTER(_SAParams), C.c_uint32, C.c_void_p,
                                       C.c_void_p, C.POINTER(_SAState)]
        L.orc_wr_policy.argtypes = [C.POINTER(_Problem), C.c_uint32, C.c_uint32, C.c_void_p]
        L.orc_exchange.restype = C.c_uint32
        L.orc_exchange.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_draw_move.restype = None
        L.orc_draw_move.argtypes = [C.POINTER(_Problem), C.POINTER(_SAParams), C.c_uint32, C.c_uint64, C.c_uint32,
                                    C.POINTER(_Move), C.POINTER(C.c_double)]
        L.orc_wr_propose.restype = C.c_int
        L.orc_wr_propose.argtypes = [C.POINTER(_WRParams), C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                     C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_double)]
        L.orc_wr_search.restype = C.c_uint64
        L.orc_wr_search.argtypes = [C.POINTER(_Problem), C.POINTER(_WRParams), C.c_void_p, C.POINTER(WRResult)]
        _lib = L
    return _lib


def _u8(a, shape):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


class Problem:
    """Holds the boolean trace arrays alive for the C side."""

    def __init__(self, tr):
        self.L, self.N, self.P, self.K = tr.L, tr.N, tr.P, tr.K
        self.access = _u8(tr.access, (tr.L, tr.N, tr.K, tr.P))
        self.alive = _u8(tr.alive, (tr.N, tr.P))
        self.persist = _u8(tr.persist, (tr.N, tr.P))
        self.written = _u8(tr.written, (tr.N, tr.P))
        al = self.alive.astype(bool)
        assert not (self.access.astype(bool) & ~al[None, :, None, :]).any(), "access outside alive"
        assert not (self.written.astype(bool) & ~al).any(), "written outside alive"
        assert not self.persist[0].any()
        assert not (self.persist[1:].astype(bool) & ~(al[1:] & al[:-1])).any(), "persist outside alive"
        assert 1 <= tr.K <= 8 and len(tr.plane_bytes) == tr.K
        c = _Problem()
        c.L, c.N, c.P, c.K = tr.L, tr.N, tr.P, tr.K
        c.access = self.access.ctypes.data
        c.alive = self.alive.ctypes.data
        c.persist = self.persist.ctypes.data
        c.written = self.written.ctypes.data
        for k in range(tr.K):
            c.plane_bytes[k] = int(tr.plane_bytes[k])
        c.page_bytes, c.token_bytes = int(tr.page_bytes), int(tr.token_bytes)
        c.bw_hbm, c.bw_link, c.bw_dram = float(tr.bw_hbm), float(tr.bw_link), float(tr.bw_dram)
        c.cap_pages = int(tr.cap_pages)
        self.c = c

    @property
    def shape(self):
        return (self.L, self.N, self.P)


def _problem(tr) -> Problem:
    return tr if isinstance(tr, Problem) else Problem(tr)


def csum(v) -> float:
    v = np.ascontiguousarray(v, dtype=np.float64)
    return lib().orc_csum(v.ctypes.data, v.size)


def step_time(tr, b6) -> float:
    q = _problem(tr)
    b = np.ascontiguousarray(b6, dtype=np.uint64)
    assert b.shape == (6,)
    return lib().orc_step_time(C.byref(q.c), b.ctypes.data)


@dataclass
class Score:
    cost: float
    excess: int          # max overshoot of the capacity (pages), bit 31: bits on dead pages
    step_bytes: np.ndarray   # [L][N][6] = hr, er, hw, ew, mi, mo
    step_t: np.ndarray       # [L][N]
    occ: np.ndarray          # [N]

    @property
    def feasible(self):
        return (self.excess & 0x7FFFFFFF) == 0


def score(tr, X) -> Score:
    q = _problem(tr)
    X = _u8(X, q.shape)
    ex = C.c_uint32(0)
    sb = np.zeros((q.L, q.N, 6), dtype=np.uint64)
    st = np.zeros((q.L, q.N), dtype=np.float64)
    occ = np.zeros(q.N, dtype=np.uint32)
    T = lib().orc_score(C.byref(q.c), X.ctypes.data, C.byref(ex), sb.ctypes.data, st.ctypes.data,
                        occ.ctypes.data)
    return Score(T, ex.value, sb, st, occ)


def cost(tr, X) -> float:
    q = _problem(tr)
    X = _u8(X, q.shape)
    return lib().orc_score(C.byref(q.c), X.ctypes.data, None, None, None, None)


def strict_excess(tr, X) -> int:
    """Largest overshoot of the capacity when it is counted after every (step, layer) slot."""
    q = _problem(tr)
    X = _u8(X, q.shape)
    return int(lib().orc_strict_excess(C.byref(q.c), X.ctypes.data))


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def _move(m) -> _Move:
    mv = _Move()
    for k in ("op", "layer", "page", "n1", "len", "layer2", "page2", "dsel"):
        setattr(mv, k, int(m[k]))
    return mv


def delta(tr, X, move):
    """(verdict, dT, base, f1, f2) of one raw move, the slow way."""
    q = _problem(tr)
    X = _u8(X, q.shape)
    d = C.c_double(0.0)
    base = C.c_int(0)
    f1 = np.zeros(q.N, dtype=np.uint8)
    f2 = np.zeros(q.N, dtype=np.uint8)
    v = lib().orc_delta(C.byref(q.c), X.ctypes.data, C.byref(_move(move)), C.byref(d), C.byref(base),
                        f1.ctypes.data, f2.ctypes.data)
    return v, d.value, base.value, f1, f2


def slot_occupancy(tr, X) -> np.ndarray:
    """[N][L]: pages in the pool after layer l of token step n has taken its placement (Eq. 5 read at
    every inference step)."""
    q = _problem(tr)
    X = _u8(X, q.shape)
    tab = np.zeros((q.N, q.L), dtype=np.uint32)
    lib().orc_slot_occupancy(C.byref(q.c), X.ctypes.data, tab.ctypes.data)
    return tab


@dataclass
class SlotScore:
    cost: float
    excess: int          # largest overshoot of the pool over all inference steps; bit 31: bits on dead pages; bit 30: a Y out of range
    slot_t: np.ndarray   # [N*L] latency of inference step g = n*L + l
    pool: np.ndarray     # [N*L] pages in HBM after step g


def score_slots(tr, X, Y) -> SlotScore:
    """A placement X whose migrating pages move in the inference steps that Y names: a page of layer l that changes
    tier going into step n moves in step n*L + l - Y[l][n][p]."""
    q = _problem(tr)
    X, Y = _u8(X, q.shape), _u8(Y, q.shape)
    ex = C.c_uint32(0)
    st = np.zeros(q.N * q.L, dtype=np.float64)
    pool = np.zeros(q.N * q.L, dtype=np.uint32)
    T = lib().orc_score_slots(C.byref(q.c), X.ctypes.data, Y.ctypes.data, C.byref(ex), st.ctypes.data, pool.ctypes.data)
    return SlotScore(T, ex.value, st, pool)


def slot_bytes(tr, X, Y, g):
    """{|H^r|, |E^r|, |H^w|, |E^w|, |M^i|, |M^o|} of inference step g."""
    q = _problem(tr)
    X, Y = _u8(X, q.shape), _u8(Y, q.shape)
    out = np.zeros(6, dtype=np.uint64)
    lib().orc_slot_bytes(C.byref(q.c), X.ctypes.data, Y.ctypes.data, int(g), out.ctypes.data)
    return out


@dataclass
class SlotWalk:
    chain: int
    Y: np.ndarray
    T_cur: float
    T_best: float
    C0: float
    accepted: int
    uphill: int
    null_moves: int
    clipped: int
    improved: int
    state: object = None


def draw_slot_moves(chain, first, count, *, seed, stream, M, L):
    """Proposals first .. first+count-1 of the annealing over migration steps: (index of the migrating page, new Y, u)."""
    idx, y, us = np.zeros(count, np.int64), np.zeros(count, np.int64), np.zeros(count)
    a, b, u, f = C.c_uint32(0), C.c_uint32(0), C.c_double(0.0), lib().orc_draw_slot_move
    for j in range(count):
        f(int(seed), int(chain), int(first) + j, int(stream), int(M), int(L), C.byref(a), C.byref(b), C.byref(u))
        idx[j], y[j], us[j] = a.value, b.value, u.value
    return idx, y, us


def refine_slots(tr, chain, X, Y0, *, seed, total_moves, move_begin=0, move_end=None, n_levels=100, p0=0.8, alpha=0.9,
                 resume=None) -> SlotWalk:
    """Annealing over the migration steps Y of the fixed placement X (one chain)."""
    q = _problem(tr)
    sp = _SAParams()
    sp.seed, sp.total_moves = int(seed), int(total_moves)
    sp.move_begin = int(move_begin)
    sp.move_end = int(total_moves if move_end is None else move_end)
    sp.n_levels, sp.max_len, sp.p0, sp.alpha = int(n_levels), 1, float(p0), float(alpha)
    for i, v in enumerate((0.4, 0.4, 0.2)):
        sp.op_prob[i] = v
    X = _u8(X, q.shape)
    if resume is None:
        Y, st = np.array(_u8(Y0, q.shape), copy=True), _SAState()
    else:
        Y, st = resume.Y.copy(), resume.state
    rc = lib().orc_refine_slots(C.byref(q.c), C.byref(sp), int(chain), X.ctypes.data, Y.ctypes.data, C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_refine_slots failed ({rc}): bad parameters or a start that overfills an inference step")
    return SlotWalk(int(chain), Y, st.T_cur, st.T_best, st.C0, st.accepted, st.uphill, st.null_moves, st.clipped,
                    st.improved, st)


def resolve(tr, X, move, per_slot=False):
    """(verdict, f1, f2, base): the steps at which a raw move flips its page (f1) and its victim (f2),
    under the capacity once per token step or, per_slot, at every inference step."""
    q = _problem(tr)
    X = _u8(X, q.shape)
    f1 = np.zeros(q.N, dtype=np.uint8)
    f2 = np.zeros(q.N, dtype=np.uint8)
    base = C.c_int(0)
    if per_slot:
        view = slot_occupancy(q, X)
        v = lib().orc_resolve_strict(C.byref(q.c), X.ctypes.data, view.ctypes.data, C.byref(_move(move)),
                                     f1.ctypes.data, f2.ctypes.data, C.byref(base))
    else:
        view = np.ascontiguousarray(score(q, X).occ, dtype=np.uint32)
        v = lib().orc_resolve(C.byref(q.c), X.ctypes.data, view.ctypes.data, C.byref(_move(move)),
                              f1.ctypes.data, f2.ctypes.data, C.byref(base))
    return v, f1, f2, base.value


def apply_move(tr, X, move):
    """Schedule after the move (a copy), and the verdict."""
    q = _problem(tr)
    v, _, _, f1, f2 = delta(q, X, move)
    Y = np.array(X, dtype=np.uint8, copy=True)
    if v != 2:
        Y[int(move["layer"]), :, int(move["page"])] ^= f1
        Y[int(move["layer2"]), :, int(move["page2"])] ^= f2
    return Y, v


def init_static_frequency(tr) -> np.ndarray:
    q = _problem(tr)
    X = np.zeros(q.shape, dtype=np.uint8)
    lib().orc_init_static_frequency(C.byref(q.c), X.ctypes.data)
    return X


def init_recency(tr) -> np.ndarray:
    q = _problem(tr)
    X = np.zeros(q.shape, dtype=np.uint8)
    lib().orc_init_recency(C.byref(q.c), X.ctypes.data)
    return X


def init_static_fill(tr) -> np.ndarray:
    q = _problem(tr)
    X = np.zeros(q.shape, dtype=np.uint8)
    lib().orc_init_static_fill(C.byref(q.c), X.ctypes.data)
    return X


def wr_policy(tr, W: int, r10: int) -> np.ndarray:
    """Schedule of the (W, R = r10/10) look-ahead policy, bool bytes [L][N][P]."""
    q = _problem(tr)
    X = np.zeros(q.shape, dtype=np.uint8)
    lib().orc_wr_policy(C.byref(q.c), int(W), int(r10), X.ctypes.data)
    return X


def wr_search(tr, w_max, total_moves, n_levels=20, seed=0, w0=1, r10_0=5, p0=0.8, alpha=0.9,
              op_prob=(0.4, 0.4, 0.2), stop_rel=1e-3, c_min_frac=1e-3, table=None):
    """The annealing over (W, R).  Returns (WRResult, table [w_max][11] of the costs evaluated, -1 elsewhere)."""
    q = _problem(tr)
    sp = _WRParams(int(w_max), int(w0), int(r10_0), int(n_levels), int(seed), int(total_moves), float(p0),
                   float(alpha), (C.c_double * 3)(*op_prob), float(stop_rel), float(c_min_frac))
    if table is None:
        table = np.full((int(w_max), 11), -1.0)
    res = WRResult()
    assert table.dtype == np.float64 and table.shape == (int(w_max), 11) and table.flags.c_contiguous
    lib().orc_wr_search(C.byref(q.c), C.byref(sp), table.ctypes.data, C.byref(res))
    return res, table


def brute_force(tr):
    """(optimal cost, an optimal schedule, number of feasible schedules)."""
    q = _problem(tr)
    X = np.zeros(q.shape, dtype=np.uint8)
    best = C.c_double(0.0)
    nf = C.c_uint64(0)
    rc = lib().orc_bruteforce(C.byref(q.c), C.byref(best), X.ctypes.data, C.byref(nf))
    if rc != 0:
        raise ValueError("instance too large for exhaustive search")
    return best.value, X, nf.value


@dataclass
class ChainResult:
    chain: int
    X: np.ndarray
    best_X: np.ndarray
    best_cost: float      # exact re-score of best_X
    T_cur: float
    T_best: float         # running value (accumulated deltas)
    C0: float
    accepted: int
    uphill: int
    null_moves: int
    clipped: int
    improved: int
    state: object = None


def anneal_chain(tr, chain, X0, *, seed, total_moves, move_begin=0, move_end=None, n_levels=100,
                 max_len=63, p0=0.8, alpha=0.9, op_prob=(0.4, 0.4, 0.2), resume=None, per_slot=False) -> ChainResult:
    q = _problem(tr)
    sp = _SAParams()
    sp.per_slot = int(bool(per_slot))
    sp.seed, sp.total_moves = int(seed), int(total_moves)
    sp.move_begin = int(move_begin)
    sp.move_end = int(total_moves if move_end is None else move_end)
    sp.n_levels, sp.max_len, sp.p0, sp.alpha = int(n_levels), int(max_len), float(p0), float(alpha)
    for i in range(3):
        sp.op_prob[i] = float(op_prob[i])
    if resume is None:
        X = np.array(_u8(X0, q.shape), copy=True)
        best = np.zeros(q.shape, dtype=np.uint8)
        st = _SAState()
    else:
        X, best, st = resume.X.copy(), resume.best_X.copy(), resume.state
    rc = lib().orc_anneal_chain(C.byref(q.c), C.byref(sp), int(chain), X.ctypes.data, best.ctypes.data,
                                C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_anneal_chain failed ({rc}): bad parameters or infeasible start")
    return ChainResult(int(chain), X, best, cost(q, best), st.T_cur, st.T_best, st.C0, st.accepted,
                       st.uphill, st.null_moves, st.clipped, st.improved, st)


def draw_moves(tr, chain, first, count, *, seed, stream0=0, max_len=63, op_prob=(0.4, 0.4, 0.2)):
    """Proposals first .. first+count-1 of `chain` as the annealer draws them: a dict of uint32 arrays
    (the fields of a raw move) and the acceptance draws u."""
    q = _problem(tr)
    sp = _SAParams()
    sp.seed, sp.max_len = int(seed), int(max_len)
    for i in range(3):
        sp.op_prob[i] = float(op_prob[i])
    names = ("op", "layer", "page", "n1", "len", "layer2", "page2", "dsel")
    out = {k: np.zeros(count, np.uint32) for k in names}
    us = np.zeros(count)
    m, u, f = _Move(), C.c_double(0.0), lib().orc_draw_move
    for j in range(count):
        f(C.byref(q.c), C.byref(sp), int(chain), int(first) + j, int(stream0), C.byref(m), C.byref(u))
        for k in names:
            out[k][j] = getattr(m, k)
        us[j] = u.value
    return out, us


def wr_proposals(w, r10, first, count, *, seed, stream=16, w_max=1 << 20, op_prob=(0.4, 0.4, 0.2)):
    """Proposals first .. first+count-1 of the (W, R) walk, all from the state (w, r10): arrays
    in_range (0/1), w2, r2 (valid where in_range) and u."""
    sp = _WRParams(int(w_max), int(w), int(r10), 1, int(seed), 0, 0.8, 0.9, (C.c_double * 3)(*op_prob), 0.0, 0.0)
    ok = np.zeros(count, np.int32)
    w2s, r2s, us = np.zeros(count, np.int64), np.zeros(count, np.int64), np.zeros(count)
    w2, r2, u, f = C.c_uint32(0), C.c_uint32(0), C.c_double(0.0), lib().orc_wr_propose
    for j in range(count):
        ok[j] = f(C.byref(sp), int(first) + j, int(stream), int(w), int(r10), C.byref(w2), C.byref(r2), C.byref(u))
        w2s[j], r2s[j], us[j] = w2.value, r2.value, u.value
    return ok, w2s, r2s, us


def temper(results, factors) -> None:
    """Spread the chains over a ladder of temperatures: chain i's current and initial
    temperature are multiplied by factors[i].  For results of a first `anneal_chain`
    slice with at least one move: a slice that begins at move 0 calibrates anew."""
    for r, f in zip(results, factors):
        r.state.C = r.state.C * float(f)
        r.state.C0 = r.state.C0 * float(f)
        r.C0 = r.state.C0


def exchange_step(seed: int, rnd: int, T, C, C0):
    """One replica-exchange round on plain arrays (see orc_exchange): returns (C, C0, pairs traded)."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    C1 = np.array(C, dtype=np.float64, copy=True)
    C01 = np.array(C0, dtype=np.float64, copy=True)
    n = lib().orc_exchange(int(seed), int(rnd), len(T), T.ctypes.data, C1.ctypes.data, C01.ctypes.data)
    return C1, C01, int(n)


def exchange(results, seed: int, rnd: int) -> int:
    """Replica exchange between neighbouring chains of `results` (in list order), in place: the
    chains carry on from the traded temperatures at their next `anneal_chain(resume=...)`."""
    C1, C01, n = exchange_step(seed, rnd, [r.state.T_cur for r in results], [r.state.C for r in results],
                               [r.state.C0 for r in results])
    for r, c, c0 in zip(results, C1, C01):
        r.state.C, r.state.C0, r.C0 = float(c), float(c0), float(c0)
    return n


def anneal(tr, chains, X0, threads: int = 1, **kw):
    """Run several chains (ids in `chains`); X0 is one schedule for all or a
    list with one per chain.  Returns the list of ChainResult and the index of
    the best (lowest exact cost, ties to the lowest chain id)."""
    q = _problem(tr)
    chains = list(chains)
    X0s = X0 if isinstance(X0, (list, tuple)) else [X0] * len(chains)
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            res = list(ex.map(lambda a: anneal_chain(q, a[0], a[1], **kw), zip(chains, X0s)))
    else:
        res = [anneal_chain(q, c, x, **kw) for c, x in zip(chains, X0s)]
    best = min(range(len(res)), key=lambda i: (res[i].best_cost, res[i].chain))
    return res, best
