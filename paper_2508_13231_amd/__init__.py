"""Python binding of libkvp (include/kvp.h): argument marshalling only.

Every step of the scoring and annealing path runs in the library's HIP kernels
on an MI355X.  There is no CPU fallback: importing this package is cheap, but
the first call that needs the library raises if libkvp.so has not been built
(`python -m paper_2508_13231_amd.build`).

The functions carry the names of the C entry points.  Device arrays are torch
tensors on the context's GPU (torch is used for device memory and streams
only); host arrays are numpy.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("KVP_LIBRARY") or os.path.join(_HERE, "libkvp.so")    # the in-tree build unless told otherwise

KVP_OK, KVP_EINVAL, KVP_ENOTRACE, KVP_ENOMEM, KVP_EHIP = 0, -1, -2, -3, -4
KVP_ESHAPE, KVP_ETRACE, KVP_ENOCHAINS, KVP_EINFEASIBLE = -5, -6, -7, -8
KVP_MAX_LEN = 63
KVP_INIT_EMPTY, KVP_INIT_GIVEN, KVP_INIT_BROADCAST, KVP_INIT_CONTINUE = 0, 1, 2, 3
KVP_CAPACITY_PER_STEP, KVP_CAPACITY_PER_SLOT = 0, 1
KVP_OP_SET, KVP_OP_SWAP, KVP_OP_SHIFT = 0, 1, 2              # kvp_move.op
KVP_MOVE_OK, KVP_MOVE_CLIPPED, KVP_MOVE_NULL = 0, 1, 2       # verdicts of kvp_delta_score
KVP_MOVE_OK, KVP_MOVE_CLIPPED, KVP_MOVE_NULL = 0, 1, 2

EXPORTS = ["kvp_create", "kvp_destroy", "kvp_trace_upload", "kvp_score", "kvp_delta_score", "kvp_anneal",
           "kvp_best", "kvp_chain_placement", "kvp_chain_stats", "kvp_plane_unit", "kvp_strerror", "kvp_last_hip_error",
           "kvp_set_score_kernel", "kvp_set_anneal_lookahead", "kvp_set_capacity_mode", "kvp_set_anneal_log_entries", "kvp_set_generator_batch_bytes", "kvp_score_kernel_used", "kvp_baseline", "kvp_wr_policy",
           "kvp_wr_search", "kvp_strict_excess", "kvp_temper", "kvp_exchange", "kvp_score_static", "kvp_score_slots",
           "kvp_refine_slots"]
KVP_STATIC_SCRATCH_BYTES = 32 << 20


class kvp_wr_params(C.Structure):
    _fields_ = [("w_max", C.c_uint32), ("w0", C.c_uint32), ("r10_0", C.c_uint32), ("n_levels", C.c_uint32),
                ("seed", C.c_uint64), ("total_moves", C.c_uint64), ("p0", C.c_double), ("alpha", C.c_double),
                ("op_prob", C.c_double * 3), ("stop_rel", C.c_double), ("c_min_frac", C.c_double)]


class kvp_wr_result(C.Structure):
    _fields_ = [("best_w", C.c_uint32), ("best_r10", C.c_uint32), ("cur_w", C.c_uint32), ("cur_r10", C.c_uint32),
                ("levels_done", C.c_uint32), ("stop_reason", C.c_uint32), ("proposals", C.c_uint64),
                ("accepted", C.c_uint64), ("out_of_range", C.c_uint64), ("evaluated", C.c_uint64),
                ("best_T", C.c_double), ("cur_T", C.c_double), ("c0", C.c_double)]


class kvp_problem(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("n_steps", C.c_uint32), ("n_pages", C.c_uint32),
                ("n_words", C.c_uint32), ("n_planes", C.c_uint32), ("reserved", C.c_uint32),
                ("plane_bytes", C.c_uint64 * 8), ("page_bytes", C.c_uint64), ("token_bytes", C.c_uint64),
                ("bw_hbm", C.c_double), ("bw_link", C.c_double), ("bw_dram", C.c_double),
                ("cap_pages", C.c_uint64)]


class kvp_anneal_params(C.Structure):
    _fields_ = [("n_chains", C.c_uint32), ("n_levels", C.c_uint32), ("seed", C.c_uint64),
                ("total_moves", C.c_uint64), ("moves", C.c_uint64), ("max_len", C.c_uint32),
                ("init_mode", C.c_uint32), ("p0", C.c_double), ("alpha", C.c_double),
                ("op_prob", C.c_double * 3)]


class kvp_chain_stats_t(C.Structure):
    _fields_ = [("t_cur", C.c_double), ("t_best", C.c_double), ("c0", C.c_double), ("c", C.c_double),
                ("moves_done", C.c_uint64), ("accepted", C.c_uint64), ("uphill", C.c_uint64),
                ("null_moves", C.c_uint64), ("clipped", C.c_uint64), ("improved", C.c_uint64)]


class KvpError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        msg = f"{what}: {strerror(code)} ({code})"
        if code in (KVP_EHIP, KVP_ENOMEM):
            line = C.c_int(0)
            msg += f" [hipError {lib().kvp_last_hip_error(C.byref(line))} at library line {line.value}]"
        super().__init__(msg)


_lib = None


def lib():
    """The loaded libkvp.so.  Raises if it is not built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2508_13231_amd.build`")
        # torch ships its own HIP runtime; it must be in the process before libkvp.so is
        # mapped, so that both use the same one (two HIP runtimes in a process do not work)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, u32, i32 = C.c_void_p, C.c_uint32, C.c_int
        L.kvp_create.restype = i32
        L.kvp_create.argtypes = [C.POINTER(vp), i32, vp]
        L.kvp_destroy.restype = None
        L.kvp_destroy.argtypes = [vp]
        L.kvp_trace_upload.restype = i32
        L.kvp_trace_upload.argtypes = [vp, C.POINTER(kvp_problem), vp, vp, vp, vp]
        L.kvp_score.restype = i32
        L.kvp_score.argtypes = [vp, vp, u32, vp, vp, vp, vp]
        L.kvp_score_static.restype = i32
        L.kvp_score_static.argtypes = [vp, vp, u32, vp, vp]
        L.kvp_delta_score.restype = i32
        L.kvp_delta_score.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp]
        L.kvp_anneal.restype = i32
        L.kvp_anneal.argtypes = [vp, C.POINTER(kvp_anneal_params), vp]
        L.kvp_best.restype = i32
        L.kvp_best.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u32), vp, vp]
        L.kvp_chain_placement.restype = i32
        L.kvp_chain_placement.argtypes = [vp, u32, i32, vp]
        L.kvp_chain_stats.restype = i32
        L.kvp_chain_stats.argtypes = [vp, vp]
        L.kvp_plane_unit.restype = C.c_uint64
        L.kvp_plane_unit.argtypes = [vp]
        L.kvp_strerror.restype = C.c_char_p
        L.kvp_strerror.argtypes = [i32]
        L.kvp_strict_excess.restype = i32
        L.kvp_strict_excess.argtypes = [vp, vp, C.c_uint32, vp]
        L.kvp_score_slots.restype = i32
        L.kvp_score_slots.argtypes = [vp, vp, vp, C.c_uint32, vp, vp]
        L.kvp_refine_slots.restype = i32
        L.kvp_refine_slots.argtypes = [vp, vp, vp, vp, vp]
        L.kvp_temper.restype = i32
        L.kvp_temper.argtypes = [vp, vp]
        L.kvp_exchange.restype = i32
        L.kvp_exchange.argtypes = [vp, C.c_uint64, vp]
        L.kvp_set_anneal_lookahead.restype = i32
        L.kvp_set_anneal_lookahead.argtypes = [vp, i32]
        L.kvp_set_capacity_mode.restype = i32
        L.kvp_set_capacity_mode.argtypes = [vp, i32]
        L.kvp_set_anneal_log_entries.restype = i32
        L.kvp_set_anneal_log_entries.argtypes = [vp, C.c_uint64]
        L.kvp_set_generator_batch_bytes.restype = i32
        L.kvp_set_generator_batch_bytes.argtypes = [vp, C.c_uint64]
        L.kvp_set_score_kernel.restype = i32
        L.kvp_set_score_kernel.argtypes = [vp, i32]
        L.kvp_wr_policy.restype = i32
        L.kvp_wr_policy.argtypes = [vp, C.c_uint32, vp, vp, vp]
        L.kvp_wr_search.restype = i32
        L.kvp_wr_search.argtypes = [vp, C.POINTER(kvp_wr_params), vp, C.POINTER(kvp_wr_result), vp]
        L.kvp_baseline.restype = i32
        L.kvp_baseline.argtypes = [vp, i32, vp]
        L.kvp_score_kernel_used.restype = i32
        L.kvp_score_kernel_used.argtypes = [vp]
        L.kvp_last_hip_error.restype = i32
        L.kvp_last_hip_error.argtypes = [C.POINTER(i32)]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().kvp_strerror(int(code)).decode()


def _check(code, what):
    if code != KVP_OK:
        raise KvpError(code, what)


def _dptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _hptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def make_problem(L, N, P, K, plane_bytes, page_bytes, token_bytes, bw_hbm, bw_link, bw_dram, cap_pages,
                 n_words=None) -> kvp_problem:
    p = kvp_problem()
    p.n_layers, p.n_steps, p.n_pages, p.n_planes = int(L), int(N), int(P), int(K)
    p.n_words = int((P + 31) // 32 if n_words is None else n_words)
    for k in range(min(int(K), 8)):
        p.plane_bytes[k] = int(plane_bytes[k])
    p.page_bytes, p.token_bytes = int(page_bytes), int(token_bytes)
    p.bw_hbm, p.bw_link, p.bw_dram = float(bw_hbm), float(bw_link), float(bw_dram)
    p.cap_pages = int(cap_pages)
    return p


# ---- the C entry points, same names -------------------------------------------
def kvp_create(device: int = 0, stream=None):
    """Returns the opaque context handle.  `stream` is a torch.cuda.Stream or None
    (torch's current stream on that device)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(device)
    h = C.c_void_p()
    _check(lib().kvp_create(C.byref(h), int(device), C.c_void_p(stream.cuda_stream)), "kvp_create")
    return h


def kvp_destroy(ctx):
    lib().kvp_destroy(ctx)


def kvp_trace_upload(ctx, problem: kvp_problem, access, alive, persist, written):
    """Host uint32 arrays: access [L][N][K][Wd]; alive, persist, written [N][Wd]."""
    arrs = [np.ascontiguousarray(a, dtype=np.uint32) for a in (access, alive, persist, written)]
    L, N, K, Wd = problem.n_layers, problem.n_steps, problem.n_planes, problem.n_words
    if arrs[0].size != L * N * K * Wd or any(a.size != N * Wd for a in arrs[1:]):
        raise KvpError(KVP_ESHAPE, "kvp_trace_upload (array sizes)")
    _check(lib().kvp_trace_upload(ctx, C.byref(problem), *[_hptr(a) for a in arrs]), "kvp_trace_upload")


def kvp_score(ctx, d_placements, S, d_cost, d_excess, d_counters=None, d_occ=None):
    _check(lib().kvp_score(ctx, _dptr(d_placements), int(S), _dptr(d_cost), _dptr(d_excess),
                           _dptr(d_counters), _dptr(d_occ)), "kvp_score")


def kvp_score_static(ctx, d_placements, S, d_cost, d_excess):
    _check(lib().kvp_score_static(ctx, _dptr(d_placements), int(S), _dptr(d_cost), _dptr(d_excess)),
           "kvp_score_static")


def kvp_delta_score(ctx, d_placements, S, d_moves, d_counters, d_occ, d_delta, d_verdict):
    _check(lib().kvp_delta_score(ctx, _dptr(d_placements), int(S), _dptr(d_moves), _dptr(d_counters),
                                 _dptr(d_occ), _dptr(d_delta), _dptr(d_verdict)), "kvp_delta_score")


def kvp_anneal(ctx, params: kvp_anneal_params, d_init=None):
    _check(lib().kvp_anneal(ctx, C.byref(params), _dptr(d_init)), "kvp_anneal")


def kvp_best(ctx, shape_words=None, n_chains=None):
    """(cost, chain, placement words [L][N][Wd] or None, per-chain costs or None).  Without `shape_words`
    the winner's schedule stays on the device (no copy to the host)."""
    cost, chain = C.c_double(0.0), C.c_uint32(0)
    pl = np.empty(shape_words, dtype=np.uint32) if shape_words is not None else None
    cc = np.zeros(int(n_chains), dtype=np.float64) if n_chains else None
    _check(lib().kvp_best(ctx, C.byref(cost), C.byref(chain), _hptr(pl), _hptr(cc)), "kvp_best")
    return cost.value, chain.value, pl, cc


def kvp_chain_placement(ctx, chain, best, shape_words):
    pl = np.zeros(shape_words, dtype=np.uint32)
    _check(lib().kvp_chain_placement(ctx, int(chain), int(best), _hptr(pl)), "kvp_chain_placement")
    return pl


def kvp_chain_stats(ctx, n_chains):
    arr = (kvp_chain_stats_t * int(n_chains))()
    _check(lib().kvp_chain_stats(ctx, C.cast(arr, C.c_void_p)), "kvp_chain_stats")
    return list(arr)


KVP_SCORE_AUTO, KVP_SCORE_ROWS, KVP_SCORE_LANES, KVP_SCORE_QUAD = 0, 1, 2, 6
KVP_SCORE_CHUNK, KVP_SCORE_ROWBLOCK, KVP_SCORE_LINE, KVP_SCORE_ROWSEG, KVP_SCORE_ROWLANE = 9, 10, 11, 12, 13
SCORE_KERNEL_NAMES = {1: "rows", 2: "lanes", 6: "quad", 9: "chunk", 10: "rowblock", 11: "line", 12: "rowseg", 13: "rowlane"}


def kvp_strict_excess(ctx, d_placements, S, d_excess):
    _check(lib().kvp_strict_excess(ctx, _dptr(d_placements), int(S), _dptr(d_excess)), "kvp_strict_excess")


def kvp_score_slots(ctx, d_placements, d_slots, S, d_cost, d_excess):
    _check(lib().kvp_score_slots(ctx, _dptr(d_placements), _dptr(d_slots), int(S), _dptr(d_cost), _dptr(d_excess)),
           "kvp_score_slots")


def kvp_refine_slots(ctx, params, d_placement, d_slots):
    """Anneal the migration steps of one placement; returns the chains' statistics (d_slots holds their final Y)."""
    arr = (kvp_chain_stats_t * int(params.n_chains))()
    _check(lib().kvp_refine_slots(ctx, C.byref(params), _dptr(d_placement), _dptr(d_slots), C.cast(arr, C.c_void_p)),
           "kvp_refine_slots")
    return list(arr)


def kvp_temper(ctx, factors):
    """Multiply chain c's temperature by factors[c] (host array of n_chains doubles)."""
    import numpy as np
    f = np.ascontiguousarray(factors, dtype=np.float64)
    _check(lib().kvp_temper(ctx, f.ctypes.data), "kvp_temper")


def kvp_exchange(ctx, round: int, count: bool = True) -> int:
    """One replica-exchange round between neighbouring chains; returns the pairs that traded
    (-1 with count=False: the call then does not wait for the stream)."""
    n = C.c_uint32(0)
    _check(lib().kvp_exchange(ctx, int(round), C.byref(n) if count else None), "kvp_exchange")
    return int(n.value) if count else -1


def kvp_set_generator_batch_bytes(ctx, nbytes: int):
    _check(lib().kvp_set_generator_batch_bytes(ctx, int(nbytes)), "kvp_set_generator_batch_bytes")


def kvp_set_anneal_log_entries(ctx, entries: int):
    _check(lib().kvp_set_anneal_log_entries(ctx, int(entries)), "kvp_set_anneal_log_entries")


def kvp_set_capacity_mode(ctx, mode: int):
    _check(lib().kvp_set_capacity_mode(ctx, int(mode)), "kvp_set_capacity_mode")


def kvp_set_anneal_lookahead(ctx, proposals_per_round: int):
    _check(lib().kvp_set_anneal_lookahead(ctx, int(proposals_per_round)), "kvp_set_anneal_lookahead")


def kvp_set_score_kernel(ctx, which: int):
    _check(lib().kvp_set_score_kernel(ctx, int(which)), "kvp_set_score_kernel")


KVP_BASELINE_STATIC, KVP_BASELINE_RECENCY, KVP_BASELINE_FILL = 0, 1, 2


def kvp_wr_policy(ctx, ws, r10s, d_placements):
    """Schedules of the (W, R = r10/10) look-ahead policy for a batch of candidates into the device
    tensor d_placements [n][L][N][Wd] int32."""
    w = np.ascontiguousarray(ws, dtype=np.uint32)
    r = np.ascontiguousarray(r10s, dtype=np.uint32)
    assert w.shape == r.shape and w.ndim == 1
    _check(lib().kvp_wr_policy(ctx, int(w.size), _hptr(w), _hptr(r), _dptr(d_placements)), "kvp_wr_policy")


def kvp_wr_search(ctx, w_max, total_moves, n_levels=20, seed=0, w0=1, r10_0=5, p0=0.8, alpha=0.9,
                  op_prob=(0.4, 0.4, 0.2), stop_rel=1e-3, c_min_frac=1e-3, table=None, d_best_placement=None):
    """The annealing over (W, R).  Returns (kvp_wr_result, table [w_max][11] of the costs known, < 0 elsewhere)."""
    sp = kvp_wr_params(int(w_max), int(w0), int(r10_0), int(n_levels), int(seed), int(total_moves), float(p0),
                       float(alpha), (C.c_double * 3)(*op_prob), float(stop_rel), float(c_min_frac))
    if table is None:
        table = np.full((int(w_max), 11), -1.0)
    assert table.dtype == np.float64 and table.shape == (int(w_max), 11) and table.flags.c_contiguous
    res = kvp_wr_result()
    _check(lib().kvp_wr_search(ctx, C.byref(sp), _hptr(table), C.byref(res), _dptr(d_best_placement)), "kvp_wr_search")
    return res, table


def kvp_baseline(ctx, kind: int, d_placement):
    """One schedule [L][N][Wd] int32 (device tensor), written in full."""
    _check(lib().kvp_baseline(ctx, int(kind), _dptr(d_placement)), "kvp_baseline")


def kvp_score_kernel_used(ctx) -> int:
    return int(lib().kvp_score_kernel_used(ctx))


def kvp_plane_unit(ctx) -> int:
    return int(lib().kvp_plane_unit(ctx))


def make_anneal_params(n_chains, total_moves, moves=None, seed=0, n_levels=100, max_len=KVP_MAX_LEN,
                       init_mode=KVP_INIT_EMPTY, p0=0.8, alpha=0.9, op_prob=(0.4, 0.4, 0.2)):
    a = kvp_anneal_params()
    a.n_chains, a.n_levels, a.seed = int(n_chains), int(n_levels), int(seed)
    a.total_moves = int(total_moves)
    a.moves = int(total_moves if moves is None else moves)
    a.max_len, a.init_mode, a.p0, a.alpha = int(max_len), int(init_mode), float(p0), float(alpha)
    for i in range(3):
        a.op_prob[i] = float(op_prob[i])
    return a
