"""Seeded synthetic KV-cache access traces.

This module only *draws inputs*: which pages exist at each decode step, which
ones attention reads, which one receives the new token.  It contains none of
the latency model, no scoring and no search: both the CPU oracle and the GPU
library consume what it emits.

The traces stand in for recorded layer-wise attention of a long-context decode
(paper Sec. IV-A): importance scores follow a parametric drift, and the access
set of a step is the top share of pages by score (the complement of the
"attention sparsity" of Sec. IV-B) plus attention sinks and the most recent
tokens.

All arrays are plain booleans (uint8 0/1), page-indexed:

    access  [L][N][K][P]   page p read by plane k at step (n, l)
    alive   [N][P]         page p holds KV data while step n executes
    persist [N][P]         page p held the same data at step n-1 and n
    written [N][P]         page p receives the token generated at step n

`pack_bits` turns the last axis into little-endian uint32 words
(bit b of word w = page 32*w + b).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np

KV_TOKEN_BYTES = 4096  # 8 KV heads x 128 dims x (K and V) x 2 B, one layer


@dataclass
class Recipe:
    name: str
    L: int
    N: int
    page_tokens: int
    prompt_lo: int
    prompt_hi: int                      # prompt length ~ U[lo, hi] tokens
    slots: int = 1                      # concurrent sequences
    slot_pages: Optional[int] = None    # page slots per sequence (default: just enough)
    K: int = 1                          # access planes (per-head sets)
    top_frac: float = 0.10              # share of alive pages read per step
    top_count: Optional[int] = None     # fixed count among non-forced pages
    sink_tokens: int = 0
    recent_tokens: int = 0
    drift: str = "ar1"                  # "ar1" | "jump"
    phi: float = 0.9
    sigma: float = 0.7
    jump_p: float = 0.02
    jump_mean: float = 3.0
    burn_in: int = 200
    lifetime_mean: float = 0.0          # 0: sequences never finish
    cap_frac: Optional[float] = None    # share of L x peak alive pages
    cap_pages: Optional[int] = None
    bw_hbm: float = 4.0e12
    bw_link: float = 0.5e12
    bw_dram: float = 0.5e12
    plane_tokens_bytes: int = KV_TOKEN_BYTES   # bytes per token across all planes
    chains: int = 16
    moves: int = 20000
    seed: int = 0


@dataclass
class Trace:
    name: str
    L: int
    N: int
    P: int
    K: int
    access: np.ndarray
    alive: np.ndarray
    persist: np.ndarray
    written: np.ndarray
    plane_bytes: list
    page_bytes: int
    token_bytes: int
    bw_hbm: float
    bw_link: float
    bw_dram: float
    cap_pages: int
    chains: int = 16
    moves: int = 20000
    seed: int = 0
    recipe: Optional[Recipe] = field(default=None, repr=False)

    @property
    def n_words(self) -> int:
        return (self.P + 31) // 32

    def with_bandwidth_ratio(self, r: float) -> "Trace":
        slow = self.bw_hbm / r
        return replace(self, bw_link=slow, bw_dram=slow)


def pack_bits(a: np.ndarray) -> np.ndarray:
    """Pack booleans along the last axis into uint32 words, LSB first."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    P = a.shape[-1]
    Wd = (P + 31) // 32
    if P != Wd * 32:
        pad = np.zeros(a.shape[:-1] + (Wd * 32 - P,), dtype=np.uint8)
        a = np.concatenate([a, pad], axis=-1)
    by = np.packbits(a, axis=-1, bitorder="little")
    return np.ascontiguousarray(by).view("<u4").reshape(a.shape[:-1] + (Wd,))


def unpack_bits(w: np.ndarray, P: int) -> np.ndarray:
    """Inverse of pack_bits."""
    w = np.ascontiguousarray(w, dtype="<u4")
    by = w.view(np.uint8).reshape(w.shape[:-1] + (w.shape[-1] * 4,))
    return np.unpackbits(by, axis=-1, bitorder="little")[..., :P].copy()


def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), tag]))


def _select_top(z: np.ndarray, eligible: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Exactly-k largest of z along the last axis among `eligible`; ties go to the
    lower index.  z: [..., S, M]; eligible: bool [S, M]; k: int [S] (a count per
    row of `eligible`, cut to the number of eligible entries)."""
    M = z.shape[-1]
    k = np.minimum(k, eligible.sum(axis=-1))
    zz = np.where(eligible, z, -np.inf)
    pos = np.clip(M - k, 0, M - 1)
    srt = np.partition(zz, np.unique(pos), axis=-1)                   # every needed position in its sorted place
    idx = np.broadcast_to(pos[:, None], zz.shape[:-1] + (1,))
    kth = np.take_along_axis(srt, idx, axis=-1)                       # [..., S, 1]: the k-th largest
    kth = np.where((k > 0)[:, None], kth, np.inf)
    gt = zz > kth
    tie = (zz == kth) & eligible
    need = k[:, None] - gt.sum(axis=-1, keepdims=True)
    if (tie.sum(axis=-1, keepdims=True) == need).all():               # no surplus of equal scores: take them all
        return gt | tie
    rank = np.cumsum(tie, axis=-1)
    return gt | (tie & (rank <= need))


def _plan(r: Recipe, slot_pages: int):
    """The sequences of every slot, step by step (no importance scores yet): context length [N][S],
    whether the slot's sequence started at the step [N][S], and the page masks that follow."""
    rng = _rng(r.seed, 1)
    N, S, pt = r.N, r.slots, r.page_tokens
    P = S * slot_pages

    def draw_prompt(n):
        if r.prompt_lo == r.prompt_hi:
            return np.full(n, r.prompt_lo, dtype=np.int64)
        return rng.integers(r.prompt_lo, r.prompt_hi + 1, size=n)

    ctx = np.zeros((N, S), dtype=np.int64)
    fresh = np.zeros((N, S), dtype=bool)
    prompt = draw_prompt(S)
    age = np.zeros(S, dtype=np.int64)
    ended = np.zeros(S, dtype=bool)
    for n in range(N):
        if n == 0:
            fresh[n] = True
        else:
            fresh[n] = ended                         # finished sequences are replaced in the same slot
            if ended.any():
                prompt[ended] = draw_prompt(int(ended.sum()))
                age[ended] = 0
            age[~ended] += 1
        ctx[n] = prompt + age + 1                    # tokens incl. the new one
        ended = rng.random(S) < 1.0 / r.lifetime_mean if r.lifetime_mean > 0 else np.zeros(S, dtype=bool)
    pages = -(-ctx // pt)                            # [N][S]
    col = np.arange(slot_pages)
    alive = col[None, None, :] < pages[:, :, None]                               # [N][S][slot_pages]
    prev = np.concatenate([np.zeros((1, S), np.int64), pages[:-1]])
    persist = (col[None, None, :] < np.minimum(pages, prev)[:, :, None]) & ~fresh[:, :, None]
    written = col[None, None, :] == ((ctx - 1) // pt)[:, :, None]
    forced = np.zeros((N, S, slot_pages), dtype=bool)
    if r.sink_tokens:
        forced |= col[None, None, :] < (-(-np.minimum(r.sink_tokens, ctx) // pt))[:, :, None]
    if r.recent_tokens:
        forced |= col[None, None, :] >= (np.maximum(ctx - r.recent_tokens, 0) // pt)[:, :, None]
    forced &= alive
    u8 = lambda a: a.reshape(N, P).astype(np.uint8)
    return ctx, pages, fresh, alive, forced, u8(alive), u8(persist), u8(written)


def _layer_group(r: Recipe, layers, slot_pages, plan, access):
    """Importance scores and access sets of a run of consecutive layers.  Every layer draws from a
    stream of its own, so the trace does not depend on how the layers are grouped."""
    ctx, pages, fresh, alive, forced = plan
    N, K, S, pt = r.N, r.K, r.slots, r.page_tokens
    G = len(layers)
    rngs = [_rng(r.seed, 16 + l) for l in layers]
    sd = r.sigma / math.sqrt(1.0 - r.phi * r.phi) if r.drift == "ar1" else 0.0

    def jumps(rng, shape):
        hit = rng.random(shape) < r.jump_p
        return np.where(hit, rng.exponential(r.jump_mean, shape), 0.0)

    def fresh_scores(rng, shape):
        if r.drift == "ar1":
            return rng.standard_normal(shape) * sd
        z = np.zeros(shape)
        for _ in range(r.burn_in):
            z = r.phi * z + jumps(rng, shape)
        return z

    z = np.stack([fresh_scores(rng, (K, S, slot_pages)) for rng in rngs])          # [G][K][S][slot_pages]
    eps = np.empty_like(z)
    for n in range(N):
        if n > 0:
            # importance drift of every slot; a slot whose sequence starts now gets fresh scores instead
            for g, rng in enumerate(rngs):
                if r.drift == "ar1":
                    rng.standard_normal(out=eps[g])
                else:
                    eps[g] = jumps(rng, eps[g].shape)
            z *= r.phi
            if r.drift == "ar1":
                eps *= r.sigma
            z += eps
            new = np.flatnonzero(fresh[n])
            if new.size:
                for g, rng in enumerate(rngs):
                    z[g][:, new, :] = fresh_scores(rng, (K, new.size, slot_pages))
        # a page that starts with the new token enters at the top score of its sequence
        for s in np.flatnonzero(((ctx[n] - 1) % pt == 0) & (pages[n] > 1)):
            ap = int(pages[n, s])
            z[:, :, s, ap - 1] = z[:, :, s, :ap - 1].max(axis=-1)
        if r.top_count is not None:
            sel = _select_top(z, alive[n] & ~forced[n], np.full(S, r.top_count, dtype=np.int64))
        else:
            sel = _select_top(z, alive[n], np.ceil(r.top_frac * pages[n]).astype(np.int64))
        sel |= forced[n]
        access[layers[0]:layers[0] + G, n] = sel.reshape(G, K, S * slot_pages)


def generate(r: Recipe, threads: Optional[int] = None) -> Trace:
    """Draw the trace of a recipe.  Layers are independent given the sequences, so runs of layers
    are drawn by a few threads (numpy releases the interpreter lock in its loops)."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    L, N, K, S = r.L, r.N, r.K, r.slots
    pt = r.page_tokens
    slot_pages = r.slot_pages or -(-(r.prompt_hi + N) // pt)
    P = S * slot_pages
    ctx, pages, fresh, alive_b, forced, alive, persist, written = _plan(r, slot_pages)
    access = np.zeros((L, N, K, P), dtype=np.uint8)
    if threads is None:
        threads = max(1, min(len(os.sched_getaffinity(0)) // 2, 8))
    # small traces: one run of layers (the per-call overhead of numpy dominates); large: a run per thread
    n_groups = 1 if L * K * P < 200_000 else max(1, min(L, threads))
    bounds = [L * g // n_groups for g in range(n_groups + 1)]
    groups = [list(range(bounds[g], bounds[g + 1])) for g in range(n_groups) if bounds[g + 1] > bounds[g]]
    plan = (ctx, pages, fresh, alive_b, forced)
    if len(groups) == 1:
        _layer_group(r, groups[0], slot_pages, plan, access)
    else:
        with ThreadPoolExecutor(len(groups)) as ex:
            list(ex.map(lambda ls: _layer_group(r, ls, slot_pages, plan, access), groups))

    page_bytes = pt * r.plane_tokens_bytes
    plane_bytes = [page_bytes // K] * K
    if r.cap_pages is not None:
        cap = int(r.cap_pages)
    else:
        peak = int(alive.sum(axis=1, dtype=np.int64).max())
        cap = int(math.floor(r.cap_frac * L * peak + 1e-9))
    return Trace(name=r.name, L=L, N=N, P=P, K=K, access=access, alive=alive,
                 persist=persist, written=written, plane_bytes=plane_bytes,
                 page_bytes=page_bytes, token_bytes=r.plane_tokens_bytes,
                 bw_hbm=r.bw_hbm, bw_link=r.bw_link, bw_dram=r.bw_dram,
                 cap_pages=cap, chains=r.chains, moves=r.moves, seed=r.seed,
                 recipe=r)


def regroup(tok: Trace, page_tokens: int, reads: str = "token") -> Trace:
    """Pages of `page_tokens` consecutive tokens from a trace whose pages are single
    tokens (a Recipe with page_tokens = 1; with several slots, slot_pages must be
    a multiple of page_tokens).  Placement and migration are then per page, as
    in the paper's page-granularity strategy (Sec. IV-A), and

      reads = "page":   a page with any accessed token is read whole (the overhead
                        of retrieving a page for a few important tokens), one plane;
      reads = "token":  a page's read costs its accessed tokens only: plane k holds
                        bit k of the number of accessed tokens in the page and
                        weighs token_bytes * 2^k.

    The capacity keeps its size in bytes (cap_pages = token capacity // page_tokens)."""
    if tok.K != 1 or tok.page_bytes != tok.token_bytes or tok.plane_bytes != [tok.token_bytes]:
        raise ValueError("regroup needs a trace whose pages are single tokens")
    pt = int(page_tokens)
    T = tok.P
    P = -(-T // pt)

    def group(a):
        pad = P * pt - T
        if pad:
            a = np.concatenate([a, np.zeros(a.shape[:-1] + (pad,), a.dtype)], axis=-1)
        return a.reshape(a.shape[:-1] + (P, pt))

    counts = group(tok.access[:, :, 0, :]).sum(axis=-1, dtype=np.int64)          # [L][N][P]
    alive = group(tok.alive).any(axis=-1).astype(np.uint8)
    persist = group(tok.persist).any(axis=-1).astype(np.uint8)
    written = group(tok.written).any(axis=-1).astype(np.uint8)
    if reads == "page":
        access = (counts > 0).astype(np.uint8)[:, :, None, :]
        plane_bytes = [pt * tok.token_bytes]
    elif reads == "token":
        K = int(pt).bit_length()
        access = np.stack([(counts >> k) & 1 for k in range(K)], axis=2).astype(np.uint8)
        plane_bytes = [tok.token_bytes << k for k in range(K)]
    else:
        raise ValueError(reads)
    return Trace(name=f"{tok.name}/p{pt}{reads[0]}", L=tok.L, N=tok.N, P=P, K=access.shape[2], access=access,
                 alive=alive, persist=persist, written=written, plane_bytes=plane_bytes,
                 page_bytes=pt * tok.token_bytes, token_bytes=tok.token_bytes, bw_hbm=tok.bw_hbm,
                 bw_link=tok.bw_link, bw_dram=tok.bw_dram, cap_pages=tok.cap_pages // pt,
                 chains=tok.chains, moves=tok.moves, seed=tok.seed, recipe=tok.recipe)


def _ratio(r: float):
    return dict(bw_hbm=4.0e12, bw_link=4.0e12 / r, bw_dram=4.0e12 / r)


# The five workload shapes and the Table-I parity case.  "scale" shrinks the
# large dimensions (layers, steps, prompt) for tests while keeping the recipe.
def recipe(name: str, scale: float = 1.0) -> Recipe:
    def sc(x, lo=1, mult=1):
        v = max(lo, int(round(x * scale)))
        return -(-v // mult) * mult

    if name == "tiny":
        return Recipe("tiny", L=1, N=sc(64), page_tokens=1, prompt_lo=sc(192), prompt_hi=sc(192),
                      top_count=20, sink_tokens=4, recent_tokens=8, phi=0.95, sigma=0.5,
                      cap_pages=sc(64), bw_hbm=4000e9, bw_link=500e9, bw_dram=500e9,
                      chains=16, moves=20000, seed=0)
    if name == "llama8b":
        return Recipe("llama8b", L=sc(32, 2), N=sc(256, 8), page_tokens=16,
                      prompt_lo=sc(4096, 64, 16), prompt_hi=sc(4096, 64, 16),
                      top_frac=0.10, sink_tokens=4, recent_tokens=8, phi=0.9, sigma=0.7,
                      cap_frac=0.30, **_ratio(8), chains=256, moves=100000, seed=1)
    if name == "longctx":
        return Recipe("longctx", L=sc(32, 2), N=sc(1024, 8), page_tokens=16,
                      prompt_lo=sc(32768, 64, 16), prompt_hi=sc(32768, 64, 16),
                      top_frac=0.05, drift="jump", phi=0.9, jump_p=0.02, jump_mean=3.0,
                      cap_frac=0.20, **_ratio(8), chains=1024, moves=200000, seed=2)
    if name == "serving":
        return Recipe("serving", L=sc(32, 2), N=sc(512, 8), page_tokens=16, slots=sc(64, 2),
                      prompt_lo=sc(1024, 32, 16), prompt_hi=sc(16384, 64, 16),
                      top_frac=0.08, phi=0.9, sigma=0.7, lifetime_mean=max(300.0 * scale, 4.0),
                      cap_frac=0.25, **_ratio(4), chains=512, moves=100000, seed=3)
    if name == "gqa70b":
        return Recipe("gqa70b", L=sc(80, 2), N=sc(2048, 8), page_tokens=128, K=8,
                      prompt_lo=sc(131072, 256, 128), prompt_hi=sc(131072, 256, 128),
                      top_frac=0.04, phi=0.9, sigma=0.7,
                      cap_frac=0.15, **_ratio(8), chains=512, moves=50000, seed=4)
    if name == "decode36k":
        # Not one of the benchmark's configurations: one long sequence in the manner of the paper's own
        # workload (Sec. IV-A: a prompt of some 30k tokens, thousands of decoded tokens), with rows of 80
        # mask words, wider than the widest single-sequence configuration above.
        return Recipe("decode36k", L=sc(32, 2), N=sc(4096, 8), page_tokens=16,
                      prompt_lo=sc(36864, 64, 16), prompt_hi=sc(36864, 64, 16),
                      top_frac=0.05, phi=0.9, sigma=0.7,
                      cap_frac=0.20, **_ratio(8), chains=256, moves=100000, seed=6)
    if name == "table1":
        # Memory system of the paper's Table I: the one case where the link and
        # the DRAM channels differ.  508-token prompt: a page is born at step 4,
        # seven of the 40 page slots never hold data.
        return Recipe("table1", L=2, N=8, page_tokens=16, prompt_lo=508, prompt_hi=508, slot_pages=40,
                      top_frac=0.25, sink_tokens=4, recent_tokens=8, phi=0.9, sigma=0.7,
                      cap_pages=20, bw_hbm=4.9e12, bw_link=900e9, bw_dram=500e9,
                      chains=4, moves=2000, seed=5)
    raise KeyError(name)


CONFIG_NAMES = ["tiny", "llama8b", "longctx", "serving", "gqa70b"]


def config(name: str, scale: float = 1.0) -> Trace:
    return generate(recipe(name, scale))


def random_trace(seed: int, L: int, N: int, P: int, K: int = 1, *, p_access: float = 0.3,
                 rebirth: bool = True, cap_pages: Optional[int] = None,
                 bw=(4.9e12, 900e9, 500e9), page_bytes: int = 65536,
                 token_bytes: int = 4096, plane_bytes=None) -> Trace:
    """Unstructured random instance: pages are born, die and are re-used at
    random, several pages may be written in a step.  For stress and brute-force
    tests, where the structure of a real decode would hide cases."""
    rng = _rng(seed, 2)
    alive = np.zeros((N, P), dtype=np.uint8)
    persist = np.zeros((N, P), dtype=np.uint8)
    written = np.zeros((N, P), dtype=np.uint8)
    cur = rng.random(P) < 0.7
    for n in range(N):
        if n > 0:
            die = cur & (rng.random(P) < (0.15 if rebirth else 0.0))
            born = ~cur & (rng.random(P) < 0.3)
            reborn = cur & ~die & (rng.random(P) < (0.05 if rebirth else 0.0))
            nxt = (cur & ~die) | born
            persist[n] = cur & nxt & ~reborn & ~born
            wr_new = born | reborn
            cur = nxt
        else:
            wr_new = np.zeros(P, dtype=bool)
        alive[n] = cur
        w = wr_new | (cur & (rng.random(P) < 0.1))
        written[n] = w & cur
    access = (rng.random((L, N, K, P)) < p_access) & alive[None, :, None, :].astype(bool)
    if plane_bytes is None:
        plane_bytes = [page_bytes // K] * K
    if cap_pages is None:
        cap_pages = max(1, int(0.4 * L * alive.sum(axis=1).max()))
    return Trace(name=f"random{seed}", L=L, N=N, P=P, K=K, access=access.astype(np.uint8),
                 alive=alive, persist=persist, written=written, plane_bytes=list(plane_bytes),
                 page_bytes=page_bytes, token_bytes=token_bytes, bw_hbm=bw[0], bw_link=bw[1],
                 bw_dram=bw[2], cap_pages=int(cap_pages), chains=4, moves=2000, seed=seed)
