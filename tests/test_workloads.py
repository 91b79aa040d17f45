"""The synthetic input generators: deterministic, and shaped as documented."""
import numpy as np
import pytest

import workloads as W


def test_tiny_config_matches_its_recipe():
    tr = W.config("tiny")
    assert (tr.L, tr.N, tr.P, tr.K, tr.n_words, tr.cap_pages) == (1, 64, 256, 1, 8, 64)
    assert (tr.page_bytes, tr.token_bytes, tr.plane_bytes) == (4096, 4096, [4096])
    assert (tr.bw_hbm, tr.bw_link, tr.bw_dram) == (4000e9, 500e9, 500e9)
    ctx = 193 + np.arange(64)
    assert (tr.alive.sum(axis=1) == ctx).all()
    assert (tr.access.sum(axis=(0, 2, 3)) == 32).all()          # 4 sinks + last 8 + top 20
    assert tr.access[0, :, 0, :4].all()
    for n in range(64):
        assert tr.access[0, n, 0, ctx[n] - 8:ctx[n]].all()
        assert tr.written[n].nonzero()[0].tolist() == [ctx[n] - 1]
    assert not tr.persist[0].any() and (tr.persist[1:] == tr.alive[:-1]).all()


def test_llama_shape_and_determinism():
    a = W.config("llama8b", 0.25)
    b = W.config("llama8b", 0.25)
    for f in ("access", "alive", "persist", "written"):
        assert (getattr(a, f) == getattr(b, f)).all()
    full = W.recipe("llama8b")
    assert (full.L, full.N, full.prompt_lo, full.page_tokens) == (32, 256, 4096, 16)
    assert not (a.access.astype(bool) & ~a.alive.astype(bool)[None, :, None, :]).any()
    k = np.ceil(0.10 * a.alive.sum(axis=1))
    got = a.access.sum(axis=(2, 3))
    assert (got >= k[None]).all() and (got <= k[None] + 3).all()   # top 10 % plus sink and recent pages
    assert a.cap_pages == int(0.30 * a.L * a.alive.sum(axis=1).max())


def test_long_decode_recipe():
    full = W.recipe("decode36k")
    assert (full.L, full.N, full.prompt_lo, full.page_tokens) == (32, 4096, 36864, 16)      # rows of 80 mask words
    tr = W.config("decode36k", 0.0625)
    assert tr.written.sum(axis=1).tolist() == [1] * tr.N                                    # one sequence
    ctx = tr.alive.sum(axis=1)
    assert (np.diff(ctx) >= 0).all() and ctx[-1] == tr.P                                    # it only grows
    assert "decode36k" not in W.CONFIG_NAMES                                                # not a benchmark configuration


def test_serving_slots_turn_over():
    tr = W.config("serving", 0.08)
    assert tr.written.sum(axis=1).min() == tr.recipe.slots      # every sequence writes one token per step
    died = (tr.alive[:-1].astype(bool) & ~tr.alive[1:].astype(bool)).any()
    reused = (tr.alive[1:].astype(bool) & tr.alive[:-1].astype(bool) & ~tr.persist[1:].astype(bool)).any()
    assert died or reused


def test_pack_bits_layout():
    a = np.zeros((2, 70), np.uint8)
    a[0, 0] = a[0, 33] = a[1, 69] = 1
    w = W.pack_bits(a)
    assert w.shape == (2, 3) and w.dtype == np.uint32
    assert w.tolist() == [[1, 2, 0], [0, 0, 1 << 5]]
    assert (W.unpack_bits(w, 70) == a).all()


def test_random_placements_are_feasible():
    tr = W.config("table1")
    X = W.random_placements(tr, 4, seed=1, density=0.6)
    assert (X.sum(axis=(1, 3)) <= tr.cap_pages).all()
    assert not (X.astype(bool) & ~tr.alive.astype(bool)[None, None]).any()
