"""kvp_score_static, the scoring entry point that allocates nothing, against kvp_score (which the
parity tests hold to the oracle bit for bit) and against the oracle itself: two calls in a row on
one context, the second on a smaller batch, so that what the first left in the static scratch
array is there when the second runs."""
import numpy as np
import pytest

import oracle as O
import paper_2508_13231_amd as K
import workloads as W
from gpu_util import Gpu

pytestmark = pytest.mark.gpu

CASES = [("llama8b", 0.25, 24, 7),       # narrow rows, L = 2^k: block sums and tile verdicts only
         ("gqa70b", 0.0625, 12, 5),      # digit planes
         ("longctx", 0.125, 10, 3),
         ("serving", 0.0625, 9, 4),      # wide rows of several sequences
         ("tiny", 1.0, 16, 1)]


def _both(g, X, S, static_first):
    torch = g.torch
    d_x = g.words(X[:S])
    out = {}
    order = ("static", "plain") if static_first else ("plain", "static")
    for which in order:
        d_cost = torch.full((S,), -1.0, dtype=torch.float64, device=g.dev)
        d_ex = torch.full((S,), -1, dtype=torch.int32, device=g.dev)
        free0 = torch.cuda.mem_get_info(g.dev)[0]
        if which == "static":
            K.kvp_score_static(g.ctx, d_x, S, d_cost, d_ex)
            torch.cuda.synchronize()
            # (once the kernels' code is on the device: the runtime loads it at a kernel's first launch)
            assert static_first or torch.cuda.mem_get_info(g.dev)[0] == free0, "free device memory changed"
        else:
            K.kvp_score(g.ctx, d_x, S, d_cost, d_ex)
            torch.cuda.synchronize()
        out[which] = (d_cost.cpu().numpy(), d_ex.cpu().numpy().view(np.uint32), g.kernel_used())
    return out


@pytest.mark.parametrize("name,scale,S1,S2", CASES)
def test_static_scratch_scoring_equals_kvp_score_on_two_calls_in_a_row(name, scale, S1, S2):
    tr = W.config(name, scale)
    q = O.Problem(tr)
    X = np.concatenate([W.random_placements(tr, S1 - 2, seed=11, density=0.3),
                        W.edge_placements(tr)[1:3]]).astype(np.uint8)
    print(f"case {name} scale {scale} S {S1} then {S2}", flush=True)
    with Gpu(tr) as g:
        first = _both(g, X, S1, static_first=True)          # the context's very first scoring call is the static one
        second = _both(g, X[S1 - S2:], S2, static_first=False)
        for got, Xs in ((first, X), (second, X[S1 - S2:])):
            assert got["static"][2] == got["plain"][2]       # the same scorer ran
            assert (got["static"][0] == got["plain"][0]).all() and (got["static"][1] == got["plain"][1]).all()
        for s in (0, S2 - 1):
            sc = O.score(q, X[S1 - S2 + s])
            assert second["static"][0][s] == sc.cost and second["static"][1][s] == sc.excess


def test_static_scratch_scoring_refuses_what_does_not_fit():
    tr = W.config("llama8b", 0.25)
    with Gpu(tr) as g:
        torch = g.torch
        nb = (tr.L * tr.N + 63) // 64
        per = nb * 8 + tr.N * 4
        S = K.KVP_STATIC_SCRATCH_BYTES // per + 2
        d_x = torch.zeros((1,) + g.shape_words, dtype=torch.int32, device=g.dev)     # never read: refused first
        d_cost = torch.full((1,), -1.0, dtype=torch.float64, device=g.dev)
        d_ex = torch.full((1,), -1, dtype=torch.int32, device=g.dev)
        with pytest.raises(K.KvpError) as e:
            K.kvp_score_static(g.ctx, d_x, S, d_cost, d_ex)
        assert e.value.code == K.KVP_ESHAPE
        torch.cuda.synchronize()
        assert d_cost.item() == -1.0 and d_ex.item() == -1
        for bad in (dict(d_placements=None), dict(d_cost=None), dict(d_excess=None)):
            args = dict(d_placements=d_x, d_cost=d_cost, d_excess=d_ex)
            args.update(bad)
            with pytest.raises(K.KvpError) as e:
                K.kvp_score_static(g.ctx, args["d_placements"], 1, args["d_cost"], args["d_excess"])
            assert e.value.code == K.KVP_EINVAL
        K.kvp_score_static(g.ctx, d_x, 0, None, None)      # S = 0 is a no-op
    # a layer count whose summation tree is not kept on chip needs the step latencies as well
    tr = W.random_trace(5, L=3, N=70, P=700, K=1, cap_pages=500)
    q = O.Problem(tr)
    X = W.random_placements(tr, 6, seed=2, density=0.3).astype(np.uint8)
    with Gpu(tr) as g:
        got = _both(g, X, 6, static_first=True)
        assert (got["static"][0] == got["plain"][0]).all() and (got["static"][1] == got["plain"][1]).all()
        assert got["static"][0][3] == O.cost(q, X[3])
