"""The strategy comparison script runs end to end on the GPU and its numbers hang together."""
import numpy as np
import pytest

import oracle as O
import workloads as W

pytestmark = pytest.mark.gpu


def test_strategy_comparison_on_a_small_trace():
    from paper_2508_13231_amd import report as R
    import paper_2508_13231_amd as K
    tok = R.token_trace(0.7, 0.9, 0.7, (2, 40, 320), seed=5)
    rows, note = R.evaluate(tok, w_max=8, refine_moves=2000, chains=8)
    assert set(rows) == set(R.ORDER)
    unl = rows["unlimited"][0]
    for name, (T, hit) in rows.items():
        assert T >= unl and 0.0 <= hit <= 1.0, name
    assert rows["unlimited"][1] == 1.0
    # the two baselines are the oracle's placements, so their latencies are the oracle's
    assert rows["static"][0] == O.score(tok, O.init_static_fill(tok)).cost
    assert rows["reactive"][0] == O.score(tok, O.init_recency(tok)).cost
    # the search keeps the best policy schedule unless the direct search improves on it
    q = O.Problem(tok)
    best = min(O.score(q, O.wr_policy(q, w, r)).cost for w in range(1, 9) for r in range(11))
    assert rows["SA-guided"][0] <= best
    # hit rate of the static placement, from the definition
    X = O.init_static_fill(tok)
    s = O.score(tok, X).step_bytes
    assert rows["static"][1] == pytest.approx(float(s[..., 0].sum()) / float(s[..., 0].sum() + s[..., 1].sum()), rel=1e-12)
