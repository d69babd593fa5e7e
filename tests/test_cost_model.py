"""The library's FLOP cost model (host arithmetic, no GPU needed) against the oracle written from the
paper's appendix A, on the constants the paper prints and on random ones."""
import numpy as np
import pytest

import paper_2012_03837_amd as lp
from oracle import cost as OC
from tests.test_oracle_cost import gold


def test_mlp_constants_match_the_paper():
    g = gold()
    f, a = lp.lp_mlp_flops(int(g["mlp_input"][0]), int(g["mlp_hidden"][0]), int(g["mlp_layers"][0]))
    assert f == g["mlp_forward_per_layer"][0] == 32514176.0
    assert a == g["mlp_aux"][0] == 77884.0
    for (i, n, l) in [(64, 256, 1), (3072, 1024, 8), (7, 5, 3)]:
        assert lp.lp_mlp_flops(i, n, l) == OC.mlp_flops(i, n, l)


@pytest.mark.parametrize("model", ["resnet50", "resnet18", "transformer_small", "transformer_large"])
def test_methods_match_the_oracle_on_the_printed_constants(model):
    f, a, bm, L, P = gold()[model]
    L = int(L)
    for steps, batch in [(1.0, 1.0), (12345.0, 512.0)]:
        for method, Ks in [("backprop", [1]), ("greedy", [1]), ("overlap", [1]), ("chunk", [1, 2, 3, L]),
                           ("last_k", [1, 2, L])]:
            for K in Ks:
                cpe, cost, time, par = lp.lp_cost_model(f, a, bm, L, P, method, steps, batch, K)
                ref = OC.cost_and_time(method, f, a, bm, L, P, steps, batch, K)
                np.testing.assert_allclose([cpe, cost, time], ref, rtol=1e-14)
                assert par == pytest.approx(OC.parallelism(method, bm, L, K), rel=1e-15)


def test_random_constants_and_errors():
    rng = np.random.default_rng(3)
    for _ in range(50):
        f, a, P = rng.uniform(1e3, 1e9, 3)
        bm = rng.uniform(1.0, 3.0)
        L = int(rng.integers(1, 40))
        K = int(rng.integers(1, L + 1))
        m = ["backprop", "greedy", "overlap", "chunk", "last_k"][int(rng.integers(0, 5))]
        got = lp.lp_cost_model(f, a, bm, L, P, m, 100.0, 32.0, K)[:3]
        np.testing.assert_allclose(got, OC.cost_and_time(m, f, a, bm, L, P, 100.0, 32.0, K), rtol=1e-13)
    with pytest.raises(lp.LpError):
        lp.lp_cost_model(1.0, 1.0, 2.0, 4, 0.0, "chunk", 1.0, 1.0, K=5)      # more chunks than layers
    with pytest.raises(lp.LpError):
        lp.lp_cost_model(1.0, 1.0, 2.0, 0, 0.0, "greedy", 1.0, 1.0)          # no layers
    with pytest.raises(lp.LpError):
        lp.lp_cost_model(1.0, 1.0, 2.0, 4, 0.0, 9, 1.0, 1.0)                 # unknown method
    with pytest.raises(lp.LpError):
        lp.lp_cost_model(1.0, 1.0, 2.0, 4, 0.0, "greedy", 0.0, 1.0)          # no steps
