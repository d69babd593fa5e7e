"""Pins of the FLOP cost-model oracle (appendix A): the values the paper prints, and reductions between
the methods that hold whatever the constants are (they fix the readings of the damaged formulas)."""
import os

import numpy as np
import pytest

from oracle import cost as OC

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cost_model_paper_values.txt")


def gold():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            out[k] = [float(x) for x in v]
    return out


def test_mlp_constants_printed_in_the_paper():
    g = gold()
    fwd, aux = OC.mlp_flops(int(g["mlp_input"][0]), int(g["mlp_hidden"][0]), int(g["mlp_layers"][0]))
    assert fwd == g["mlp_forward_per_layer"][0]
    assert aux == g["mlp_aux"][0]


def test_mlp_formula_pieces():
    # one layer, I = N = 1: a 1x1 matrix-vector product is 1 multiply (2*1*1 - 1), + 1 bias + 2 ReLU
    assert OC.mlp_flops(1, 1, 1)[0] == 4
    # the average weights the first layer once and the others L-1 times
    f2, _ = OC.mlp_flops(3, 5, 2)
    assert f2 == ((2 * 3 * 5 - 3 + 15) + (2 * 5 * 5 - 5 + 15)) / 2


@pytest.mark.parametrize("model", ["resnet50", "resnet18", "transformer_small", "transformer_large"])
def test_reductions_between_methods(model):
    f, a, bm, L, P = gold()[model]
    L = int(L)
    steps, batch = 1000.0, 64.0
    bp = OC.cost_and_time("backprop", f, a, bm, L, P, steps, batch)
    gr = OC.cost_and_time("greedy", f, a, bm, L, P, steps, batch)
    # K chunks = L layers is greedy; one chunk is backprop (cost and time)
    np.testing.assert_allclose(OC.cost_and_time("chunk", f, a, bm, L, P, steps, batch, K=L), gr, rtol=1e-15)
    np.testing.assert_allclose(OC.cost_and_time("chunk", f, a, bm, L, P, steps, batch, K=1), bp, rtol=1e-15)
    # backward through all L layers is backprop, with no parallelism
    assert OC.parallelism("last_k", bm, L, K=L) == pytest.approx(1.0, rel=1e-15)
    np.testing.assert_allclose(OC.cost_and_time("last_k", f, a, bm, L, P, steps, batch, K=L), bp, rtol=1e-14)
    # a one-layer network: overlapping = greedy = backprop per example
    one = [OC.cost_per_example(m, f, a, bm, 1) for m in ("backprop", "greedy", "overlap")]
    assert one[0] == pytest.approx(one[1], rel=1e-15) and one[0] == pytest.approx(one[2], rel=1e-15)
    # greedy pays L-1 more auxiliary heads than backprop and is L times more parallel
    assert gr[0] - bp[0] == pytest.approx((1 + bm) * (L - 1) * a, rel=1e-12)
    assert gr[2] == pytest.approx(gr[1] / (batch * L), rel=1e-15)
    # overlapping: one forward and one head per layer, 2L-1 layer backward passes, L head backward passes
    ov = OC.cost_per_example("overlap", f, a, bm, L)
    assert ov == pytest.approx(L * (f + a) + bm * ((2 * L - 1) * f + L * a), rel=1e-14)
    # its per-step extra is the optimizer's 10 FLOPs/parameter plus 2 per parameter for the averaging
    c1 = OC.cost_and_time("overlap", f, a, bm, L, P, 1.0, batch)[1]
    assert c1 - ov * batch == pytest.approx(12.0 * P, rel=1e-12, abs=1e-6)


def test_last_k_parallelism_counts_chunks_of_k_layers():
    # with a backward multiplier of 1 a layer's backward costs as much as its forward: the last K layers
    # (forward + backward = 2K units) are the atomic chunk and the network is (L + K) units long
    assert OC.parallelism("last_k", 1.0, 8, K=2) == pytest.approx((8 + 2) / 4)
