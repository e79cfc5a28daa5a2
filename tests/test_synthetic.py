"""The seeded input generators: what the GPU tests check and what bench.py times must be the
same layers."""
import numpy as np
import pytest

from synthetic import config_cases, draw_layer


@pytest.mark.parametrize("shape", [dict(B=2, L=5, J=7, I=24, O=16, H=3, K=3),
                                   dict(B=3, L=1, J=1, I=64, O=40),
                                   dict(B=4, L=33, J=31, I=136, O=8, H=1, K=7)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_weights_and_mask_do_not_depend_on_drawing_x(shape, dtype):
    a = draw_layer("a", dtype=dtype, seed=77, draw_x=True, **shape)
    b = draw_layer("b", dtype=dtype, seed=77, draw_x=False, **shape)
    assert b.X.shape[0] == 0
    assert np.array_equal(a.W.view(np.uint32), b.W.view(np.uint32))
    assert np.array_equal(a.bias.view(np.uint32), b.bias.view(np.uint32))
    assert np.array_equal(a.gamma, b.gamma)


def test_network_cases_agree_with_and_without_x():
    # a few layers of the ResNet50-shaped configuration at a reduced batch (same seeds)
    with_x = list(zip(range(6), config_cases(3, batch=2)))
    without = list(zip(range(6), config_cases(3, batch=2, draw_x=False)))
    for (_, a), (_, b) in zip(with_x, without):
        assert a.name == b.name
        assert np.array_equal(a.W.view(np.uint32), b.W.view(np.uint32))
        assert np.array_equal(a.gamma, b.gamma) and np.array_equal(a.bias, b.bias)
