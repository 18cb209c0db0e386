"""Pins for the rotary oracle (CPU only): complex multiplication written with numpy's complex type,
closed forms (zero angle, quarter turn), norm preservation, composition of angles."""
import numpy as np
import pytest

from oracle import attn_oracle as orc

RNG = np.random.default_rng(1207)


@pytest.mark.parametrize("shape", [(1, 2), (5, 8), (3, 2, 7, 16), (2, 9, 128)])
def test_rotary_is_complex_multiplication(shape):
    x = RNG.standard_normal(shape)
    N, D = shape[-2:]
    theta = RNG.uniform(-4, 4, (N, D // 2))
    o = orc.rotary(x, np.sin(theta), np.cos(theta))
    z = (x[..., :D // 2] + 1j * x[..., D // 2:]) * np.exp(1j * theta)
    np.testing.assert_allclose(o[..., :D // 2], z.real, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o[..., D // 2:], z.imag, rtol=0, atol=1e-13)


def test_rotary_closed_forms_and_norm():
    x = RNG.standard_normal((2, 6, 8))
    zero, one = np.zeros((6, 4)), np.ones((6, 4))
    np.testing.assert_array_equal(orc.rotary(x, zero, one), x)                     # zero angle
    q = orc.rotary(x, one, zero)                                                    # quarter turn
    np.testing.assert_array_equal(q[..., :4], -x[..., 4:])
    np.testing.assert_array_equal(q[..., 4:], x[..., :4])
    theta = RNG.uniform(-3, 3, (6, 4))
    o = orc.rotary(x, np.sin(theta), np.cos(theta))
    np.testing.assert_allclose(o[..., :4] ** 2 + o[..., 4:] ** 2, x[..., :4] ** 2 + x[..., 4:] ** 2, rtol=1e-13)
    # a sign error in either output row breaks the composition of two rotations
    t2 = RNG.uniform(-3, 3, (6, 4))
    twice = orc.rotary(o, np.sin(t2), np.cos(t2))
    np.testing.assert_allclose(twice, orc.rotary(x, np.sin(theta + t2), np.cos(theta + t2)), rtol=0, atol=1e-13)


def test_rotary_rejects_bad_shapes():
    with pytest.raises(ValueError):
        orc.rotary(np.zeros((4, 8)), np.zeros((4, 8)), np.zeros((4, 8)))
