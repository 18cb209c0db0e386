"""Pins for the GEMM oracle (CPU only): numpy's matmul (a library routine), hand-computed small
cases, identities (unit matrices, transposition, a single non-zero entry)."""
import numpy as np
import pytest

from oracle import attn_oracle as orc

RNG = np.random.default_rng(840)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (16, 8, 33), (64, 48, 100)])
def test_gemm_matches_numpy(M, N, K):
    a, b = RNG.standard_normal((M, K)), RNG.standard_normal((K, N))
    np.testing.assert_allclose(orc.gemm(a, b), a @ b, rtol=0, atol=1e-12)


def test_gemm_hand_cases():
    a = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    b = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -1.0]])
    np.testing.assert_array_equal(orc.gemm(a, b), np.array([[7.0, -1.0], [16.0, -1.0]]))
    # not symmetric in its operands: a transposed-operand mistake changes the result
    x = RNG.standard_normal((5, 5)); y = RNG.standard_normal((5, 5))
    assert np.abs(orc.gemm(x, y) - orc.gemm(y, x)).max() > 1e-3
    np.testing.assert_allclose(orc.gemm(x, y).T, orc.gemm(y.T, x.T), rtol=0, atol=1e-13)
    np.testing.assert_array_equal(orc.gemm(x, np.eye(5)), x)
    e = np.zeros((4, 6)); e[2, 3] = 1.0            # picks row 3 of b into row 2 of c
    bb = RNG.standard_normal((6, 3))
    c = orc.gemm(e, bb)
    np.testing.assert_array_equal(c[2], bb[3])
    assert np.count_nonzero(np.delete(c, 2, axis=0)) == 0


def test_gemm_elements_match_full():
    a, b = RNG.standard_normal((20, 31)), RNG.standard_normal((31, 17))
    rows, cols = RNG.integers(0, 20, 50), RNG.integers(0, 17, 50)
    np.testing.assert_allclose(orc.gemm_elements(a, b, rows, cols), (a @ b)[rows, cols], rtol=0, atol=1e-12)
