"""The gradient comparison used by the GPU tests must reject what a whole-head norm lets through.

Runs on the CPU: a reference gradient comes from the fp64 oracle, the "kernel result" is that
reference rounded to bf16 (what a correct kernel returns, up to accumulation order), and mistakes
are planted in it.
"""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from grad_check import check_grad, check_head, relf, GRAD_RELF


def bf16_round(x):
    return torch.from_numpy(x).to(torch.bfloat16).double().numpy()


@pytest.fixture(scope="module")
def grads():
    rng = np.random.default_rng(5)
    N, D = 1024, 64
    q, k, v, d_o = (bf16_round(rng.standard_normal((1, 2, N, D))) for _ in range(4))
    return orc.attn_bwd(q, k, v, d_o, True, 0.125)


def test_correctly_rounded_gradients_pass(grads):
    for r in grads:
        check_grad(bf16_round(r), r, "ok")


def test_one_wrong_row_fails_although_the_head_norm_passes(grads):
    for r in grads:
        g = bf16_round(r)
        g[0, 1, 517] = 0.0                       # one row of 1024 lost
        assert relf(g[0, 1], r[0, 1]) <= GRAD_RELF, "the whole-head norm does not see it"
        with pytest.raises(AssertionError):
            check_grad(g, r, "row")


def test_wrong_last_row_and_wrong_block_fail(grads):
    for r in grads:
        g = bf16_round(r)
        g[0, 0, -1] = g[0, 0, -17]               # the tail row holds another row's values
        with pytest.raises(AssertionError):
            check_grad(g, r, "tail")
        g = bf16_round(r)
        g[0, 0, 96:128] *= 1.06                  # a 32-row block off by 6 %
        with pytest.raises(AssertionError):
            check_grad(g, r, "block")


def test_single_element_fails(grads):
    r = grads[0]
    g = bf16_round(r)
    i = np.unravel_index(np.argmax(np.abs(r[0, 0])), r[0, 0].shape)
    g[0, 0][i] *= 0.5
    with pytest.raises(AssertionError):
        check_head(g[0, 0], r[0, 0], "element")


def test_all_zero_reference():
    z = np.zeros((4, 8))
    check_head(z.copy(), z, "zeros")
    with pytest.raises(AssertionError):
        check_head(z + 1e-3, z, "zeros")
