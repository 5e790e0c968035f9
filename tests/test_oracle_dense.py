"""Pins for the CPU oracle's dense-layer arithmetic (oracle/dense.c).

Checked against closed forms, special cases, hand-computed roundings and
library routines (numpy float64 matmul, torch's bfloat16 cast, math.erf) - never
against the oracle's own formulas.
"""
import math

import numpy as np
import pytest
import torch

from oracle import dense
from paper_1902_04610_amd import synth


def test_identity_zero_and_onehot_weights():
    rng = np.random.default_rng(0)
    X = rng.uniform(-1, 1, (5, 16)).astype(np.float32)
    eye = np.eye(16, dtype=np.float32)
    assert (dense.dense_f32(X, eye, dense.ACT_NONE) == X).all()
    assert (dense.dense_f32(X, eye, dense.ACT_RELU) == np.maximum(X, 0)).all()
    assert (dense.dense_f32(X, np.zeros((16, 7), np.float32), dense.ACT_GELU) == 0).all()
    # a weight matrix with a single one at (k=3, n=5) copies column 3 into column 5:
    # fails if the operand is read transposed
    W = np.zeros((16, 9), np.float32)
    W[3, 5] = 1.0
    Y = dense.dense_f32(X, W, dense.ACT_NONE)
    assert (Y[:, 5] == X[:, 3]).all() and (np.delete(Y, 5, axis=1) == 0).all()


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 70, 5), (8, 256, 256), (33, 129, 65)])
def test_matches_float64_library_matmul(M, K, N):
    rng = np.random.default_rng(M * 1000 + K)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((K, N)).astype(np.float32)
    ref = (X.astype(np.float64) @ W.astype(np.float64))
    Y = dense.dense_f32(X, W, dense.ACT_NONE)
    # the exact sum rounded once: at most half an ulp away from float64's result
    assert np.abs(Y - ref).max() <= np.spacing(np.abs(ref).max().astype(np.float32))
    Xb, Wb = synth.f32_to_bf16_bits(X), synth.f32_to_bf16_bits(W)
    refb = synth.bf16_bits_to_f32(Xb).astype(np.float64) @ synth.bf16_bits_to_f32(Wb).astype(np.float64)
    Yb = dense.dense_bf16(Xb, Wb, dense.ACT_NONE)
    assert np.abs(Yb - refb).max() <= np.spacing(np.abs(refb).max().astype(np.float32))


def test_bf16_rounding_hand_values():
    f = dense.lib().orc_bf16_from_f32
    # bf16 keeps 8 significant bits: spacing 2^-7 at 1.0
    assert f(1.0) == 0x3F80
    assert f(1.0 + 2 ** -8) == 0x3F80            # tie -> even mantissa (0)
    assert f(1.0 + 3 * 2 ** -8) == 0x3F82        # tie -> even mantissa (2)
    assert f(1.0 + 2 ** -8 + 2 ** -20) == 0x3F81  # just above the tie
    assert f(-2.5) == 0xC020
    assert f(0.0) == 0 and f(-0.0) == 0x8000
    assert f(3.3895313892515355e38) == 0x7F7F     # largest finite bf16
    assert f(float("inf")) == 0x7F80
    assert dense.lib().orc_f32_from_bf16(0x3FC0) == 1.5


def test_bf16_rounding_against_two_other_implementations():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        [0.0, 1.0, 1.0 + 2 ** -8, 65504.0]]).astype(np.float32)
    got = dense.round_bf16(x)
    via_torch = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (got == via_torch).all()
    assert (got == synth.f32_to_bf16_bits(x)).all()
    assert (dense.bf16_to_f32(got) == torch.from_numpy(x).to(torch.bfloat16).float().numpy()).all()


def test_activation_values():
    z = np.array([[-3.0, -1.0, -0.5, 0.0, 0.5, 1.0, 3.0, 10.0]], np.float32)
    one = np.ones((1, 1), np.float32)
    for act, fn in ((dense.ACT_RELU, lambda v: max(v, 0.0)),
                    (dense.ACT_GELU, lambda v: v * 0.5 * (1.0 + math.erf(v / math.sqrt(2.0))))):
        got = np.array([dense.dense_f32(np.array([[v]], np.float32), one, act)[0, 0] for v in z[0]])
        want = np.array([fn(float(v)) for v in z[0]], np.float32)
        assert (got == want).all()
    # GELU(1) = Phi(1) = 0.841344746..., GELU(-1) = -(1 - Phi(1))
    g = dense.dense_f32(np.array([[1.0], [-1.0]], np.float32), one, dense.ACT_GELU)
    assert abs(g[0, 0] - 0.8413447460685429) < 1e-7 and abs(g[1, 0] + 0.15865525393145707) < 1e-7


def test_mlp_bf16_recipe_rounds_between_layers():
    """Second layer sees the bf16-rounded first-layer output, not the float one."""
    X = synth.f32_to_bf16_bits(np.array([[1.0]], np.float32))
    W1 = synth.f32_to_bf16_bits(np.array([[1.0 + 2 ** -7]], np.float32))      # exact in bf16
    W2 = synth.f32_to_bf16_bits(np.array([[1.0 + 2 ** -7]], np.float32))
    h1, y = dense.mlp_forward_bf16(X, [W1, W2], [dense.ACT_NONE, dense.ACT_NONE])
    assert h1[0, 0] == np.float32(1.0 + 2 ** -7)
    # (1+2^-7)^2 = 1 + 2^-6 + 2^-14 exactly, representable in float
    assert y[0, 0] == np.float32(1.0 + 2 ** -6 + 2 ** -14)
    # with a first-layer result that is NOT a bf16 number the rounding shows:
    W1 = synth.f32_to_bf16_bits(np.array([[1.0 + 2 ** -7]], np.float32))
    X = synth.f32_to_bf16_bits(np.array([[1.0 + 2 ** -7]], np.float32))
    h1, y = dense.mlp_forward_bf16(X, [W1, np.array([[0x3F80]], np.uint16)], [0, 0])
    assert h1[0, 0] == np.float32(1.0 + 2 ** -6 + 2 ** -14)
    assert y[0, 0] == np.float32(1.0 + 2 ** -6)                                # 2^-14 rounded away


def test_mlp_f32_against_float64_library():
    w = synth.workload1(seed=0)
    for job in range(2):
        H = w['X'][job][0].astype(np.float64)
        H = np.maximum(H @ w['W'][job][0].astype(np.float64), 0.0)
        ref = H.astype(np.float32).astype(np.float64) @ w['W'][job][1].astype(np.float64)
        got = dense.mlp_forward_f32(w['X'][job][0], w['W'][job], [dense.ACT_RELU, dense.ACT_NONE])[-1]
        assert np.abs(got - ref).max() <= 1e-6 * np.abs(ref).max()


def test_backward_products_against_float64_library():
    rng = np.random.default_rng(9)
    M, K, N = 6, 20, 11
    H = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    dY = synth.f32_to_bf16_bits(rng.standard_normal((M, N)).astype(np.float32))
    W = synth.f32_to_bf16_bits(rng.standard_normal((K, N)).astype(np.float32))
    f = lambda b: synth.bf16_bits_to_f32(b).astype(np.float64)
    dX = dense.dense_bwd_input_bf16(dY, W)
    dW = dense.dense_bwd_weight_bf16(H, dY)
    assert dX.shape == (M, K) and dW.shape == (K, N)
    assert np.abs(dX - f(dY) @ f(W).T).max() < 1e-5
    assert np.abs(dW - f(H).T @ f(dY)).max() < 1e-5


def test_softmax_xent_closed_forms_and_finite_differences():
    M, N = 4, 10
    loss, d = dense.softmax_xent(np.zeros((M, N), np.float32), np.arange(M, dtype=np.int32))
    assert abs(loss - math.log(N)) < 1e-12                 # uniform prediction
    assert np.allclose(d.sum(axis=1), 0, atol=1e-7)
    assert np.allclose(d[0], (np.full(N, 0.1) - np.eye(N)[0]) / M, atol=1e-7)
    # huge logits must not overflow (max-subtraction)
    big = np.zeros((1, 3), np.float32)
    big[0] = [1000.0, 0.0, -1000.0]
    loss, _ = dense.softmax_xent(big, np.array([0], np.int32))
    assert loss == 0.0
    # gradient = finite difference of the loss
    rng = np.random.default_rng(1)
    z = rng.standard_normal((M, N)).astype(np.float32)
    y = rng.integers(0, N, M).astype(np.int32)
    _, d = dense.softmax_xent(z, y)
    for (m, n) in [(0, 0), (1, 7), (3, int(y[3]))]:
        zp, zm = z.copy(), z.copy()
        zp[m, n] += 1e-2
        zm[m, n] -= 1e-2
        fd = (dense.softmax_xent(zp, y)[0] - dense.softmax_xent(zm, y)[0]) / (zp[m, n] - zm[m, n])
        assert abs(fd - d[m, n]) < 1e-4


def test_sgd_update():
    Wm = np.array([1.0, -2.0, 0.3], np.float32)
    Wb = np.zeros(3, np.uint16)
    keep = Wm.copy()
    dense.sgd_update(Wm, Wb, np.array([5.0, 5.0, 5.0], np.float32), 0.0)
    assert (Wm == keep).all() and (Wb == synth.f32_to_bf16_bits(keep)).all()   # lr = 0 changes nothing
    dense.sgd_update(Wm, Wb, np.array([2.0, -4.0, 0.0], np.float32), 0.25)
    assert (Wm == np.array([0.5, -1.0, 0.3], np.float32)).all()
    assert (Wb == synth.f32_to_bf16_bits(Wm)).all()
