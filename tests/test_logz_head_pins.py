"""Pins of the log-Z head oracle: closed forms, finite differences, and an independent library evaluation."""
import math

import numpy as np
import pytest
import torch

from oracle import logz_head_oracle as lz


def _case(seed=3, P=5, H=12, M=9, lens=(4, 1, 0, 7, 3)):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)])
    X = rng.normal(size=(int(cu[-1]), H))
    W1 = rng.normal(size=(M, H)) * 0.4
    b1 = rng.normal(size=M) * 0.3
    w2 = rng.normal(size=M)
    b2 = 0.37
    d = rng.normal(size=P)
    return X, cu, W1, b1, w2, b2, d


def test_gelu_values_and_derivative():
    assert lz.gelu(np.array([0.0]))[0] == 0.0
    assert lz.gelu(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-15)      # Phi(1)
    assert lz.gelu(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-14)   # -Phi(-1)
    x = np.linspace(-4, 4, 33)
    np.testing.assert_allclose(lz.gelu(x) - lz.gelu(-x), x, atol=1e-15)                      # gelu(x) - gelu(-x) = x
    h = 1e-6
    np.testing.assert_allclose(lz.gelu_grad(x), (lz.gelu(x + h) - lz.gelu(x - h)) / (2 * h), atol=1e-9)
    assert lz.gelu_grad(np.array([0.0]))[0] == 0.5


def test_pooling_and_closed_forms():
    X, cu, W1, b1, w2, b2, d = _case()
    pooled = lz.prompt_pool(X, cu)
    np.testing.assert_allclose(pooled[0], X[0:4].mean(0), atol=1e-15)
    np.testing.assert_array_equal(pooled[1], X[4])
    assert np.all(pooled[2] == 0)                                   # empty prompt
    # W1 = 0: logZ is the same constant for every prompt, w2 . gelu(b1) + b2
    f = lz.logz_head_forward(X, cu, W1 * 0, b1, w2, b2)
    np.testing.assert_allclose(f["log_z"], float(lz.gelu(b1) @ w2) + b2, atol=1e-15)
    # w2 = 0: logZ = b2 and only db2 / dw2 are non-zero
    f = lz.logz_head_forward(X, cu, W1, b1, w2 * 0, b2)
    np.testing.assert_array_equal(f["log_z"], np.full(5, b2))
    g = lz.logz_head_backward(f, W1, w2 * 0, d)
    assert np.all(g["dW1"] == 0) and np.all(g["db1"] == 0) and g["db2"] == pytest.approx(d.sum())
    np.testing.assert_allclose(g["dw2"], f["g"].T @ d, atol=1e-15)
    # the empty prompt sees only the biases
    f = lz.logz_head_forward(X, cu, W1, b1, w2, b2)
    assert f["log_z"][2] == pytest.approx(float(lz.gelu(b1) @ w2) + b2, rel=1e-14)
    # bf16 bit patterns are widened exactly
    Xb = torch.from_numpy(X).to(torch.bfloat16)
    np.testing.assert_array_equal(lz.prompt_pool(Xb.view(torch.int16).numpy(), cu), lz.prompt_pool(Xb.double().numpy(), cu))


def test_gradients_by_finite_differences():
    X, cu, W1, b1, w2, b2, d = _case()
    f = lz.logz_head_forward(X, cu, W1, b1, w2, b2)
    g = lz.logz_head_backward(f, W1, w2, d)
    obj = lambda W1_, b1_, w2_, b2_: float(lz.logz_head_forward(X, cu, W1_, b1_, w2_, b2_)["log_z"] @ d)
    h = 1e-6
    num = np.zeros_like(W1)
    for i in range(W1.shape[0]):
        for j in range(W1.shape[1]):
            e = np.zeros_like(W1); e[i, j] = h
            num[i, j] = (obj(W1 + e, b1, w2, b2) - obj(W1 - e, b1, w2, b2)) / (2 * h)
    np.testing.assert_allclose(g["dW1"], num, rtol=1e-6, atol=1e-8)
    for name, vec in (("db1", b1), ("dw2", w2)):
        num = np.zeros_like(vec)
        for i in range(vec.size):
            e = np.zeros_like(vec); e[i] = h
            args_p = (W1, b1 + e, w2, b2) if name == "db1" else (W1, b1, w2 + e, b2)
            args_m = (W1, b1 - e, w2, b2) if name == "db1" else (W1, b1, w2 - e, b2)
            num[i] = (obj(*args_p) - obj(*args_m)) / (2 * h)
        np.testing.assert_allclose(g[name], num, rtol=1e-6, atol=1e-8)
    assert g["db2"] == pytest.approx((obj(W1, b1, w2, b2 + h) - obj(W1, b1, w2, b2 - h)) / (2 * h), rel=1e-7)


def test_same_network_in_an_independent_library():
    X, cu, W1, b1, w2, b2, d = _case(seed=8, P=4, H=16, M=11, lens=(3, 5, 2, 6))
    f = lz.logz_head_forward(X, cu, W1, b1, w2, b2)
    g = lz.logz_head_backward(f, W1, w2, d)
    tW1 = torch.tensor(W1, requires_grad=True); tb1 = torch.tensor(b1, requires_grad=True)
    tw2 = torch.tensor(w2, requires_grad=True); tb2 = torch.tensor(b2, dtype=torch.float64, requires_grad=True)
    pooled = torch.stack([torch.tensor(X[cu[p]:cu[p + 1]]).mean(0) for p in range(4)])
    out = torch.nn.functional.gelu(torch.nn.functional.linear(pooled, tW1, tb1)) @ tw2 + tb2
    np.testing.assert_allclose(f["log_z"], out.detach().numpy(), rtol=1e-13)
    (out * torch.tensor(d)).sum().backward()
    np.testing.assert_allclose(g["dW1"], tW1.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["db1"], tb1.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dw2"], tw2.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert g["db2"] == pytest.approx(float(tb2.grad), rel=1e-13)
