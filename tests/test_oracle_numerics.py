"""Pins for oracle/numerics.py: hand values, closed forms, finite differences and torch (library) routines."""
import math

import numpy as np
import pytest
import torch

from oracle import numerics as N


def test_bf16_round_hand_values():
    # 8 significant bits: spacing at 1.0 is 2^-7; exact halves go to the even neighbour
    assert N.bf16_round(1.0) == 1.0
    assert N.bf16_round(1.0 + 2.0 ** -8) == 1.0                      # tie -> even (mantissa 0)
    assert N.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2 * 2.0 ** -7  # tie -> even (mantissa 2)
    assert N.bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert N.bf16_round(-0.1) == -0.10009765625                      # 0xBDCD
    assert N.bf16_round(3.0e38) == float(torch.tensor(3.0e38).bfloat16().double())


def test_bf16_round_matches_torch_and_is_idempotent():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000), [0.0, -0.0, 1e-40]])
    got = N.bf16_round(x)
    want = torch.from_numpy(x.astype(np.float32)).bfloat16().double().numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(N.bf16_round(got), got)
    nz = np.abs(x) > 1e-30
    assert np.max(np.abs(got[nz] - x[nz]) / np.abs(x[nz])) <= 2.0 ** -8


def test_gelu_closed_forms():
    assert N.gelu(0.0) == 0.0
    assert abs(N.gelu(1.0) - 0.8413447460685429) < 1e-15          # Phi(1) from the normal table
    assert abs(N.gelu(-1.0) - (0.8413447460685429 - 1.0)) < 1e-15  # gelu(-x) = gelu(x) - x
    x = np.linspace(-6, 6, 241)
    assert np.allclose(N.gelu(-x), N.gelu(x) - x, atol=1e-14)
    assert np.allclose(N.gelu(x), torch.nn.functional.gelu(torch.from_numpy(x)).numpy(), atol=1e-14)
    assert abs(N.gelu_grad(0.0) - 0.5) < 1e-15


def test_gelu_grad_finite_difference():
    x = np.linspace(-5, 5, 101)
    h = 1e-6
    fd = (N.gelu(x + h) - N.gelu(x - h)) / (2 * h)
    assert np.max(np.abs(fd - N.gelu_grad(x))) < 1e-8


def test_layernorm_forward_properties_and_torch():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 7, 16)) * 3 + 1
    g, b = rng.standard_normal(16), rng.standard_normal(16)
    y, mean, rstd = N.layernorm_fwd(x, np.ones(16), np.zeros(16))
    assert np.allclose(y.mean(-1), 0, atol=1e-12)
    assert np.allclose(y.var(-1), x.var(-1) / (x.var(-1) + 1e-5), atol=1e-12)
    y2, _, _ = N.layernorm_fwd(x, g, b)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    assert np.allclose(y2, want.numpy(), atol=1e-12)


def test_layernorm_backward_autograd_and_fd():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 12))
    g, b, dy = rng.standard_normal(12), rng.standard_normal(12), rng.standard_normal((6, 12))
    _, mean, rstd = N.layernorm_fwd(x, g, b)
    dx, dg, db = N.layernorm_bwd(dy, x, g, mean, rstd)
    xt, gt, bt = (torch.tensor(a, requires_grad=True) for a in (x, g, b))
    (torch.nn.functional.layer_norm(xt, (12,), gt, bt, 1e-5) * torch.from_numpy(dy)).sum().backward()
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12)
    assert np.allclose(dg, gt.grad.numpy(), atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), atol=1e-12)
    # one finite difference, independent of any library
    f = lambda xx: float((N.layernorm_fwd(xx, g, b)[0] * dy).sum())
    e = np.zeros_like(x); e[3, 5] = 1e-6
    assert abs((f(x + e) - f(x - e)) / 2e-6 - dx[3, 5]) < 1e-7


def test_softmax_and_cross_entropy():
    rng = np.random.default_rng(3)
    s = rng.standard_normal((4, 9)) * 5
    p = N.softmax_rows(s)
    assert np.allclose(p.sum(-1), 1, atol=1e-14)
    assert np.allclose(N.softmax_rows(s + 100.0), p, atol=1e-12)           # shift invariance
    v = 50257
    loss, d = N.cross_entropy_mean(np.zeros((3, v)), np.array([0, 5, v - 1]))
    assert abs(loss - math.log(v)) < 1e-12 and abs(math.log(v) - 10.82490511) < 1e-7
    assert np.allclose(d.sum(-1), 0, atol=1e-15)
    t = np.array([1, 0, 8, 3])
    loss, d = N.cross_entropy_mean(s, t)
    st = torch.tensor(s, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(st, torch.from_numpy(t))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12 and np.allclose(d, st.grad.numpy(), atol=1e-14)
