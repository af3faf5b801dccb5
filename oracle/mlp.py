"""Two-Linear MLP of the Tiny configuration (fp32 on the GPU, fp64 here).

  h = GELU(x W1^T + b1),  y = h W2^T + b2,  loss = mean((y - t)^2) / 2,  theta <- theta - lr * grad

Weights are stored [out_features, in_features].  The paper does not define this model; it is the smallest
training instance that produces kernels to monitor and a bubble to fill (Sec. 3.1).
"""
import numpy as np
from .numerics import gelu, gelu_grad


def mlp_forward(p, x):
    x = np.asarray(x, dtype=np.float64)
    z = x @ p["w1"].T + p["b1"]
    h = gelu(z)
    y = h @ p["w2"].T + p["b2"]
    return y, (x, z, h)


def mlp_loss_and_grads(p, x, t):
    y, (x, z, h) = mlp_forward(p, x)
    diff = y - np.asarray(t, dtype=np.float64)
    loss = 0.5 * float((diff ** 2).mean())
    dy = diff / diff.size
    g = {}
    g["w2"] = dy.T @ h
    g["b2"] = dy.sum(axis=0)
    dh = dy @ p["w2"]
    dz = dh * gelu_grad(z)
    g["w1"] = dz.T @ x
    g["b1"] = dz.sum(axis=0)
    return loss, g


def mlp_train_step(p, x, t, lr):
    """One SGD step; returns (loss before the update, new parameter dict, grads)."""
    loss, g = mlp_loss_and_grads(p, x, t)
    new = {k: np.asarray(p[k], dtype=np.float64) - lr * g[k] for k in p}
    return loss, new, g
