"""Elementary numerics of the oracle: rounding model and the textbook layer functions.

The paper names models only (Sec. 5.1 "Workloads"); the numerics are the textbook definitions of the layers
those models are made of.  Everything is fp64 unless a value is explicitly rounded with `Prec.store`.
"""
import numpy as np
from scipy.special import erf as _erf

LN_EPS = 1e-5


def bf16_round(x):
    """Round to the nearest bfloat16 (ties to even), returned as float64.

    bfloat16 is the upper 16 bits of an IEEE binary32; the value is first rounded to binary32 (what an
    fp32 accumulator holds) and then to 8 significant bits.
    """
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


class Prec:
    """Storage precision model: which values get rounded when a tensor is written to memory.

    'f32'  : nothing is rounded (the oracle stays in fp64; the fp32 GPU path is compared at rel 1e-4).
    'bf16' : every tensor the GPU path keeps in memory as bfloat16 is rounded at that point.
    """

    def __init__(self, kind):
        assert kind in ("f32", "bf16")
        self.kind = kind

    def store(self, x):
        return bf16_round(x) if self.kind == "bf16" else np.asarray(x, dtype=np.float64)


def gelu(x):
    """GELU(x) = x * Phi(x), Phi the standard normal CDF (exact erf form)."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    """d/dx GELU(x) = Phi(x) + x * phi(x)."""
    x = np.asarray(x, dtype=np.float64)
    cdf = 0.5 * (1.0 + _erf(x / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return cdf + x * pdf


def layernorm_fwd(x, g, b):
    """Row-wise LayerNorm with biased variance and eps = 1e-5.  Returns (y, mean, rstd)."""
    x = np.asarray(x, dtype=np.float64)
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    y = (x - mean) * rstd * g + b
    return y, mean, rstd


def layernorm_bwd(dy, x, g, mean, rstd):
    """Gradients of LayerNorm: returns (dx, dg, db); x is the tensor the forward pass read."""
    dy = np.asarray(dy, dtype=np.float64)
    xhat = (x - mean) * rstd
    dxhat = dy * g
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def softmax_rows(s):
    s = np.asarray(s, dtype=np.float64)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def cross_entropy_mean(logits, targets):
    """Mean token cross entropy and its gradient w.r.t. the logits.  logits [M,V], targets [M] ints."""
    logits = np.asarray(logits, dtype=np.float64)
    m = logits.shape[0]
    p = softmax_rows(logits)
    mx = logits.max(axis=-1)
    lse = mx + np.log(np.exp(logits - mx[:, None]).sum(axis=-1))
    loss = float((lse - logits[np.arange(m), targets]).mean())
    dlogits = p
    dlogits[np.arange(m), targets] -= 1.0
    return loss, dlogits / m
