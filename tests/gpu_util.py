"""Helpers for the GPU parity tests: tensor marshalling and the comparison bars.

Bars (per tensor): max|gpu - ref| / max|ref| <= 2e-2 for bf16 results and <= 1e-4 for fp32 results.  For single
kernels an element-wise bar is checked as well: one bf16 rounding step (2^-8 relative) plus fp32-accumulation
noise, which catches a wrong index or a dropped term that the per-tensor bar could hide."""
import numpy as np
import torch

from oracle.numerics import bf16_round

DEV = "cuda:0"


def bf(x):
    """numpy -> bf16 device tensor (values are rounded to bf16)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV).to(torch.bfloat16).contiguous()


def f32(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV).contiguous()


def i32(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(DEV).contiguous()


def up(t):
    """device tensor -> float64 numpy."""
    return t.detach().float().cpu().double().numpy()


def q(x):
    """The value a bf16 tensor made from x holds, as float64."""
    return bf16_round(np.asarray(x, dtype=np.float32))


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref)) / (den if den > 0 else 1.0))


def assert_bf16_close(got, ref, name="", elem_slack=2e-3):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), name
    e = rel_err(got, ref)
    assert e <= 2e-2, (name, e)
    bound = 2.0 ** -7 * np.abs(ref) + elem_slack * np.max(np.abs(ref)) + 1e-30
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (name, int(bad.sum()), np.argwhere(bad)[:5].tolist(), got[bad][:5], ref[bad][:5])


def assert_f32_close(got, ref, name="", tol=1e-4):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), name
    e = rel_err(got, ref)
    assert e <= tol, (name, e)


def lse_reference(qkv64, h, dh, causal=True):
    """log sum exp of the scaled, masked scores, written out from its definition on the bf16-rounded inputs."""
    b, s, _ = qkv64.shape
    da = h * dh
    qh = qkv64[..., 0:da].reshape(b, s, h, dh).transpose(0, 2, 1, 3)
    kh = qkv64[..., da:2 * da].reshape(b, s, h, dh).transpose(0, 2, 1, 3)
    sc = qh @ kh.transpose(0, 1, 3, 2) / np.sqrt(dh)
    if causal:
        sc = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
    mx = sc.max(axis=-1, keepdims=True)
    return (mx + np.log(np.exp(sc - mx).sum(axis=-1, keepdims=True)))[..., 0].reshape(b * h, s)
