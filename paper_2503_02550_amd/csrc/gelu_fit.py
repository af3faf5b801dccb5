"""Derivation of the constants of gelu_fast / gelu_grad_fast in common.h.

GELU(x) = x * Phi(x) with Phi the standard normal distribution function.  For t = |x|,
    1 - Phi(t) = erfc(t / sqrt 2) / 2 = 2^p(t) / 2,     p(t) = log2 erfc(t / sqrt 2),
and p(t) / t is smooth enough on [0, 6] for a quartic: p(t) ~ t * (c0 + c1 t + c2 t^2 + c3 t^3 + c4 t^4).
The fit is a weighted least-squares fit of p(t)/t, re-weighted a few times towards the largest error of GELU.
Run:  python gelu_fit.py   (numpy + scipy; prints the coefficients and the largest absolute errors in float32)."""
import numpy as np
from scipy.special import erf, erfc

T, DEG = 6.0, 5
t = np.linspace(1e-4, T, 200001)
target = np.log2(erfc(t / np.sqrt(2)))
A = np.vander(t, DEG, increasing=True)
ww = erfc(t / np.sqrt(2)) * np.maximum(t, 0.05) * t
for _ in range(30):
    coef, *_ = np.linalg.lstsq(A * ww[:, None], (target / t) * ww, rcond=None)
    err = np.abs(0.5 * np.exp2(t * (A @ coef)) - 0.5 * erfc(t / np.sqrt(2))) * np.maximum(t, 1.0)
    ww = ww * (1 + 4 * err / err.max()) ** 0.5
c = coef.astype(np.float32)
print("coefficients c0..c4:", ", ".join(f"{float(v):.9g}f" for v in c))

x = np.linspace(-12, 12, 2400001).astype(np.float32)
ax = np.abs(x)
r = np.zeros_like(ax)
for v in c[::-1]:
    r = (r * ax + v).astype(np.float32)
assert np.all(r < 0), "p(t) must stay negative so that 2^p(t) decays"
h = np.float32(0.5) * np.exp2((ax * r).astype(np.float32)).astype(np.float32)
phi = np.where(x < 0, h, np.float32(1) - h).astype(np.float32)
x64 = x.astype(np.float64)
Phi = 0.5 * (1 + erf(x64 / np.sqrt(2)))
pdf = np.exp(-0.5 * x64 * x64) / np.sqrt(2 * np.pi)
gelu = x * phi
grad = phi + x * (np.float32(0.3989422804) * np.exp2((np.float32(-0.72134752) * x * x).astype(np.float32))).astype(np.float32)
print("largest |gelu - exact|      :", np.abs(gelu - x64 * Phi).max())
print("largest |gelu' - exact|     :", np.abs(grad - (Phi + x64 * pdf)).max())
