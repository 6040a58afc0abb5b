"""Derives the constants of gelu_fast_f32() in lessdec_common.h.

Upper tail of the standard normal, Q(t) = 0.5 erfc(t / sqrt 2), t >= 0, is written as
Q(t) = exp(-t^2 / 2) * sum_{k=1..7} c_k u^k with u = 1 / (1 + p t): exp(t^2/2) Q(t) is a smooth,
slowly decaying function of t and a low-degree polynomial in u captures it to 1e-9.  Then
gelu(x) = x - |x| Q(|x|) for x >= 0 and -|x| Q(|x|) for x < 0.  Weighted least squares on a
dense grid (the weight is the factor exp(-t^2/2) t that multiplies the polynomial's error in
gelu).  Prints p, c_1..c_7 and the error of a float32 evaluation against float64 erfc.
"""
import numpy as np
from scipy.special import erfc, erfcx

P, N = 0.24, 7


def fit(p=P, n=N):
    t = np.concatenate([np.linspace(0, 8, 20001), np.linspace(8, 14, 2001)])
    u = 1 / (1 + p * t)
    target = 0.5 * erfcx(t / np.sqrt(2))                    # exp(t^2/2) Q(t), computed stably
    A = np.stack([u ** k for k in range(1, n + 1)], axis=1)
    w = np.exp(-t * t / 2) * np.maximum(t, 0.5)
    c, *_ = np.linalg.lstsq(A * w[:, None], target * w, rcond=None)
    return c


def gelu32(x, p, c):
    x = x.astype(np.float32)
    t = np.abs(x)
    u = (np.float32(1) / (np.float32(1) + np.float32(p) * t)).astype(np.float32)
    acc = np.full_like(u, np.float32(c[-1]))
    for k in range(len(c) - 2, -1, -1):
        acc = (acc * u + np.float32(c[k])).astype(np.float32)
    acc = (acc * u).astype(np.float32)
    e = np.exp2((np.float32(-0.5 * np.log2(np.e)) * t * t).astype(np.float32)).astype(np.float32)
    tq = (t * (acc * e).astype(np.float32)).astype(np.float32)
    return np.where(x >= 0, (x - tq).astype(np.float32), -tq)


if __name__ == "__main__":
    c = fit()
    print("p =", P)
    for k, v in enumerate(c, 1):
        print(f"c{k} = {v:.10e}")
    x = np.linspace(-12, 12, 2000001)
    exact = 0.5 * x * erfc(-x / np.sqrt(2))
    err = np.abs(gelu32(x, P, c).astype(np.float64) - exact)
    print("max abs error on [-12, 12]:", err.max(), "; on [-4, 4]:", err[np.abs(x) <= 4].max())
    print("max error / max(|gelu|, |x| 6e-8, 1e-30):", (err / np.maximum(np.abs(exact), 1e-30))[np.abs(x) > 1e-3].max())
