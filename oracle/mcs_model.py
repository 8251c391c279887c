"""Magnitude-aware Clipping Strategy: the error model behind the clip rules.

TEST INFRASTRUCTURE ONLY.  Nothing here runs on the hot path -- at run time the
clip value is the closed-form rule of Eq. "gaus" / Eq. "fats".  These helpers
restate the objective the rules were derived from, so tests can check the rules'
premises by brute force:

* ``quantize_literal`` / ``dequantize_literal``: Eq. "suq" and the de-quantization
  formula evaluated literally in fp64.
* ``E_emp``: the magnitude-weighted quantization error, Eq. "e", on samples.
* ``E_model``: its simplified form, Eq. "e2", by numerical quadrature for a
  symmetric density ``p`` given on ``g >= 0``.
* ``dE_ds_invT``: the closed-form derivative printed for the Inverted-T density,
  Eq. "invT".
"""
from __future__ import annotations

import numpy as np


def quantize_literal(x, s):
    """Eq. "suq": round(127 * clamp(x, s) / s), ties to even, in fp64."""
    x = np.asarray(x, dtype=np.float64)
    clamped = np.where(np.abs(x) <= s, x, np.sign(x) * s)
    return np.rint(127.0 * clamped / s).astype(np.int64)


def dequantize_literal(q, s):
    """x^ = q * s / 127."""
    return np.asarray(q, dtype=np.float64) * (s / 127.0)


def E_emp(g, s, alpha):
    """Eq. "e" on samples: mean |g - g^| * exp(alpha |g|)."""
    g = np.asarray(g, dtype=np.float64)
    ghat = dequantize_literal(quantize_literal(g, s), s)
    return float(np.mean(np.abs(g - ghat) * np.exp(alpha * np.abs(g))))


def invT_density(eps, gmax, a, b):
    """Eq. "invT" on g >= 0 (one half of the symmetric density)."""

    def p(g):
        g = np.asarray(g, dtype=np.float64)
        return np.where(g < eps, a, np.where(g <= gmax, b, 0.0))

    return p


def _integrate(fn, lo, hi, breaks, n):
    """Trapezoid rule on [lo, hi], split at the density's discontinuities."""
    pts = [lo] + [x for x in sorted(breaks) if lo < x < hi] + [hi]
    total = 0.0
    for u, v in zip(pts[:-1], pts[1:]):
        # evaluate strictly inside the piece so a jump at an end point is not straddled
        g = np.linspace(u, v, n)
        gi = np.clip(g, u + (v - u) * 1e-12, v - (v - u) * 1e-12)
        total += float(np.trapezoid(fn(gi), g))
    return total


def E_model(s, alpha, p, gmax, n=20001, breaks=()):
    """Eq. "e2":  I1 + I2  with
    I1 = int_0^s (s/127) f p dg,   I2 = 2 int_s^gmax (g - s) f p dg,   f = exp(alpha g).
    ``breaks`` lists the points where the density ``p`` jumps."""
    i1 = _integrate(lambda g: (s / 127.0) * np.exp(alpha * g) * p(g), 0.0, s, breaks, n)
    if s >= gmax:
        return i1
    i2 = 2.0 * _integrate(lambda g: (g - s) * np.exp(alpha * g) * p(g), s, gmax, breaks, n)
    return i1 + i2


def dE_ds_invT(s, alpha, eps, gmax, a, b):
    """The derivative printed after Eq. "invT" (valid for eps < s <= gmax):
    [(a-b) e^{alpha eps} + b (255 + alpha s) e^{alpha s} - 254 b e^{alpha gmax} - a] / (127 alpha)."""
    num = (a - b) * np.exp(alpha * eps) + b * (255.0 + alpha * s) * np.exp(alpha * s) \
        - 254.0 * b * np.exp(alpha * gmax) - a
    return num / (127.0 * alpha)
