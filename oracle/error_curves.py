"""Regenerates, from the integer oracle, the approximation-error figures the paper reports: the distances from GELU of
h-GELU and i-GELU over [-4, 4] (Table 1), the gap between i-exp and exp over (-inf, 0] (Sec. 3.5), and samples of the
curves drawn in Fig. 2.  Test infrastructure like the rest of this package; prints a small text report.

    python -m oracle.error_curves [--scale 0.0078125] [--samples 9]

Every integer value comes from the oracle's scalar functions (orc_igelu_t, orc_hgelu_t, orc_iexp) on the integers
q = round(x / S); nothing here is used by the library or by the tests' expected values.
"""
from __future__ import annotations

import argparse
import math

import numpy as np
from scipy.special import erf

import oracle
from oracle import params as P


def _gelu(x):
    return x * 0.5 * (1.0 + erf(x / math.sqrt(2.0)))


def gelu_distances(S: float, lo: float = -4.0, hi: float = 4.0):
    """(L2, Linf) of integer i-GELU and integer h-GELU from GELU on the grid of representable inputs q S in [lo, hi];
    L2 is the root mean square over the grid, which is what reproduces the printed column."""
    gp, hp = P.gelu_params(S, 1.0), P.hgelu_params(S, 1.0)
    S_t = P.gelu_t_scale(S)
    qs = np.arange(math.ceil(lo / S), math.floor(hi / S) + 1)
    step = max(1, qs.size // 20000)
    qs = qs[::step]
    x = qs * S
    ig = np.array([oracle.igelu_t(int(q), gp) for q in qs]) * S_t
    hg = np.array([oracle.hgelu_t(int(q), hp) for q in qs]) * (S * S / 6.0)
    ref = _gelu(x)
    out = {}
    for name, v in (("i-GELU", ig), ("h-GELU", hg)):
        err = v - ref
        out[name] = (float(np.sqrt(np.mean(err ** 2))), float(np.max(np.abs(err))))
    return out, x, ref, ig, hg


def iexp_gap(S: float, lo: float = -12.0):
    """Largest |i-exp(x) - exp(x)| over the representable x = q S in [lo, 0]."""
    sp = P.softmax_params(S)
    S_out = 0.3585 * S * S
    qs = np.arange(math.ceil(lo / S), 1)
    step = max(1, qs.size // 20000)
    qs = qs[::step]
    vals = np.array([oracle.iexp(int(q), sp.q_ln2, sp.q_b, sp.q_c)[0] for q in qs]) * S_out
    err = vals - np.exp(qs * S)
    return float(np.max(np.abs(err))), qs * S, vals


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--scale", type=float, default=2.0 ** -7)
    ap.add_argument("--samples", type=int, default=9)
    a = ap.parse_args(argv)
    S = a.scale
    dist, x, ref, ig, hg = gelu_distances(S)
    print("input scale S = %g" % S)
    print("Table 1 (distance from GELU over [-4, 4]; paper: h-GELU 0.031 / 0.068, i-GELU 0.0082 / 0.018)")
    for name in ("h-GELU", "i-GELU"):
        print("  %-7s L2 %.4f   Linf %.4f" % (name, dist[name][0], dist[name][1]))
    gap, xe, ve = iexp_gap(S)
    print("i-exp in integers at this S: largest gap to exp on [-12, 0] = %.2e (paper, real-valued polynomial: 1.9e-3)" % gap)
    print("Fig. 2 samples: x, GELU, h-GELU, i-GELU")
    for i in np.linspace(0, x.size - 1, a.samples).astype(int):
        print("  %+7.3f  %+9.5f  %+9.5f  %+9.5f" % (x[i], ref[i], hg[i], ig[i]))
    print("Fig. 2 samples: x, exp, i-exp")
    for i in np.linspace(0, xe.size - 1, a.samples).astype(int):
        print("  %+7.3f  %9.6f  %9.6f" % (xe[i], math.exp(xe[i]), ve[i]))
    return dist, gap


if __name__ == "__main__":
    main()
