"""Writes closed_form_constants.txt: constants of the symmetric normal-quantile codebook
(Sec. 1 / Sec. 3.2: data points are quantile points of N(0,1)) computed from closed forms with
scipy only -- no code of this repository, neither the oracle nor the library, takes part.

    python tests/golden/make_closed_form_golden.py
"""
import os

import numpy as np
from scipy import integrate, stats

HERE = os.path.dirname(os.path.abspath(__file__))


def levels(k):
    L = 1 << k
    raw = stats.norm.ppf((np.arange(L) + 0.5) / L)
    return raw, raw / raw[-1]


def fixed_scale_distortion(k):
    """E (x - c(x))^2 for x ~ N(0,1), raw levels c_i, mid-point cells."""
    raw, _ = levels(k)
    edges = np.concatenate([[-np.inf], (raw[:-1] + raw[1:]) / 2, [np.inf]])
    return sum(integrate.quad(lambda x, c=c: (x - c) ** 2 * stats.norm.pdf(x), a, b)[0]
               for c, a, b in zip(raw, edges[:-1], edges[1:]))


def absmax_block_mse(k, n):
    """Per-element MSE of absmax-scaled blocks of n unit Gaussians: the maximum |x| = s has density
    n (2 Phi(s) - 1)^(n-1) 2 phi(s) and is reproduced exactly; the other n-1 elements are N(0,1)
    truncated to [-s, s] and fall on the levels s * c_i."""
    _, lev = levels(k)

    def trunc_mse(s):
        c = lev * s
        edges = np.concatenate([[-s], (c[:-1] + c[1:]) / 2, [s]])
        tot = sum(integrate.quad(lambda x, cj=cj: (x - cj) ** 2 * stats.norm.pdf(x), a, b)[0]
                  for cj, a, b in zip(c, edges[:-1], edges[1:]))
        return tot / (2 * stats.norm.cdf(s) - 1)

    dens = lambda s: n * (2 * stats.norm.cdf(s) - 1) ** (n - 1) * 2 * stats.norm.pdf(s)
    val, _ = integrate.quad(lambda s: trunc_mse(s) * dens(s), 0.3, 8.0, limit=400, epsabs=1e-12)
    return (n - 1) / n * val


def main():
    out = ["# Constants of the symmetric normal-quantile codebook c_i = Phi^-1((i + 1/2) / 2^k) / c_max",
           "# (Sec. 1: quantile points of a normal distribution as data points), from closed forms;",
           "# written by make_closed_form_golden.py (scipy only).  Format: name = value [value ...]", ""]
    for k in (2, 3, 4):
        raw, lev = levels(k)
        L = 1 << k
        out.append("raw_max_k%d = %.10f" % (k, raw[-1]))
        out.append("positive_half_k%d = %s" % (k, " ".join("%.10f" % v for v in lev[L // 2:])))
        out.append("half_largest_gap_k%d = %.7f" % (k, np.diff(lev).max() / 2))
        out.append("fixed_scale_distortion_k%d = %.7f" % (k, fixed_scale_distortion(k)))
        for n in (64, 128):
            out.append("absmax_block_mse_k%d_n%d = %.7f" % (k, n, absmax_block_mse(k, n)))
        out.append("")
    with open(os.path.join(HERE, "closed_form_constants.txt"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
