"""Theoretical (data-free) MSE and MAE centroids for Gaussian weights - TEST INFRASTRUCTURE, used to pin the oracle.

Implements the closed form of appendix B.2 ("Simplified Solution for Gaussian Network Weights") by numerical
integration over the block maximum m:

    level(l) = - INT m [g(m x)]_{a}^{b} (2G(m)-1)^(I-2) g(m) dm  /  INT m^2 [G(m x)]_{a}^{b} (2G(m)-1)^(I-2) g(m) dm

with a = xi(l-1), b = xi(l) the mid-point thresholds, g / G the standard normal pdf / cdf.  The leading minus
comes from the antiderivative INT x g(m x) dx = -g(m x)/m^2 and is present in the un-boxed form of the
equation; the boxed copy printed right after it omits it (reading: the minus belongs there - without it every
level changes sign and the printed theoretical codebook is not a fixed point).

The formula covers regions inside (-1, 1).  For the leftmost region of a signed codebook (no probability mass
at -1, appendix B.2 "Expectation of the Outermost Reconstruction Levels") the lower limit -inf is replaced by
-1.  A region that would contain the point mass at +1 or -1 is not supported (those levels are pinned in every
codebook of the paper).
"""
import numpy as np
from scipy.special import ndtr

_SQRT2PI = np.sqrt(2.0 * np.pi)


def _pdf(t):
    return np.exp(-0.5 * t * t) / _SQRT2PI


def _grid(m_max=14.0, points=40001):
    assert points % 2 == 1
    m = np.linspace(0.0, m_max, points)
    h = m[1] - m[0]
    wts = np.ones(points)
    wts[1:-1:2] = 4.0
    wts[2:-1:2] = 2.0
    return m, wts * (h / 3.0)  # composite Simpson


def region_integrals(a, b, block, m=None, wts=None):
    """(numerator, denominator, mass) of one region [a, b) inside [-1, 1] for block size `block`.

    mass is INT p_M(m) [F_X^cont(x|m)]_a^b dm scaled by (I-1)/I, i.e. P[X in region] for the continuous part.
    """
    if m is None:
        m, wts = _grid()
    core = np.zeros_like(m)
    G = ndtr(m)
    absG = 2.0 * G - 1.0  # F_|W|(m)
    core[1:] = absG[1:] ** (block - 2) * _pdf(m[1:])
    num = np.sum(wts * m * (_pdf(m * b) - _pdf(m * a)) * core)
    den = np.sum(wts * m * m * (ndtr(m * b) - ndtr(m * a)) * core)
    # p_M(m) = 2 I F_|W|^(I-1) g(m);  F_X^cont(x|m) = (G(mx) - G(-m)) / (2G(m)-1)
    mass = np.sum(wts * 2.0 * block * core * (ndtr(m * b) - ndtr(m * a))) * (block - 1) / block
    return num, den, mass


def centroid_update(cb, block, pinned_mask):
    """One theoretical Lloyd iteration: thresholds at mid-points, every unpinned level moved to its centroid."""
    cb = np.asarray(cb, dtype=np.float64)
    xi = 0.5 * (cb[:-1] + cb[1:])
    m, wts = _grid()
    new = cb.copy()
    for l in range(16):
        if (pinned_mask >> l) & 1:
            continue
        a = xi[l - 1] if l > 0 else -1.0
        if l == 15:
            raise ValueError("the region holding the point mass at +1 is not supported; pin level 15")
        b = xi[l]
        a = max(a, -1.0)
        num, den, _ = region_integrals(a, b, block, m, wts)
        new[l] = -num / den
    return new


def fixed_point(cb0, block, pinned_mask, iters=200, tol=1e-13):
    cb = np.asarray(cb0, dtype=np.float64).copy()
    for _ in range(iters):
        nxt = centroid_update(cb, block, pinned_mask)
        if np.max(np.abs(nxt - cb)) < tol:
            return nxt
        cb = nxt
    return cb


def region_probabilities(cb, block, signed):
    """P[X in region l] for all 16 regions, including the point masses at the ends (appendix B.1)."""
    cb = np.asarray(cb, dtype=np.float64)
    xi = np.concatenate([[-1.0], 0.5 * (cb[:-1] + cb[1:]), [1.0]])
    m, wts = _grid()
    p = np.array([region_integrals(xi[l], xi[l + 1], block, m, wts)[2] for l in range(16)])
    if signed:
        p[15] += 1.0 / block
    else:
        p[0] += 0.5 / block
        p[15] += 0.5 / block
    return p


def distance_db(theo, emp, block, signed):
    """Weighted distance between two codebooks in dB (appendix C, equation before the emp-vs-theo table)."""
    theo = np.asarray(theo, dtype=np.float64)
    emp = np.asarray(emp, dtype=np.float64)
    p = region_probabilities(theo, block, signed)
    return 10.0 * np.log10(np.sum(p * (theo - emp) ** 2) / np.sum(p * theo ** 2))


def _weighted_mass_below(x, block, m, wts):
    """INT m p_M(m) F_X^cont(x | M = m) dm up to factors that do not depend on x (and a term constant in x):
    INT m (2G(m) - 1)^(I-2) g(m) G(m x) dm - the quantity whose differences appear in the MAE condition of
    section 3.2 eq. 7 (appendix B.4) for Gaussian weights."""
    core = np.zeros_like(m)
    core[1:] = (2.0 * ndtr(m[1:]) - 1.0) ** (block - 2) * _pdf(m[1:])
    return np.sum(wts * m * core * ndtr(m * x))


def mae_centroid_update(cb, block, pinned_mask):
    """One theoretical Lloyd iteration under the MAE criterion: every unpinned level moves to the point of its region
    below which half of the region's mass, weighted by the block maximum, lies (eq. 7: the zero of a monotone function,
    found by bisection).  Same restrictions on the outermost regions as centroid_update."""
    cb = np.asarray(cb, dtype=np.float64)
    xi = 0.5 * (cb[:-1] + cb[1:])
    m, wts = _grid()
    new = cb.copy()
    for l in range(16):
        if (pinned_mask >> l) & 1:
            continue
        if l == 15:
            raise ValueError("the region holding the point mass at +1 is not supported; pin level 15")
        a = max(xi[l - 1], -1.0) if l > 0 else -1.0
        b = xi[l]
        ha, hb = _weighted_mass_below(a, block, m, wts), _weighted_mass_below(b, block, m, wts)
        target = ha + 0.5 * (hb - ha)
        lo, hi = a, b
        for _ in range(100):
            mid = 0.5 * (lo + hi)
            if _weighted_mass_below(mid, block, m, wts) < target:
                lo = mid
            else:
                hi = mid
        new[l] = 0.5 * (lo + hi)
    return new
