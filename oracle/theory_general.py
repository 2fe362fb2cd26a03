"""Theoretical (data-free) MSE centroids for an arbitrary symmetric weight distribution given as tables -
TEST INFRASTRUCTURE (the oracle of bof4_theory_centroids).

Section 3.2 eq. 5 (= the boxed general result of appendix B.2, "General Centroid Criterion") with the conditional
expectation of "Expectation of Normalized Weights" (boxed) and p_M, F_X of appendix B.1 substituted:

    level(l) = INT_0^inf m [Phi1(m x)]_a^b A(m)^(I-2) p_W(m) dm  /  INT_0^inf m^2 [F_W(m x)]_a^b A(m)^(I-2) p_W(m) dm

with a = xi(l-1), b = xi(l) the mid-point thresholds, A(m) = 2 F_W(m) - 1 the CDF of |W|, and Phi1(t) = INT_-inf^t
u p_W(u) du the first partial moment (the factors 2 (I-1) of p_M times F_X^cont and the 1 / (2 F_W(m) - 1) of the
truncated distribution are common to numerator and denominator up to A(m)^(I-2)).  For Gaussian weights
Phi1(t) = -g(t), which gives the closed form that oracle/theory.py integrates.

The distribution comes as two tables on the uniform grid u_k = k h, k = 0 .. n-1 (n odd), h = u_max / (n - 1):
pdf[k] = p_W(u_k) and cdf[k] = F_W(u_k) (F_W(0) = 1/2); p_W is even, so the negative side is implied.  The recipe,
stated so that another implementation can follow it to the last bit but the order of additions:
  * Psi[k] = INT_{u_k}^{u_max} u p_W(u) du by the trapezoid rule on the grid (Psi[n-1] = 0); Phi1(t) = -Psi(|t|);
  * F_W and Psi between grid points by linear interpolation; F_W(-t) = 1 - F_W(t);
  * the integrals over m by the composite Simpson rule on the same grid (m_j = u_j);
  * regions as in oracle/theory.py: unpinned levels only, the leftmost region of a signed codebook starts at -1, the
    region holding the point mass at +1 (and at -1 for absolute normalisation) must be pinned.
"""
import numpy as np


def tables(pdf_fn, cdf_fn, u_max, n):
    """pdf / cdf tables of a distribution given by two callables."""
    assert n % 2 == 1 and n >= 3
    u = np.linspace(0.0, u_max, n)
    return np.asarray(pdf_fn(u), dtype=np.float64), np.asarray(cdf_fn(u), dtype=np.float64)


def upper_first_moment(pdf, u_max):
    """Psi[k] = INT_{u_k}^{u_max} u p(u) du, trapezoid rule."""
    n = pdf.size
    h = u_max / (n - 1)
    f = np.arange(n) * h * pdf
    seg = 0.5 * h * (f[:-1] + f[1:])
    psi = np.zeros(n)
    psi[:-1] = np.cumsum(seg[::-1])[::-1]
    return psi


def _interp(table, t_abs, h):
    pos = t_abs / h
    k = np.minimum(np.floor(pos).astype(np.int64), table.size - 2)
    fr = pos - k
    return table[k] + fr * (table[k + 1] - table[k])


def centroid_update(cb, block, pinned_mask, signed, pdf, cdf, u_max):
    """One theoretical Lloyd iteration for the tabulated distribution: thresholds at mid-points, every unpinned level
    moved to its centroid.  Returns the new float64[16] codebook."""
    cb = np.asarray(cb, dtype=np.float64)
    pdf = np.asarray(pdf, dtype=np.float64)
    cdf = np.asarray(cdf, dtype=np.float64)
    n = pdf.size
    assert n % 2 == 1 and cdf.size == n
    h = u_max / (n - 1)
    m = np.arange(n) * h
    ws = np.ones(n)
    ws[1:-1:2] = 4.0
    ws[2:-1:2] = 2.0
    ws *= h / 3.0
    psi = upper_first_moment(pdf, u_max)
    core = np.zeros(n)
    core[1:] = (2.0 * cdf[1:] - 1.0) ** (block - 2) * pdf[1:]
    xi = 0.5 * (cb[:-1] + cb[1:])

    def F(t):  # F_W(t), t of either sign, |t| <= u_max
        v = _interp(cdf, np.abs(t), h)
        return np.where(t < 0, 1.0 - v, v)

    def Phi1(t):
        return -_interp(psi, np.abs(t), h)

    new = cb.copy()
    for l in range(16):
        if (pinned_mask >> l) & 1:
            continue
        if l == 15 or (l == 0 and not signed):
            raise ValueError("a region that holds a point mass of the normalised weights must be pinned")
        a = xi[l - 1] if l > 0 else -1.0
        a = max(a, -1.0)
        b = xi[l]
        num = np.sum(ws * m * (Phi1(m * b) - Phi1(m * a)) * core)
        den = np.sum(ws * m * m * (F(m * b) - F(m * a)) * core)
        new[l] = num / den
    return new
