"""bof4_theory_centroids (section 3.2 eq. 5 evaluated on the GPU from tables of p_W and F_W) against its oracle
(oracle/theory_general.py: the same recipe in numpy).  Both follow one discrete recipe, so they must agree far below
the accuracy of the quadrature itself: 1e-10 relative on every level (sums in another order, another pow)."""
import numpy as np
import pytest
from scipy import stats
from scipy.special import ndtr

from oracle import theory_general
from paper_2505_06653_amd import binding, codebooks

pytestmark = pytest.mark.gpu


def close(a, b):
    return np.all(np.abs(a - b) <= 1e-10 * np.maximum(np.abs(b), 1e-3))


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("signed", [0, 1])
def test_theory_centroids_gaussian_tables(block, signed):
    pdf, cdf = theory_general.tables(lambda u: np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi), ndtr, 16.0, 65537)
    pin = codebooks.PIN_BOF4S if signed else codebooks.PIN_BOF4
    cb = codebooks.gaussian_quantile_init() if signed else codebooks.array(codebooks.BOF4_MSE_64)
    want = theory_general.centroid_update(cb, block, pin, signed, pdf, cdf, 16.0)
    got = binding.bof4_theory_centroids(pdf, cdf, 16.0, block, cb, pin, signed)
    assert close(got, want)
    assert np.array_equal(got[[7, 15]], cb[[7, 15]]) and np.max(np.abs(got - cb)) > 1e-5


def test_theory_centroids_iterated_to_the_fixed_point_of_the_printed_codebook():
    """The printed theoretical BOF4 (MSE) codebook is a fixed point of the GPU update to 2e-7 per step; 400 GPU
    iterations from the quantile start land within 1e-5 of it (the iteration contracts slowly, so the residual of
    the printed digits is amplified to about 5e-6 at the fixed point) and on the oracle's own iterate."""
    from conftest import load_table
    theo = load_table("table_bof4_mse_emp_vs_theo_I64.txt")[:, 1]
    pdf, cdf = theory_general.tables(lambda u: np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi), ndtr, 16.0, 16385)
    once = binding.bof4_theory_centroids(pdf, cdf, 16.0, 64, theo.copy(), codebooks.PIN_BOF4, 0)
    assert np.max(np.abs(once - theo)) < 2e-7
    cb = codebooks.gaussian_quantile_init()
    cb[0] = -1.0
    want = cb.copy()
    for _ in range(400):
        cb = binding.bof4_theory_centroids(pdf, cdf, 16.0, 64, cb, codebooks.PIN_BOF4, 0)
        want = theory_general.centroid_update(want, 64, codebooks.PIN_BOF4, 0, pdf, cdf, 16.0)
    assert np.max(np.abs(cb - theo)) < 1e-5
    assert np.max(np.abs(cb - want)) < 1e-9


def test_theory_centroids_student_t_tables_ragged_grid_and_errors():
    t5 = stats.t(5)
    for n, u_max in ((4097, 300.0), (100001, 512.0), (3, 8.0)):
        pdf, cdf = theory_general.tables(t5.pdf, t5.cdf, u_max, n)
        cb = codebooks.array(codebooks.BOF4S_MSE[64])
        want = theory_general.centroid_update(cb, 64, codebooks.PIN_BOF4S, 1, pdf, cdf, u_max)
        got = binding.bof4_theory_centroids(pdf, cdf, u_max, 64, cb, codebooks.PIN_BOF4S, 1)
        assert close(got, want)
    pdf, cdf = theory_general.tables(t5.pdf, t5.cdf, 64.0, 1025)
    cb = codebooks.array(codebooks.BOF4S_MSE[64])
    with pytest.raises(binding.Bof4Error):   # the region with the point mass at +1 must be pinned
        binding.bof4_theory_centroids(pdf, cdf, 64.0, 64, cb, 1 << 7, 1)
    with pytest.raises(binding.Bof4Error):   # absolute normalisation: level 0 as well
        binding.bof4_theory_centroids(pdf, cdf, 64.0, 64, cb, codebooks.PIN_BOF4S, 0)
    with pytest.raises(binding.Bof4Error):   # even number of grid points
        binding.bof4_theory_centroids(pdf[:-1], cdf[:-1], 64.0, 64, cb, codebooks.PIN_BOF4S, 1)
