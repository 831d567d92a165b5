"""Pins for the oracle's codebook training (Sec. 3.5, Eq. 2) and its sample generator."""
import numpy as np
import pytest
import scipy.stats


def test_samples_are_unit_circular_gaussian(orc):
    """Eq. 2: density exp(-(x^2+y^2)/2)/(2 pi): zero mean, identity covariance, Rayleigh radius,
    uniform angle, independent of each other."""
    n = 1 << 17
    xy = orc.gauss_samples(0, n)
    assert np.abs(xy.mean(0)).max() < 5 / np.sqrt(n)
    cov = np.cov(xy.T)
    assert np.abs(cov - np.eye(2)).max() < 6 / np.sqrt(n)
    r = np.hypot(xy[:, 0], xy[:, 1])
    th = np.arctan2(xy[:, 1], xy[:, 0])
    assert scipy.stats.kstest(r, scipy.stats.rayleigh.cdf).pvalue > 1e-3
    assert scipy.stats.kstest((th + np.pi) / (2 * np.pi), "uniform").pvalue > 1e-3
    assert abs(np.corrcoef(r, th)[0, 1]) < 5 / np.sqrt(n)
    assert abs(r.mean() - np.sqrt(np.pi / 2)) < 5 * 0.655 / np.sqrt(n)      # Rayleigh mean of Sec. 3.4
    # streams: deterministic, seed-dependent, prefix-stable
    assert np.array_equal(xy[:100], orc.gauss_samples(0, 100))
    assert not np.array_equal(xy[:100], orc.gauss_samples(1, 100))


@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_lloyd_small_K_closed_form(orc, K):
    """For K <= 4 the optimal codebook of the circular Gaussian is K points on a ring of radius
    rho = sqrt(pi/2) * sin(pi/K)/(pi/K) (K=1: the origin) with distortion D = 2 - rho^2."""
    n = 1 << 16
    xy = orc.gauss_samples(3, n)
    cb, mse, iters = orc.lloyd(xy, K, max_iters=200, tol=1e-9)
    rho = 0.0 if K == 1 else np.sqrt(np.pi / 2) * np.sin(np.pi / K) / (np.pi / K)
    assert abs(mse - (2 - rho ** 2)) < 0.02
    assert np.abs(np.hypot(cb[:, 0], cb[:, 1]) - rho).max() < 0.05
    if K > 1:
        ang = np.sort(np.mod(np.arctan2(cb[:, 1], cb[:, 0]), 2 * np.pi))
        gaps = np.diff(np.concatenate([ang, ang[:1] + 2 * np.pi]))
        assert np.abs(gaps - 2 * np.pi / K).max() < 0.08


@pytest.fixture(scope="module")
def trained(orc):
    out = {}
    xy = orc.gauss_samples(0, 1 << 16)
    for K in (16, 128, 256):
        cb, mse, iters = orc.lloyd(xy, K, max_iters=150, tol=1e-7)
        out[K] = (cb, mse, iters)
    return xy, out


@pytest.mark.parametrize("K", [16, 128, 256])
def test_lloyd_fixed_point_conditions(orc, trained, K):
    xy, out = trained
    cb, mse, iters = out[K]
    n = xy.shape[0]
    a, e = orc.assign(xy, cb)
    # nearest-neighbour condition, brute force with numpy on a subset
    sub = slice(0, 2000)
    d = ((xy[sub, None, :] - cb[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(a[sub], d.argmin(1))
    assert abs(e.mean() - mse) <= 1e-12 * mse
    # centroid condition: how far is every codeword from the mean of its cell
    cnt = np.bincount(a, minlength=K)
    assert cnt.min() > 0
    mean = np.stack([np.bincount(a, weights=xy[:, 0], minlength=K), np.bincount(a, weights=xy[:, 1], minlength=K)], 1) / cnt[:, None]
    drift = np.abs(mean - cb).max()
    assert drift < 2e-3                                    # stopped by the relative-MSE rule, near the fixed point
    # one more centroid step from here barely lowers the distortion
    _, e2 = orc.assign(xy, mean)
    assert 0 <= mse - e2.mean() < 1e-5 * mse + 1e-9
    # centroid identity (2-D analogue of E[Q^2] = E[X^2] - D), exact when codewords are the cell means
    lhs = (cnt * (mean ** 2).sum(1)).sum()
    a2, e3 = orc.assign(xy, mean)
    emean = ((xy - mean[a]) ** 2).sum()
    assert abs(lhs - ((xy ** 2).sum() - emean)) < 1e-9 * (xy ** 2).sum()
    # symmetry of the source: count-weighted mean of the codebook is the sample mean
    assert np.allclose((cnt[:, None] * mean).sum(0) / n, xy.mean(0), atol=1e-12)


@pytest.mark.parametrize("K", [16, 128])
def test_lloyd_conditions_on_fresh_samples(orc, trained, K):
    xy, out = trained
    cb, mse, _ = out[K]
    fresh = orc.gauss_samples(777, 1 << 17)
    a, e = orc.assign(fresh, cb, threads=4)
    assert abs(e.mean() / mse - 1.0) < 0.05                 # generalises: no over-fit to the training draw
    cnt = np.bincount(a, minlength=K)
    for ax in (0, 1):
        m = np.bincount(a, weights=fresh[:, ax], minlength=K) / cnt
        v = np.bincount(a, weights=fresh[:, ax] ** 2, minlength=K) / cnt - m ** 2
        # the trained point is itself a noisy cell mean of the (smaller) training set: allow both errors
        se = np.sqrt(v / cnt + v / np.maximum(1, cnt // 2))
        assert np.all(np.abs(m - cb[:, ax]) < 5.5 * se + 2e-3)


def test_zador_slope_and_constant(orc, trained):
    """High-rate scaling: one more bit per pair halves D_B; the level is about 2 G(2) * 8 pi / K
    for this source (G(2) = 5/(36 sqrt 3), the hexagonal-lattice constant)."""
    _, out = trained
    D7, D8 = out[128][1], out[256][1]
    assert abs(D7 / D8 - 2.0) < 0.3
    G2 = 5 / (36 * np.sqrt(3))
    for K in (128, 256):
        assert abs(out[K][1] / (2 * G2 * 8 * np.pi / K) - 1.0) < 0.25


def test_init_is_spread_over_the_source(orc):
    cb = orc.codebook_init(2048)
    r = np.hypot(cb[:, 0], cb[:, 1])
    assert np.all(np.diff(r) > 0) and r.max() < 6.0 and r.min() < 0.1
    # no two initial points coincide
    d = ((cb[:200, None, :] - cb[None, :200, :]) ** 2).sum(-1) + np.eye(200)
    assert d.min() > 1e-6
