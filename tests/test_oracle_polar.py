"""Pins of the oracle's polar baseline (Sec. 3 'Polar Baseline', the pair distortion theorem and the
Rayleigh-Lloyd corollary): none of them re-uses the oracle's own formulas."""
import numpy as np
import pytest


def rayleigh_pdf(r):
    return r * np.exp(-0.5 * r * r)


def simpson(f, a, b, n=20000):
    x = np.linspace(a, b, 2 * n + 1)
    y = f(x)
    return (b - a) / (6 * n) * (y[0] + y[-1] + 4 * y[1::2].sum() + 2 * y[2:-1:2].sum())


@pytest.mark.parametrize("Na", [1, 2, 4, 8, 32])
def test_lloyd_max_conditions_by_quadrature(orc, Na):
    """Each level is the centroid of its cell (thresholds at midpoints), checked by numerical
    integration of r f(r) / f(r); C_LM equals the integrated squared error."""
    lv, c_lm, iters = orc.rayleigh_lloyd_max(Na)
    assert np.all(np.diff(lv) > 0) and lv[0] > 0
    edges = np.concatenate([[0.0], 0.5 * (lv[1:] + lv[:-1]), [8.0]])
    D = 0.0
    for i in range(Na):
        mass = simpson(rayleigh_pdf, edges[i], edges[i + 1])
        cen = simpson(lambda r: r * rayleigh_pdf(r), edges[i], edges[i + 1]) / mass
        assert abs(cen - lv[i]) < 1e-9, (i, cen, lv[i])
        D += simpson(lambda r: (r - lv[i]) ** 2 * rayleigh_pdf(r), edges[i], edges[i + 1])
    assert abs(D - c_lm) < 1e-9                       # the tail beyond 8 carries e^-32
    assert abs(orc.rayleigh_distortion(lv) - c_lm) < 1e-15


def test_one_level_is_the_rayleigh_mean(orc):
    """Na = 1: the level is E U = sqrt(pi/2) and C_LM = Var U = 2 - pi/2 (textbook values)."""
    lv, c_lm, _ = orc.rayleigh_lloyd_max(1)
    assert abs(lv[0] - np.sqrt(np.pi / 2)) < 1e-12
    assert abs(c_lm - (2 - np.pi / 2)) < 1e-12


def test_centroid_identity_and_monotone_distortion(orc):
    """M_a = E[U Q(U)] = E[Q(U)^2] = 2 - C_LM for a centroid quantiser (proof of the corollary), on samples;
    C_LM falls roughly by 4 per extra bit."""
    rng = np.random.default_rng(3)
    u = np.sqrt(-2.0 * np.log(1.0 - rng.random(1 << 20)))
    prev = None
    for Na in (2, 4, 8, 16, 32, 64):
        lv, c_lm, _ = orc.rayleigh_lloyd_max(Na)
        q = lv[np.abs(u[:, None] - lv[None, :]).argmin(1)] if Na <= 16 else lv[np.searchsorted(0.5 * (lv[1:] + lv[:-1]), u)]
        assert abs(np.mean((u - q) ** 2) - c_lm) < 0.02 * c_lm + 1e-4
        assert abs(np.mean(u * q) - (2 - c_lm)) < 5e-3
        if prev is not None:
            assert 2.5 < prev / c_lm < 4.5
        prev = c_lm


def test_polar_quantize_brute_force(orc):
    """Index = nearest amplitude level and nearest phase centre, by brute force over the table's own
    polar coordinates; margins are the distances to the decision boundaries."""
    rng = np.random.default_rng(11)
    lv = orc.rayleigh_lloyd_max(8)[0].astype(np.float32)
    Np = 16
    x = rng.standard_normal((5000, 2)) * 1.3
    q = orc.polar_quantize(x, lv, Np)
    a = np.hypot(x[:, 0], x[:, 1])
    th = np.mod(np.arctan2(x[:, 1], x[:, 0]), 2 * np.pi)
    centres = (2 * np.arange(Np) + 1) * np.pi / Np
    ia = np.abs(a[:, None] - lv[None, :].astype(np.float64)).argmin(1)
    dphi = np.abs(np.angle(np.exp(1j * (th[:, None] - centres[None, :]))))
    ip = dphi.argmin(1)
    assert np.array_equal(q["idx"], ia * Np + ip)
    assert np.allclose(q["phase_margin"], np.pi / Np - dphi.min(1), atol=1e-12)
    # special points: origin, the positive and negative x axis, a bin boundary
    sp = orc.polar_quantize(np.array([[0.0, 0.0], [1.0, 0.0], [-1.0, 0.0], [-1.0, -0.0], [0.0, -2.0]]), lv, Np)
    assert list(sp["idx"] % Np) == [0, 0, Np // 2, Np // 2, 3 * Np // 4]


def test_polar_table_is_the_quantiser_output(orc):
    """Decoding through the 2^B-entry table reproduces amplitude level x unit vector of the phase centre."""
    lv = orc.rayleigh_lloyd_max(4)[0].astype(np.float32)
    Np = 8
    t = orc.polar_table(lv, Np)
    assert t.shape == (32, 2)
    for ia in range(4):
        for ip in range(Np):
            ph = (2 * ip + 1) * np.pi / Np
            assert np.allclose(t[ia * Np + ip], [lv[ia] * np.cos(ph), lv[ia] * np.sin(ph)], rtol=1e-6, atol=1e-7)
    # a table entry quantises to its own index
    q = orc.polar_quantize(t.astype(np.float64), lv, Np)
    assert np.array_equal(q["idx"], np.arange(32))


@pytest.mark.parametrize("Ba,Bp", [(3, 5), (5, 6)])
def test_pair_distortion_theorem_and_corollary(orc, Ba, Bp):
    """Theorem: |z - zh|^2 = (a - ah)^2 + 2 a ah (1 - cos(theta - thetah)) for every pair (exact identity);
    corollary: for circular-Gaussian pairs the mean is C_LM + 2 (2 - C_LM) eta(Np), eta = 1 - sin(h)/h."""
    rng = np.random.default_rng(21)
    Na, Np = 1 << Ba, 1 << Bp
    lv64, c_lm, _ = orc.rayleigh_lloyd_max(Na)
    lv = lv64.astype(np.float32)
    x = rng.standard_normal((1 << 20, 2))
    q = orc.polar_quantize(x, lv, Np)
    zh = orc.polar_table(lv, Np)[q["idx"]].astype(np.float64)
    err = ((x - zh) ** 2).sum(1)
    a, ah = np.hypot(x[:, 0], x[:, 1]), np.hypot(zh[:, 0], zh[:, 1])
    dth = np.arctan2(x[:, 1], x[:, 0]) - np.arctan2(zh[:, 1], zh[:, 0])
    assert np.allclose(err, (a - ah) ** 2 + 2 * a * ah * (1 - np.cos(dth)), rtol=1e-5, atol=1e-9)
    h = np.pi / Np
    eta = 1 - np.sin(h) / h
    closed = c_lm + 2 * (2 - c_lm) * eta
    assert abs(err.mean() - closed) < 0.01 * closed
    assert closed <= c_lm + (2 - c_lm) * np.pi ** 2 / (3 * Np ** 2) + 1e-15     # the corollary's bound


def test_encode_polar_front_half_is_the_joint_front_half(orc):
    """encode_polar quantises exactly the normalised pairs the joint encoder sees."""
    rng = np.random.default_rng(5)
    W = rng.standard_normal((6, 256)).astype(np.float32)
    lv = orc.rayleigh_lloyd_max(8)[0].astype(np.float32)
    sg = orc.sign_mask(9, 256)
    cb = rng.standard_normal((16, 2)).astype(np.float32)
    joint = orc.encode(W, cb, 4, 64, signs=sg, want_x=True)
    pol = orc.encode_polar(W, lv, 4, 64, signs=sg)
    assert np.array_equal(joint["x"], pol["x"]) and np.array_equal(joint["norms"], pol["norms"])
    assert np.array_equal(pol["idx"], orc.polar_quantize(joint["x"], lv, 16)["idx"])
