"""Pins for the oracle's rotation (Defs 1-3, Lemma 1 and the two remarks after it)."""
import os

import numpy as np
import pytest
import scipy.linalg

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("b", [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_hadamard_matrix_def1(orc, b):
    H = orc.hadamard(b).astype(np.int64)
    # Def. 1: H^T H = b I and H = H^T, exactly, in integers
    assert np.array_equal(H.T @ H, b * np.eye(b, dtype=np.int64))
    assert np.array_equal(H, H.T)
    assert set(np.unique(H)) <= {-1, 1}
    # library routine: scipy builds the same Sylvester matrix
    assert np.array_equal(H, scipy.linalg.hadamard(b).astype(np.int64))
    # closed form of the Sylvester recursion: entry (i, j) = (-1)^popcount(i & j)
    i, j = np.meshgrid(np.arange(b), np.arange(b), indexing="ij")
    pop = np.vectorize(lambda v: bin(v).count("1"))(i & j)
    assert np.array_equal(H, 1 - 2 * (pop & 1))


def test_block_size_rule_worked_examples(orc):
    for line in open(os.path.join(GOLD, "block_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d_in, b = map(int, line.split())
        assert orc.paper_block_size(d_in) == b
    assert orc.paper_block_size(4096) == 1024          # cap
    assert orc.paper_block_size(11008) == 256          # 11008 = 2^8 * 43
    assert orc.paper_block_size(6) == 2


@pytest.mark.parametrize("b,m", [(2, 3), (8, 5), (128, 4), (256, 2), (1024, 1)])
def test_rotation_isometry_lemma1(orc, b, m):
    rng = np.random.default_rng(b + m)
    d = b * m
    s = orc.sign_mask(1234 + b, d)
    v, w = rng.standard_normal(d), rng.standard_normal(d)
    yv, yw = orc.rotate_fwd_truth(v, b, s), orc.rotate_fwd_truth(w, b, s)
    # norms, inner products, distances
    assert abs(np.linalg.norm(yv) - np.linalg.norm(v)) <= 1e-13 * np.linalg.norm(v)
    assert abs(yv @ yw - v @ w) <= 1e-12 * np.linalg.norm(v) * np.linalg.norm(w)
    assert abs(np.linalg.norm(yv - yw) - np.linalg.norm(v - w)) <= 1e-12 * np.linalg.norm(v - w)
    # per-block energy
    eb = (v.reshape(m, b) ** 2).sum(1)
    assert np.allclose((yv.reshape(m, b) ** 2).sum(1), eb, rtol=1e-12)
    # R_inv R_fwd = I and R_fwd R_inv = I
    assert np.allclose(orc.rotate_inv_truth(yv, b, s), v, atol=1e-13 * np.abs(v).max() * b)
    assert np.allclose(orc.rotate_fwd_truth(orc.rotate_inv_truth(v, b, s), b, s), v, atol=1e-12)


def test_rotation_is_F_times_S_not_S_times_F(orc):
    """R_fwd = F S (sign first, then Hadamard): checked against a dense product built with a
    library Hadamard matrix; also the remark that F and S do not commute / no involution."""
    b, m = 16, 3
    d = b * m
    rng = np.random.default_rng(0)
    s = orc.sign_mask(99, d).astype(np.float64)
    assert len(set(s[:b])) == 2                              # non-trivial mask
    F = np.kron(np.eye(m), scipy.linalg.hadamard(b) / np.sqrt(b))
    S = np.diag(s)
    v = rng.standard_normal(d)
    y = orc.rotate_fwd_truth(v, b, s.astype(np.int8))
    assert np.allclose(y, F @ S @ v, atol=1e-13)
    assert not np.allclose(y, S @ F @ v, atol=1e-3)          # swapped order is a different map
    assert np.allclose(orc.rotate_inv_truth(v, b, s.astype(np.int8)), S @ F @ v, atol=1e-13)
    # not an involution: applying R_fwd twice does not return the input
    assert not np.allclose(orc.rotate_fwd_truth(y, b, s.astype(np.int8)), v, atol=1e-3)
    # with the trivial mask it IS an involution (F symmetric orthogonal)
    y1 = orc.rotate_fwd_truth(v, b, None)
    assert np.allclose(orc.rotate_fwd_truth(y1, b, None), v, atol=1e-13)


@pytest.mark.parametrize("b", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_butterflies_equal_explicit_matrix(orc, b):
    """The fp32 butterfly network reproduces H_b v exactly when every intermediate is an
    integer below 2^24 (no rounding happens), for every block size."""
    rng = np.random.default_rng(b)
    v = rng.integers(-8, 9, size=b).astype(np.float32)
    t = orc.fwht_spec(v)
    H = scipy.linalg.hadamard(b).astype(np.int64)
    assert np.array_equal(t.astype(np.int64), H @ v.astype(np.int64))


def test_spec_rotation_close_to_truth(orc):
    rng = np.random.default_rng(5)
    for b, d in [(128, 2048), (256, 1024), (1024, 2048)]:
        s = orc.sign_mask(7, d)
        u = rng.standard_normal(d)
        u /= np.linalg.norm(u)
        yt = orc.rotate_fwd_truth(u, b, s)
        ys = orc.rotate_fwd_spec(u.astype(np.float32), b, s)
        yt32 = orc.rotate_fwd_truth(u.astype(np.float32).astype(np.float64), b, s)
        assert np.abs(ys - yt32).max() <= 4e-7 * np.abs(yt).max() * np.log2(b)


def test_sign_mask_spreads_energy_remark(orc):
    """Remark after Lemma 1: over Rademacher signs E[(R_fwd v)_j] = 0 and
    E[(R_fwd v)_j^2] = ||v_B(j)||^2 / b.  Averaged over 4000 seeded masks."""
    b, m = 32, 2
    d = b * m
    rng = np.random.default_rng(3)
    v = rng.standard_normal(d) * np.exp(rng.standard_normal(d))      # coherent, spiky
    n = 4000
    acc1, acc2 = np.zeros(d), np.zeros(d)
    balance = 0.0
    for seed in range(n):
        s = orc.sign_mask(seed, d)
        balance += s.astype(np.float64).mean()
        y = orc.rotate_fwd_truth(v, b, s)
        acc1 += y
        acc2 += y * y
    target = np.repeat((v.reshape(m, b) ** 2).sum(1) / b, b)
    assert np.abs(acc2 / n - target).max() <= 0.12 * target.max()
    assert np.abs(acc1 / n).max() <= 5 * np.sqrt(target.max() / n)
    assert abs(balance / n) < 0.01                                     # masks are balanced


def test_sign_mask_definition(orc):
    s = orc.sign_mask(0xDEADBEEF, 200)
    assert s.dtype == np.int8 and set(np.unique(s)) == {-1, 1}
    assert np.array_equal(s, orc.sign_mask(0xDEADBEEF, 200))           # deterministic in the seed
    assert not np.array_equal(s, orc.sign_mask(0xDEADBEEF + 1, 200))
    assert np.array_equal(s[:130], orc.sign_mask(0xDEADBEEF, 130))     # prefix-stable
