"""Pins for the oracle's encode / decode path (Sec. 3.1-3.6, Sec. B.2, Cor. 2, Eq. weight-mse)."""
import os

import numpy as np
import pytest
import scipy.linalg
import torch

from paper_2605_26339_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(lines):
    for line in lines:
        line = line.strip()
        if line and not line.startswith("#"):
            yield line


# ----------------------------------------------------------------------------- bit rate
def test_bpw_printed_values(orc):
    """Eq. 3 and the printed per-model bpw figures (weight-count-weighted over the MLP shapes)."""
    for line in _rows(open(os.path.join(GOLD, "bpw_printed.txt"))):
        tok = line.split()
        label, bits, scaled, printed = tok[0], int(tok[1]), int(tok[2]), tok[3]
        shapes = np.array(list(map(int, tok[4:]))).reshape(-1, 2)
        n = (shapes[:, 0] * shapes[:, 1]).astype(np.float64)
        vals = np.array([orc.bpw(int(di), int(do), bits, bool(scaled)) for do, di in shapes])
        mean = float((vals * n).sum() / n.sum())
        decimals = len(printed.split(".")[1])
        assert abs(mean - float(printed)) <= 0.5 * 10 ** (-decimals) + 1e-12, (label, mean, printed)


# ----------------------------------------------------------------------------- packing
def test_pack_hand_computed_bytes(orc):
    for line in _rows(open(os.path.join(GOLD, "pack_example.txt"))):
        left, right = line.split(":")
        tok = left.split()
        bits = int(tok[0])
        idx = np.array([[int(t, 16) for t in tok[1:]]], dtype=np.int32)
        want = np.array([int(t, 16) for t in right.split()], dtype=np.uint8)
        got = orc.pack(idx, bits)
        assert got.shape == (1, want.size)
        assert np.array_equal(got[0], want)
        assert np.array_equal(orc.unpack(got, 2 * idx.shape[1], bits), idx)


@pytest.mark.parametrize("bits", range(1, 13))
def test_pack_round_trip_all_widths(orc, bits):
    rng = np.random.default_rng(bits)
    for P in (1, 3, 8, 31, 33, 64, 127):
        idx = rng.integers(0, 1 << bits, size=(3, P), dtype=np.int32)
        idx[0, :] = (1 << bits) - 1                               # all ones
        packed = orc.pack(idx, bits)
        rb = orc.packed_row_bytes(2 * P, bits)
        assert packed.shape == (3, rb) and rb % 4 == 0 and rb >= (P * bits + 7) // 8 and rb < (P * bits + 7) // 8 + 4
        assert np.array_equal(orc.unpack(packed, 2 * P, bits), idx)
        # independent statement of the layout: little-endian big integer of the row
        big = int.from_bytes(packed[1].tobytes(), "little")
        for k in range(P):
            assert (big >> (k * bits)) & ((1 << bits) - 1) == idx[1, k]
        assert big >> (P * bits) == 0                             # padding bits are zero


# ----------------------------------------------------------------------------- argmin
def test_argmin_brute_force_tiny(orc):
    """Sec. 3.5 nearest codeword: every pair checked against a numpy brute force in fp64 on a tiny
    problem (K=16, sigma=1, no rotation spread needed: block=2)."""
    rng = np.random.default_rng(11)
    bits, K, d_in, d_out, b = 4, 16, 8, 50, 2
    cb = rng.standard_normal((K, 2)).astype(np.float32)
    W = rng.standard_normal((d_out, d_in)).astype(np.float32)
    sigma = np.full(d_in // 2, 0.5, dtype=np.float32)
    res = orc.encode(W, cb, bits, b, pair_sigma=sigma, mode=orc.MODE_TRUTH, want_x=True)
    x = res["x"]                                                   # [d_out][P][2]
    # independent recomputation of the front half with library routines
    u = W.astype(np.float64) / np.linalg.norm(W.astype(np.float64), axis=1, keepdims=True)
    F = np.kron(np.eye(d_in // b), scipy.linalg.hadamard(b) / np.sqrt(b))
    y = u @ F.T
    assert np.allclose(x.reshape(d_out, d_in), y / 0.5, atol=1e-13)
    d = ((x[:, :, None, :] - cb.astype(np.float64)[None, None, :, :]) ** 2).sum(-1)
    assert np.array_equal(res["idx"], d.argmin(-1))
    srt = np.sort(d, axis=-1)
    assert np.allclose(res["d1"], srt[..., 0], rtol=1e-14) and np.allclose(res["d2"], srt[..., 1], rtol=1e-14)


def test_argmin_exact_ties_take_lowest_index(orc):
    """Planted exact ties: duplicated codewords, and a point exactly on a cell edge."""
    bits, K = 3, 8
    cb = np.array([[1, 0], [0, 1], [-1, 0], [0, -1], [1, 0], [0, 1], [2, 2], [-2, -2]], dtype=np.float32)
    # rows built so that the rotated, normalised pairs are known exactly: d_in=2, block=2:
    # y = (w0+w1, w0-w1)/sqrt(2)/||w||.  w=(1,0): y=(1,1)/sqrt2 -> x = y*sqrt(2) = (1,1) with sigma=1/sqrt(2)
    W = np.array([[1.0, 0.0], [1.0, 1.0], [-3.0, -3.0]], dtype=np.float32)
    sigma = np.array([1.0], dtype=np.float32)
    res = orc.encode(W, cb, bits, 2, pair_sigma=sigma, mode=orc.MODE_TRUTH, want_x=True)
    # row 0: x = (1,1)/sqrt2: equidistant from (1,0) [0 and 4] and (0,1) [1 and 5] -> index 0
    # row 1: x = (1,0): codewords 0 and 4 coincide -> index 0
    # row 2: x = (-1,0): codeword 2
    assert np.allclose(res["x"][1, 0], [1.0, 0.0], atol=1e-15)
    assert res["idx"][:, 0].tolist() == [0, 0, 2]
    assert res["d2"][1, 0] == res["d1"][1, 0] and res["d1"][1, 0] < 1e-30
    assert res["d2"][0, 0] == res["d1"][0, 0]


# ----------------------------------------------------------------------------- front half
def _problem(seed, d_out, d_in, bits, with_scale=True, row_sigma=0.5):
    W = synth.weight_host(seed, d_out, d_in, row_sigma)
    a = synth.act_rms_host(seed + 1, d_in)
    return W, a


def test_front_half_against_library_routines(orc):
    """Steps 1-4 of the encoder with channel scaling: x = (F S (W D_s / r)) / sigma, recomputed
    with numpy/scipy dense algebra.  Catches a dropped scale, a transposed Hadamard, a wrong
    pairing or a wrong division."""
    d_out, d_in, b, bits = 6, 64, 16, 5
    W, a = _problem(21, d_out, d_in, bits)
    s = orc.channel_scales(a, 0.3)
    sg = orc.sign_mask(5, d_in)
    sigma = (np.abs(np.random.default_rng(0).standard_normal(d_in // 2)) * 0.1 + 0.05).astype(np.float32)
    cb = np.random.default_rng(1).standard_normal((1 << bits, 2)).astype(np.float32)
    res = orc.encode(W, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH, want_x=True)
    Ws = W.astype(np.float64) * s.astype(np.float64)[None, :]
    r = np.sqrt((Ws ** 2).sum(1))
    assert np.allclose(res["norms"], r, rtol=1e-14)
    assert np.allclose(res["norms"], np.linalg.norm(Ws, axis=1), rtol=1e-14)   # library norm
    F = np.kron(np.eye(d_in // b), scipy.linalg.hadamard(b) / np.sqrt(b))
    y = (Ws / r[:, None] * sg[None, :]) @ F.T
    x = y.reshape(d_out, d_in // 2, 2) / sigma.astype(np.float64)[None, :, None]
    assert np.allclose(res["x"], x, atol=1e-12)
    # spec mode sees the same numbers up to fp32 rounding
    res32 = orc.encode(W, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_SPEC, want_x=True)
    assert np.abs(res32["x"] - x).max() <= 2e-6 * np.abs(x).max()
    assert np.all(res32["norms"] == res32["norms"].astype(np.float32))
    assert np.allclose(res32["norms"], r, rtol=1e-7)


def test_default_sigma_is_inverse_sqrt_d_in(orc):
    d_out, d_in, b, bits = 4, 32, 8, 4
    W, _ = _problem(3, d_out, d_in, bits)
    cb = np.random.default_rng(1).standard_normal((1 << bits, 2)).astype(np.float32)
    r0 = orc.encode(W, cb, bits, b, mode=orc.MODE_TRUTH, want_x=True)
    r1 = orc.encode(W, cb, bits, b, pair_sigma=np.full(d_in // 2, 1 / np.sqrt(d_in), dtype=np.float64),
                    mode=orc.MODE_TRUTH, want_x=True)
    assert np.allclose(r0["x"], r1["x"], rtol=1e-7)                  # sigma array is fp32
    # a unit-norm row spread evenly has pairs of unit variance per coordinate on average
    assert abs((r0["x"] ** 2).sum() / (d_out * d_in) - 1.0) < 1e-12


def test_zero_row(orc):
    """Sec. 3.1 step 1: a zero row is encoded as a zero row -- decode returns exact zeros."""
    d_in, b, bits = 32, 8, 4
    cb = np.random.default_rng(1).standard_normal((1 << bits, 2)).astype(np.float32)
    W = np.zeros((2, d_in), dtype=np.float32)
    W[1] = 1.0
    for mode in (orc.MODE_TRUTH, orc.MODE_SPEC):
        enc = orc.encode(W, cb, bits, b, mode=mode)
        assert enc["norms"][0] == 0.0
        nearest_origin = int(((cb.astype(np.float64)) ** 2).sum(1).argmin())
        assert np.all(enc["idx"][0] == nearest_origin)
        dec = orc.decode(enc["idx"], enc["norms"], cb, bits, b, mode=mode)
        assert np.all(dec["w"][0] == 0.0) and not np.any(np.signbit(dec["w"][0]) & (dec["w"][0] != 0))
        if mode == orc.MODE_SPEC:
            assert np.all((dec["bf16"][0] & 0x7FFF) == 0)


# ----------------------------------------------------------------------------- channel scales
def test_channel_scales_sec_b2(orc):
    a = synth.act_rms_host(8, 4096)
    for alpha in (0.3, 0.5, 0.8):
        s = orc.channel_scales(a, alpha).astype(np.float64)
        p = a.astype(np.float64) ** alpha
        p /= np.exp(np.log(p).mean())                                   # geometric mean exactly 1
        assert np.allclose(s, np.clip(p, 1 / 16, 16), rtol=2e-7)
        assert s.min() >= 1 / 16 and s.max() <= 16
        if alpha == 0.3:                                                # deployed exponent: clamp never reached
            assert s.min() > 1 / 16 and s.max() < 16
            assert abs(np.exp(np.log(s).mean()) - 1.0) < 1e-6
    assert np.all(orc.channel_scales(a, 0.0) == 1.0)
    # clamp: adversarial spread; power, normalise, then clamp -- no renormalisation afterwards
    adv = np.array([1e-12, 1.0, 1.0, 1e12], dtype=np.float32)
    s = orc.channel_scales(adv, 1.0)
    assert s.tolist() == [1 / 16, 1.0, 1.0, 16.0]
    adv2 = np.array([1.0, 1.0, 1.0, 1e8], dtype=np.float32)          # geo-mean 100 -> 0.01,..,1e6
    s2 = orc.channel_scales(adv2, 1.0)
    assert np.allclose(s2, [1 / 16, 1 / 16, 1 / 16, 16.0])
    # zero activation RMS does not produce inf/nan
    assert np.all(np.isfinite(orc.channel_scales(np.array([0.0, 1.0, 2.0, 4.0], dtype=np.float32), 0.3)))


# ----------------------------------------------------------------------------- sigma calibration
def test_sigma_calibration_eq1(orc):
    """Eq. 1: for iid Gaussian rows the Rayleigh mean gives sigma_k * sqrt(d_in) -> 1."""
    d_out, d_in, b = 1024, 256, 64
    W = np.random.default_rng(2).standard_normal((d_out, d_in)).astype(np.float32)
    sg = orc.sign_mask(4, d_in)
    for mode in (orc.MODE_TRUTH, orc.MODE_SPEC):
        sig = orc.calibrate_sigma(W, b, signs=sg, mode=mode).astype(np.float64)
        z = sig * np.sqrt(d_in)
        # std of one estimate = sqrt((4-pi)/pi)/sqrt(n) = 0.523/sqrt(1024) = 0.0163
        assert abs(z.mean() - 1.0) < 4 * 0.0163 / np.sqrt(d_in // 2) + 2e-3
        assert np.abs(z - 1.0).max() < 6 * 0.0163
    # independent recomputation with dense algebra (truth mode)
    F = np.kron(np.eye(d_in // b), scipy.linalg.hadamard(b) / np.sqrt(b))
    u = W.astype(np.float64) / np.linalg.norm(W.astype(np.float64), axis=1, keepdims=True)
    y = (u * sg[None, :]) @ F.T
    amp = np.sqrt((y.reshape(d_out, -1, 2) ** 2).sum(-1))
    want = amp.mean(0) / np.sqrt(np.pi / 2)
    got = orc.calibrate_sigma(W, b, signs=sg, mode=orc.MODE_TRUTH)
    assert np.allclose(got, want, rtol=2e-7)
    # only the first max_rows rows are used
    got64 = orc.calibrate_sigma(W, b, signs=sg, max_rows=64, mode=orc.MODE_TRUTH)
    assert np.allclose(got64, amp[:64].mean(0) / np.sqrt(np.pi / 2), rtol=2e-7)
    # spec mode agrees with truth mode to fp32 accuracy
    assert np.allclose(orc.calibrate_sigma(W, b, signs=sg, mode=orc.MODE_SPEC), want, rtol=3e-6)


def test_sigma_zero_falls_back(orc):
    W = np.zeros((4, 16), dtype=np.float32)
    W[:, 0] = 1.0                                    # block 0 has energy, block 1 (cols 8..15) none
    sig = orc.calibrate_sigma(W, 8, mode=orc.MODE_TRUTH)
    assert np.all(sig[4:] == np.float32(1 / np.sqrt(16)))
    assert np.all(sig[:4] > 0)


# ----------------------------------------------------------------------------- bf16
def test_bf16_cast_matches_torch(orc):
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(2000).astype(np.float32) * np.exp(rng.standard_normal(2000) * 8).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38, -3.4e38, 1e-40, -1e-45,
                  np.float32(1.0) + np.float32(2 ** -8), np.float32(1.0) + np.float32(2 ** -8) + np.float32(2 ** -23),
                  np.float32(1.0) + np.float32(3 * 2 ** -8)], dtype=np.float32)])
    got = orc.bf16_rne(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- decode identities
@pytest.fixture(scope="module")
def small_codebook(orc):
    samples = orc.gauss_samples(0, 1 << 14)
    cb, mse, it = orc.lloyd(samples, 64, max_iters=60, tol=1e-6)
    return cb.astype(np.float32), mse


def test_decode_against_dense_algebra(orc, small_codebook):
    """Decoder of Sec. 3.2 + Sec. B.2: w_hat = r * S F (sigma * c[idx]) / s, with library algebra."""
    cb, _ = small_codebook
    bits, d_out, d_in, b = 6, 5, 64, 32
    rng = np.random.default_rng(4)
    idx = rng.integers(0, 64, size=(d_out, d_in // 2), dtype=np.int32)
    norms = np.exp(rng.standard_normal(d_out)).astype(np.float32)
    s = orc.channel_scales(synth.act_rms_host(2, d_in), 0.3)
    sg = orc.sign_mask(6, d_in)
    sigma = (0.1 + 0.05 * rng.random(d_in // 2)).astype(np.float32)
    dec = orc.decode(idx, norms, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH,
                     want_yhat=True)
    yhat = (cb.astype(np.float64)[idx] * sigma.astype(np.float64)[None, :, None]).reshape(d_out, d_in)
    assert np.allclose(dec["yhat"], yhat, atol=1e-15)
    F = np.kron(np.eye(d_in // b), scipy.linalg.hadamard(b) / np.sqrt(b))
    want = (yhat @ F.T) * sg[None, :] * norms.astype(np.float64)[:, None] / s.astype(np.float64)[None, :]
    assert np.allclose(dec["w"], want, rtol=1e-12, atol=1e-15)
    spec = orc.decode(idx, norms, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_SPEC)
    rowmax = np.abs(want).max(1, keepdims=True)
    assert (np.abs(spec["w"] - want) / rowmax).max() < 2e-6
    assert np.array_equal(spec["bf16"], orc.bf16_rne(spec["w"].astype(np.float32)))


def test_rotated_domain_error_accounting(orc, small_codebook):
    """Cor. 2: ||u - u~||^2 = sum_k ||z_k - z^_k||^2 and MSE_coord = mean_k(e_k)/2 (truth mode)."""
    cb, _ = small_codebook
    bits, d_out, d_in, b = 6, 8, 256, 64
    W = synth.weight_host(12, d_out, d_in)
    sg = orc.sign_mask(1, d_in)
    sigma = orc.calibrate_sigma(W, b, signs=sg, mode=orc.MODE_TRUTH)
    enc = orc.encode(W, cb, bits, b, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH, want_x=True)
    dec = orc.decode(enc["idx"], enc["norms"], cb, bits, b, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH,
                     want_yhat=True)
    r = np.linalg.norm(W.astype(np.float64), axis=1)
    u = W.astype(np.float64) / r[:, None]
    ut = dec["w"] / enc["norms"].astype(np.float32).astype(np.float64)[:, None]
    z = enc["x"] * sigma.astype(np.float64)[None, :, None]
    zh = dec["yhat"].reshape(d_out, -1, 2)
    e_k = ((z - zh) ** 2).sum(-1)
    lhs = ((u - ut) ** 2).sum(1)
    assert np.allclose(lhs, e_k.sum(1), rtol=1e-6)        # rtol from the fp32 row norm handed to decode
    assert np.allclose(((u - ut) ** 2).mean(1), 0.5 * e_k.mean(1), rtol=1e-6)
    # the decoder's own pair errors equal sigma^2 times the encoder's recorded best distances
    assert np.allclose(e_k, enc["d1"] * sigma.astype(np.float64)[None, :] ** 2, rtol=1e-9, atol=1e-18)


def test_weight_error_matches_codebook_distortion(orc):
    """Eq. weight-mse: E||dW||_F^2 <= (1/2) D_B E||W||_F^2; on Gaussian rows with calibrated
    sigma the relative Frobenius error is close to sqrt(D_B/2)."""
    bits, K = 7, 128
    train = orc.gauss_samples(0, 1 << 15)
    cb64, D_B, _ = orc.lloyd(train, K, max_iters=80, tol=1e-6)
    cb = cb64.astype(np.float32)
    d_out, d_in, b = 96, 512, 128
    W = np.random.default_rng(9).standard_normal((d_out, d_in)).astype(np.float32)
    sg = orc.sign_mask(2, d_in)
    sigma = orc.calibrate_sigma(W, b, signs=sg, mode=orc.MODE_TRUTH)
    enc = orc.encode(W, cb, bits, b, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH)
    dec = orc.decode(enc["idx"], enc["norms"], cb, bits, b, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH)
    rel = np.linalg.norm(dec["w"] - W) / np.linalg.norm(W)
    assert abs(rel / np.sqrt(D_B / 2) - 1.0) < 0.08, (rel, np.sqrt(D_B / 2))


def test_reencode_is_idempotent(orc, small_codebook):
    """encode(decode(idx)) == idx on the value before the bf16 cast."""
    cb, _ = small_codebook
    bits, d_out, d_in, b = 6, 16, 256, 128
    W = synth.weight_host(30, d_out, d_in)
    a = synth.act_rms_host(31, d_in)
    s = orc.channel_scales(a, 0.3)
    sg = orc.sign_mask(3, d_in)
    sigma = orc.calibrate_sigma(W, b, chan_scale=s, signs=sg)
    for mode in (orc.MODE_TRUTH, orc.MODE_SPEC):
        enc = orc.encode(W, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=mode)
        dec = orc.decode(enc["idx"], enc["norms"], cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=mode)
        re = orc.encode(dec["w"].astype(np.float32), cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=mode)
        assert np.array_equal(re["idx"], enc["idx"])


def test_spec_and_truth_modes_agree(orc, small_codebook):
    """fp32 rounding upstream of the argmin may only flip pairs that sit next to a cell edge."""
    cb, _ = small_codebook
    bits, d_out, d_in, b = 6, 64, 512, 128
    W = synth.weight_host(40, d_out, d_in)
    s = orc.channel_scales(synth.act_rms_host(41, d_in), 0.3)
    sg = orc.sign_mask(3, d_in)
    sigma = orc.calibrate_sigma(W, b, chan_scale=s, signs=sg)
    t = orc.encode(W, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH)
    p = orc.encode(W, cb, bits, b, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_SPEC)
    diff = t["idx"] != p["idx"]
    assert diff.mean() < 1e-3
    gap = (t["d2"] - t["d1"]) / t["d2"]
    assert np.all(gap[diff] < 1e-4)
    assert np.allclose(p["norms"], t["norms"], rtol=1e-7)


def test_bf16_input_is_widened_exactly(orc, small_codebook):
    cb, _ = small_codebook
    W = synth.weight_host(50, 4, 64)
    bits16 = synth.to_bf16_bits(W)
    Wb = orc.bf16_bits_to_f32(bits16)
    assert np.array_equal(Wb, torch.from_numpy(W).to(torch.bfloat16).to(torch.float32).numpy())
    assert np.array_equal(orc.bf16_rne(Wb), bits16)


def test_product_with_decoded_rows_equals_product_in_the_rotated_domain(orc):
    """The decoder is linear and F is symmetric (Lemma 1), so <w_i, x> = r_i <yhat_i, F S (x / s)>: a
    product with the decoded matrix can rotate the activation instead of the weights.  Checked on the
    oracle's own fp64 decode; the right-hand side is assembled here from the rotation alone."""
    rng = np.random.default_rng(17)
    d_out, d_in, bits, block = 12, 512, 6, 128
    P = d_in // 2
    cb = rng.standard_normal((1 << bits, 2)).astype(np.float32)
    idx = rng.integers(0, 1 << bits, (d_out, P)).astype(np.int32)
    norms = rng.uniform(0.5, 2.0, d_out).astype(np.float32)
    s = rng.uniform(0.25, 4.0, d_in).astype(np.float32)
    sg = orc.sign_mask(3, d_in)
    sigma = rng.uniform(0.02, 0.08, P).astype(np.float32)
    W = orc.decode(idx, norms, cb, bits, block, chan_scale=s, signs=sg, pair_sigma=sigma, mode=orc.MODE_TRUTH)["w"]
    X = rng.standard_normal((3, d_in))
    direct = X @ W.T
    inv_s = 1.0 / s.astype(np.float64)                             # the fp64 decoder divides by s_j
    Z = np.stack([orc.rotate_fwd_truth(x * inv_s, block, signs=sg) for x in X])        # F S (x / s)
    Zp = Z.reshape(3, P, 2) * sigma.astype(np.float64)[None, :, None]
    C2 = cb.astype(np.float64)[idx]                                # [d_out][P][2]
    rotated = np.einsum("ipe,tpe->ti", C2, Zp) * norms.astype(np.float64)[None, :]
    assert np.allclose(direct, rotated, rtol=1e-10, atol=1e-12)
