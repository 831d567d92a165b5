"""The acceptance checks of the GPU parity tests, exercised on the CPU with the oracle's own output standing in for
the kernels' and mistakes planted in it: a check that cannot fail proves nothing."""
import numpy as np
import pytest

from tests.gpu_common import Case, check_encode


def _case_and_ref(orc, bits=5, d_out=12, d_in=256, block=64):
    rng = np.random.default_rng(5)
    W = rng.standard_normal((d_out, d_in)).astype(np.float32)
    cb = orc.lloyd(orc.gauss_samples(1, 1 << 12), 1 << bits, max_iters=20, tol=1e-5)[0].astype(np.float32)
    sigma = orc.calibrate_sigma(W, block)
    ref = orc.encode(W, cb, bits, block, pair_sigma=sigma, want_x=True)
    case = Case.__new__(Case)
    case.d_in, case.bits, case.cb = d_in, bits, cb
    return case, ref


def _bump(norms, row):
    out = norms.copy()
    out.view(np.int32)[row] += 1
    return out


def test_check_encode_accepts_the_oracles_own_bytes_and_a_one_ulp_norm(orc):
    case, ref = _case_and_ref(orc)
    packed, norms = orc.pack(ref["idx"], case.bits), ref["norms"].astype(np.float32)
    rep = {}
    assert check_encode(orc, case, packed, norms, ref, report=rep) == 0
    assert rep["norm_ulp_rows"] == 0 and rep["mismatches"] == 0
    rep = {}
    check_encode(orc, case, packed, _bump(norms, 2), ref, report=rep)
    assert rep["norm_ulp_rows"] == 1 and rep["norm_ulp_row_mismatches"] == 0


def test_check_encode_rejects_a_wrong_index_in_a_row_with_an_equal_norm(orc):
    case, ref = _case_and_ref(orc)
    idx = ref["idx"].copy()
    idx[3, 5] = (idx[3, 5] + 7) % (1 << case.bits)
    with pytest.raises(AssertionError, match="near-tie"):
        check_encode(orc, case, orc.pack(idx, case.bits), ref["norms"].astype(np.float32), ref)


def test_check_encode_rejects_a_wrong_index_in_a_row_whose_norm_is_one_ulp_off(orc):
    """The hole this closes: such rows used to be left out of the index comparison altogether."""
    case, ref = _case_and_ref(orc)
    norms = _bump(ref["norms"].astype(np.float32), 2)
    idx = ref["idx"].copy()
    idx[2, 9] = (idx[2, 9] + 7) % (1 << case.bits)
    with pytest.raises(AssertionError, match="one ulp off"):
        check_encode(orc, case, orc.pack(idx, case.bits), norms, ref)
    # the runner-up codeword is not accepted either unless the pair is a near-tie: find it by brute force
    x = ref["x"][2, 9]
    d = ((np.asarray(case.cb, dtype=np.float64) - x) ** 2).sum(-1)
    second = int(np.argsort(d, kind="stable")[1])
    assert d[second] > d.min() * (1 + 1e-3)
    idx = ref["idx"].copy()
    idx[2, 9] = second
    with pytest.raises(AssertionError, match="one ulp off"):
        check_encode(orc, case, orc.pack(idx, case.bits), norms, ref)
    # without the oracle's points the check refuses to pass silently
    ref_no_x = dict(ref, x=None)
    with pytest.raises(AssertionError, match="points were not kept"):
        check_encode(orc, case, orc.pack(idx, case.bits), norms, ref_no_x)


def test_check_encode_rejects_a_norm_two_ulps_off_and_nonzero_padding(orc):
    case, ref = _case_and_ref(orc, bits=3, d_in=24, block=8)          # 12 pairs x 3 bits = 36 bits: 28 padding bits
    packed, norms = orc.pack(ref["idx"], case.bits), ref["norms"].astype(np.float32)
    with pytest.raises(AssertionError, match="more than one ulp"):
        check_encode(orc, case, packed, _bump(_bump(norms, 1), 1), ref)
    bad = packed.copy()
    bad[4, -1] |= 0x80
    with pytest.raises(AssertionError, match="padding"):
        check_encode(orc, case, bad, norms, ref)
