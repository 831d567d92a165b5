"""CPU-side checks of libqamw: the library loads, exports every declared symbol, rejects invalid
arguments before any launch, and its host helpers agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_26339_amd import qamw, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "qamw.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(qamw_[a-z0-9_]+)\s*\(", header)))
    assert len(declared) >= 12
    L = qamw.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(qamw.EXPORTS) == declared


def test_status_strings():
    seen = {qamw.status_string(s) for s in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert qamw.status_string(99) == "unknown status"


def test_host_helpers_match_oracle(orc):
    for d_in, bits in [(2048, 11), (2048, 7), (5632, 11), (11008, 7), (2, 1), (6, 3), (62, 11), (13824, 12)]:
        assert qamw.packed_row_bytes(d_in, bits) == orc.packed_row_bytes(d_in, bits)
    for d_in in [2, 6, 24, 2048, 4096, 5120, 5632, 11008, 13824, 14336, 1 << 20]:
        assert qamw.paper_block_size(d_in) == orc.paper_block_size(d_in)
    for d_in, d_out, bits, sc in [(2048, 5632, 11, False), (5632, 2048, 7, True), (4096, 14336, 8, True)]:
        assert qamw.bpw(d_in, d_out, bits, sc) == orc.bpw(d_in, d_out, bits, sc)
    for seed, d in [(0, 1), (1, 64), (2**63 + 5, 65), (12345, 13824)]:
        assert np.array_equal(qamw.sign_mask(seed, d), orc.sign_mask(seed, d))
    for seed in (1, 2):
        a = synth.act_rms_host(seed, 4096)
        for alpha in (0.0, 0.3, 0.5, 1.0):
            got, want = qamw.channel_scales(a, alpha), orc.channel_scales(a, alpha)
            assert np.allclose(got, want, rtol=2e-7, atol=0)
    adv = np.array([0.0, 1e-12, 1.0, 1e12], dtype=np.float32)
    assert np.allclose(qamw.channel_scales(adv, 1.0), orc.channel_scales(adv, 1.0), rtol=2e-7)


def test_host_helper_errors():
    L = qamw.lib()
    out = C.c_size_t()
    assert L.qamw_packed_row_bytes(2048, 0, C.byref(out)) == qamw.ERR_INVALID_ARG
    assert L.qamw_packed_row_bytes(2048, 13, C.byref(out)) == qamw.ERR_INVALID_ARG
    assert L.qamw_packed_row_bytes(2047, 11, C.byref(out)) == qamw.ERR_SHAPE
    assert L.qamw_packed_row_bytes(0, 11, C.byref(out)) == qamw.ERR_SHAPE
    assert L.qamw_packed_row_bytes(2048, 11, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_sign_mask(0, 16, None) == qamw.ERR_INVALID_ARG
    a = np.ones(4, dtype=np.float32)
    assert L.qamw_channel_scales(a.ctypes.data, 4, C.c_float(1.5), a.ctypes.data) == qamw.ERR_INVALID_ARG
    cb = np.zeros((4, 2), dtype=np.float32)
    assert L.qamw_train_codebook(0, 1024, 0, 10, 1e-6, cb.ctypes.data, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_train_codebook(2, 3, 0, 10, 1e-6, cb.ctypes.data, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_train_codebook(2, 1024, 0, 0, 1e-6, cb.ctypes.data, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_train_codebook(2, 1024, 0, 10, 1e-6, None, None, None) == qamw.ERR_INVALID_ARG


def test_device_entry_points_reject_bad_arguments_before_any_launch():
    """Every argument error is reported synchronously, on the host, before HIP is touched: these
    calls run on a machine with no GPU.  Pointers are dummies that are never dereferenced."""
    L = qamw.lib()
    p = C.c_void_p(0x1000)
    good = dict(W=p, dtype=0, d_out=8, d_in=256, ldw=256, s=None, sg=None, sig=None, cb=p, bits=11, block=128,
                packed=p, norms=p, stream=None)

    def enc(**kw):
        a = {**good, **kw}
        return L.qamw_encode(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], a["s"], a["sg"], a["sig"], a["cb"],
                             a["bits"], a["block"], a["packed"], a["norms"], a["stream"])

    def dec(fn=None, **kw):
        a = {**good, **kw}
        fn = fn or L.qamw_decode
        return fn(a["packed"], a["norms"], a["d_out"], a["d_in"], a["s"], a["sg"], a["sig"], a["cb"], a["bits"],
                  a["block"], a["W"], a["ldw"], a["stream"])

    for f in (enc, dec, lambda **kw: dec(fn=L.qamw_decode_f32, **kw)):
        assert f(W=None) == qamw.ERR_INVALID_ARG
        assert f(cb=None) == qamw.ERR_INVALID_ARG
        assert f(packed=None) == qamw.ERR_INVALID_ARG
        assert f(norms=None) == qamw.ERR_INVALID_ARG
        assert f(d_out=0) == qamw.ERR_INVALID_ARG
        assert f(d_in=-2) == qamw.ERR_INVALID_ARG
        assert f(bits=0) == qamw.ERR_INVALID_ARG
        assert f(bits=13) == qamw.ERR_INVALID_ARG
        assert f(d_in=255, ldw=255) == qamw.ERR_SHAPE          # odd row length
        assert f(block=96) == qamw.ERR_SHAPE                   # not a power of two
        assert f(block=1) == qamw.ERR_SHAPE
        assert f(block=2048) == qamw.ERR_SHAPE                 # above the largest block
        assert f(d_in=384, ldw=384, block=256) == qamw.ERR_SHAPE   # does not divide d_in
        assert f(ldw=255) == qamw.ERR_SHAPE                    # leading dimension too small
    assert enc(dtype=7) == qamw.ERR_INVALID_ARG
    # the packed stream is handled in 32-bit words: a buffer that is not 4-byte aligned is rejected
    assert enc(packed=C.c_void_p(0x1002)) == qamw.ERR_INVALID_ARG
    assert dec(packed=C.c_void_p(0x1001)) == qamw.ERR_INVALID_ARG
    a = good
    assert L.qamw_encode_stats(a["W"], 0, 8, 256, 256, None, None, None, a["cb"], 11, 128, a["packed"], a["norms"], None,
                               None) == qamw.ERR_INVALID_ARG          # the counter is required
    assert L.qamw_encode_stats(None, 0, 8, 256, 256, None, None, None, a["cb"], 11, 128, a["packed"], a["norms"], p,
                               None) == qamw.ERR_INVALID_ARG

    def cal(**kw):
        a = {**good, "max_rows": 1024, "ws": p, "ws_bytes": 1 << 30, **kw}
        return L.qamw_calibrate_sigma(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], a["s"], a["sg"], a["block"],
                                      a["max_rows"], a["ws"], a["ws_bytes"], a["packed"], a["stream"])

    assert cal(W=None) == qamw.ERR_INVALID_ARG
    assert cal(ws=None) == qamw.ERR_INVALID_ARG
    assert cal(packed=None) == qamw.ERR_INVALID_ARG
    assert cal(max_rows=0) == qamw.ERR_INVALID_ARG
    assert cal(block=3) == qamw.ERR_SHAPE
    assert cal(ldw=10) == qamw.ERR_SHAPE
    assert cal(dtype=2) == qamw.ERR_INVALID_ARG
    need = qamw.calibrate_workspace_bytes(256, 8, 1024)
    assert need >= 8 * 4 + 128 * 8
    assert cal(ws_bytes=need - 1) == qamw.ERR_INVALID_ARG          # workspace too small
    assert cal(ws=C.c_void_p(0x1004)) == qamw.ERR_INVALID_ARG      # workspace not 16-byte aligned
    # the workspace grows with the rows used and the row length, and is capped by max_rows
    assert qamw.calibrate_workspace_bytes(4096, 11008, 1024) == qamw.calibrate_workspace_bytes(4096, 1024, 1024)
    assert qamw.calibrate_workspace_bytes(4096, 11008, 64) < qamw.calibrate_workspace_bytes(4096, 11008, 1024)
    out = C.c_size_t()
    assert L.qamw_calibrate_workspace_bytes(255, 8, 1024, C.byref(out)) == qamw.ERR_SHAPE
    assert L.qamw_calibrate_workspace_bytes(256, 8, 0, C.byref(out)) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_workspace_bytes(256, 8, 1024, None) == qamw.ERR_INVALID_ARG


    # the variant with the library's own static scratch: same checks, and the size limit, all before HIP is touched
    def cal_static(**kw):
        a = {**good, "max_rows": 1024, **kw}
        return L.qamw_calibrate_sigma_static(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], a["s"], a["sg"], a["block"],
                                             a["max_rows"], a["packed"], a["stream"])

    assert cal_static(W=None) == qamw.ERR_INVALID_ARG
    assert cal_static(packed=None) == qamw.ERR_INVALID_ARG
    assert cal_static(max_rows=0) == qamw.ERR_INVALID_ARG
    assert cal_static(block=3) == qamw.ERR_SHAPE
    assert cal_static(ldw=10) == qamw.ERR_SHAPE
    assert cal_static(dtype=2) == qamw.ERR_INVALID_ARG
    assert qamw.calibrate_workspace_bytes(16384, 4096, 1024) <= qamw.STATIC_SCRATCH_BYTES
    assert cal_static(d_out=2048, d_in=16512, ldw=16512) == qamw.ERR_UNSUPPORTED   # beyond the static scratch


def test_encode_batch_rejects_bad_arguments():
    L = qamw.lib()
    p = C.c_void_p(0x1000)
    arr = (qamw.EncodeItem * 2)()
    for i in range(2):
        arr[i] = qamw.EncodeItem(0x1000, 256, None, None, None, 0x2000, 0x3000, 8, 256)
    assert L.qamw_encode_batch(None, 2, 0, p, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_encode_batch(arr, 0, 0, p, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_encode_batch(arr, qamw.MAX_BATCH + 1, 0, p, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_encode_batch(arr, 2, 0, None, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_encode_batch(arr, 2, 5, p, 11, 128, None) == qamw.ERR_INVALID_ARG          # element type
    assert L.qamw_encode_batch(arr, 2, 0, p, 13, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_encode_batch(arr, 2, 0, p, 11, 96, None) == qamw.ERR_SHAPE
    arr[1].ldw = 100
    assert L.qamw_encode_batch(arr, 2, 0, p, 11, 128, None) == qamw.ERR_SHAPE                # leading dimension too small
    arr[1].ldw = 256
    arr[1].packed_out = None
    assert L.qamw_encode_batch(arr, 2, 0, p, 11, 128, None) == qamw.ERR_INVALID_ARG
    arr[1].packed_out = 0x2000
    arr[0].d_in = 255
    assert L.qamw_encode_batch(arr, 2, 0, p, 11, 128, None) == qamw.ERR_SHAPE


def test_calibrate_batch_rejects_bad_arguments():
    L = qamw.lib()
    p = C.c_void_p(0x1000)
    arr = (qamw.CalibrateItem * 2)()
    for i in range(2):
        arr[i] = qamw.CalibrateItem(0x1000, 256, None, None, 0x2000, 8, 256)
    big = 1 << 30
    assert L.qamw_calibrate_sigma_batch(None, 2, 0, 128, 1024, p, big, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_sigma_batch(arr, 0, 0, 128, 1024, p, big, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_sigma_batch(arr, qamw.MAX_BATCH + 1, 0, 128, 1024, p, big, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 1024, None, big, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 1024, C.c_void_p(0x1004), big, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_calibrate_sigma_batch(arr, 2, 3, 128, 1024, p, big, None) == qamw.ERR_INVALID_ARG      # element type
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 0, p, big, None) == qamw.ERR_INVALID_ARG         # max_rows
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 96, 1024, p, big, None) == qamw.ERR_SHAPE
    need = 2 * ((qamw.calibrate_workspace_bytes(256, 8, 1024) + 255) // 256 * 256)
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 1024, p, need - 1, None) == qamw.ERR_INVALID_ARG   # workspace too small
    arr[1].sigma_out = None
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 1024, p, big, None) == qamw.ERR_INVALID_ARG
    arr[1].sigma_out = 0x2000
    arr[1].ldw = 10
    assert L.qamw_calibrate_sigma_batch(arr, 2, 0, 128, 1024, p, big, None) == qamw.ERR_SHAPE


def test_decode_batch_rejects_bad_arguments():
    L = qamw.lib()
    p = 0x1000
    def item(**kw):
        a = dict(packed=p, row_norms=p, chan_scale=None, signs=None, pair_sigma=None, W_out=p, ldo=256, d_out=8, d_in=256)
        a.update(kw)
        return qamw.DecodeItem(**a)
    arr = (qamw.DecodeItem * 2)(item(), item())
    cb = C.c_void_p(p)
    assert L.qamw_decode_batch(None, 2, cb, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_decode_batch(arr, 0, cb, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_decode_batch(arr, qamw.MAX_BATCH + 1, cb, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_decode_batch(arr, 2, None, 11, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_decode_batch(arr, 2, cb, 0, 128, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_decode_batch(arr, 2, cb, 11, 96, None) == qamw.ERR_SHAPE
    for bad, want in [(item(packed=None), qamw.ERR_INVALID_ARG), (item(W_out=None), qamw.ERR_INVALID_ARG),
                      (item(row_norms=None), qamw.ERR_INVALID_ARG), (item(d_in=255), qamw.ERR_SHAPE),
                      (item(ldo=100), qamw.ERR_SHAPE), (item(d_out=0), qamw.ERR_INVALID_ARG),
                      (item(d_in=384, ldo=384), qamw.ERR_SHAPE)]:
        arr2 = (qamw.DecodeItem * 2)(item(), bad)
        assert L.qamw_decode_batch(arr2, 2, cb, 11, 256 if bad.d_in == 384 else 128, None) == want


def test_polar_codebook_matches_oracle_and_rejects_bad_arguments(orc):
    """The library integrates the Rayleigh density numerically, the oracle in closed form: same levels."""
    for ba, bp in [(0, 4), (1, 1), (3, 5), (5, 6), (6, 4)]:
        lv, table, c_lm = qamw.polar_codebook(ba, bp)
        olv, oc, _ = orc.rayleigh_lloyd_max(1 << ba)
        assert np.abs(lv - olv).max() < 3e-7 and abs(c_lm - oc) < 1e-9
        assert np.array_equal(table, orc.polar_table(lv, 1 << bp))
    L = qamw.lib()
    buf = np.zeros(8192, dtype=np.float32)
    ptr = buf.ctypes.data_as(C.c_void_p)
    assert L.qamw_polar_codebook(7, 2, ptr, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_polar_codebook(-1, 2, ptr, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_polar_codebook(0, 0, ptr, None, None) == qamw.ERR_INVALID_ARG
    assert L.qamw_polar_codebook(6, 7, ptr, None, None) == qamw.ERR_INVALID_ARG          # 13 bits in all
    assert L.qamw_polar_codebook(3, 3, None, None, None) == qamw.ERR_INVALID_ARG
    p = C.c_void_p(0x1000)

    def enc(**kw):
        a = dict(W=p, dtype=0, d_out=8, d_in=256, ldw=256, lv=p, ba=5, bp=6, block=128, packed=p, norms=p)
        a.update(kw)
        return L.qamw_encode_polar(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], None, None, None, a["lv"], a["ba"],
                                   a["bp"], a["block"], a["packed"], a["norms"], None)

    assert enc(W=None) == qamw.ERR_INVALID_ARG
    assert enc(lv=None) == qamw.ERR_INVALID_ARG
    assert enc(packed=None) == qamw.ERR_INVALID_ARG
    assert enc(ba=7) == qamw.ERR_INVALID_ARG
    assert enc(ba=6, bp=7) == qamw.ERR_INVALID_ARG           # 13 bits
    assert enc(ba=0, bp=0) == qamw.ERR_INVALID_ARG
    assert enc(dtype=3) == qamw.ERR_INVALID_ARG
    assert enc(d_in=255, ldw=255) == qamw.ERR_SHAPE
    assert enc(block=96) == qamw.ERR_SHAPE
    assert enc(ldw=100) == qamw.ERR_SHAPE
    # valid arguments outside the kernel's range: reported as unsupported, nothing launched
    assert enc(d_in=64, ldw=64, block=32) == qamw.ERR_UNSUPPORTED
    assert enc(d_in=72, ldw=72, block=8) == qamw.ERR_UNSUPPORTED
    assert enc(W=C.c_void_p(0x1004)) == qamw.ERR_UNSUPPORTED  # W not 16-byte aligned


def test_matmul_rejects_bad_arguments():
    L = qamw.lib()
    p = C.c_void_p(0x1000)
    need = qamw.matmul_workspace_bytes(256, 8, 2)
    assert need == 2 * 256 * 4
    assert qamw.matmul_workspace_bytes(11008, 4096, 8) == 8 * 11008 * 4

    def mm(**kw):
        a = dict(X=p, xd=0, m=2, ldx=256, packed=p, norms=p, d_out=8, d_in=256, cb=p, bits=11, block=128, ws=p,
                 ws_bytes=need, Y=p, ldy=8)
        a.update(kw)
        return L.qamw_matmul(a["X"], a["xd"], a["m"], a["ldx"], a["packed"], a["norms"], a["d_out"], a["d_in"], None, None,
                             None, a["cb"], a["bits"], a["block"], a["ws"], a["ws_bytes"], a["Y"], a["ldy"], None)

    for k in ("X", "packed", "norms", "cb", "ws", "Y"):
        assert mm(**{k: None}) == qamw.ERR_INVALID_ARG
    assert mm(m=0) == qamw.ERR_INVALID_ARG
    assert mm(m=qamw.MATMUL_MAX_ROWS + 1) == qamw.ERR_INVALID_ARG
    assert mm(xd=5) == qamw.ERR_INVALID_ARG
    assert mm(bits=0) == qamw.ERR_INVALID_ARG
    assert mm(ws_bytes=need - 1) == qamw.ERR_INVALID_ARG
    assert mm(ws=C.c_void_p(0x1008)) == qamw.ERR_INVALID_ARG
    assert mm(ldx=100) == qamw.ERR_SHAPE
    assert mm(ldy=4) == qamw.ERR_SHAPE
    assert mm(block=96) == qamw.ERR_SHAPE
    assert mm(bits=9) == qamw.ERR_UNSUPPORTED                 # only 7, 8 and 11 bits
    assert mm(d_in=64, ldx=64, block=32) == qamw.ERR_UNSUPPORTED
    assert mm(packed=C.c_void_p(0x1002)) == qamw.ERR_UNSUPPORTED
    out = C.c_size_t()
    assert L.qamw_matmul_workspace_bytes(256, 8, qamw.MATMUL_MAX_ROWS + 1, C.byref(out)) == qamw.ERR_INVALID_ARG
    # beyond 64 rows: the workspace of one tile (65 rows = tiles of 33 and 32; 200 rows = four tiles of 50), padded to 32
    assert L.qamw_matmul_workspace_bytes(256, 8, 65, C.byref(out)) == qamw.OK and out.value == 64 * 256 * 2
    assert L.qamw_matmul_workspace_bytes(256, 8, 200, C.byref(out)) == qamw.OK and out.value == 64 * 256 * 2
    assert L.qamw_matmul_workspace_bytes(256, 8, 4096, C.byref(out)) == qamw.OK and out.value == 64 * 256 * 2
    assert L.qamw_matmul_workspace_bytes(256, 8, 9, C.byref(out)) == qamw.OK and out.value == 32 * 256 * 2   # bf16 rows, padded to 32
    assert L.qamw_matmul_workspace_bytes(256, 8, 33, C.byref(out)) == qamw.OK and out.value == 64 * 256 * 2
    assert L.qamw_matmul_workspace_bytes(255, 8, 1, C.byref(out)) == qamw.ERR_SHAPE
    assert L.qamw_matmul_workspace_bytes(256, 8, 1, None) == qamw.ERR_INVALID_ARG


def test_device_lloyd_and_pairs_reject_bad_arguments():
    L = qamw.lib()
    p = C.c_void_p(0x1000)
    need = C.c_size_t()
    assert L.qamw_lloyd_workspace_bytes(11, C.byref(need)) == qamw.OK and need.value >= 2048 * 40
    assert L.qamw_lloyd_workspace_bytes(0, C.byref(need)) == qamw.ERR_INVALID_ARG
    assert L.qamw_lloyd_workspace_bytes(11, None) == qamw.ERR_INVALID_ARG

    def ll(**kw):
        a = dict(samples=p, n=4096, bits=4, cb=p, iters=10, tol=1e-6, ws=p, ws_bytes=1 << 20)
        a.update(kw)
        return L.qamw_lloyd_device(a["samples"], a["n"], a["bits"], a["cb"], a["iters"], a["tol"], a["ws"], a["ws_bytes"], None,
                                   None, None)

    assert ll(samples=None) == qamw.ERR_INVALID_ARG
    assert ll(cb=None) == qamw.ERR_INVALID_ARG
    assert ll(ws=None) == qamw.ERR_INVALID_ARG
    assert ll(bits=0) == qamw.ERR_INVALID_ARG
    assert ll(bits=13) == qamw.ERR_INVALID_ARG
    assert ll(n=8) == qamw.ERR_INVALID_ARG                    # fewer samples than points
    assert ll(n=(1 << 24) + 1) == qamw.ERR_INVALID_ARG
    assert ll(iters=0) == qamw.ERR_INVALID_ARG
    assert ll(tol=-1.0) == qamw.ERR_INVALID_ARG
    assert ll(ws_bytes=100) == qamw.ERR_INVALID_ARG
    assert ll(ws=C.c_void_p(0x1008)) == qamw.ERR_INVALID_ARG
    assert ll(samples=C.c_void_p(0x1004)) == qamw.ERR_INVALID_ARG

    def pr(**kw):
        a = dict(W=p, dtype=0, d_out=8, d_in=256, ldw=256, block=128, pairs=p, norms=p)
        a.update(kw)
        return L.qamw_normalised_pairs(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], None, None, None, a["block"],
                                       a["pairs"], a["norms"], None)

    assert pr(W=None) == qamw.ERR_INVALID_ARG
    assert pr(pairs=None) == qamw.ERR_INVALID_ARG
    assert pr(norms=None) == qamw.ERR_INVALID_ARG
    assert pr(dtype=4) == qamw.ERR_INVALID_ARG
    assert pr(d_in=255, ldw=255) == qamw.ERR_SHAPE
    assert pr(block=48) == qamw.ERR_SHAPE
    assert pr(d_in=64, ldw=64, block=32) == qamw.ERR_UNSUPPORTED
    assert pr(pairs=C.c_void_p(0x1004)) == qamw.ERR_UNSUPPORTED


def test_kernel_path_switch():
    prev = qamw.set_kernel_path(1)
    assert qamw.set_kernel_path(0) == 1
    assert qamw.set_kernel_path(5) == 0          # invalid value: unchanged, returns current
    qamw.set_kernel_path(prev)


# ----------------------------------------------------------------------------- codebook trainer
@pytest.mark.parametrize("bits", [2, 4, 6])
def test_trainer_follows_the_oracle_lloyd(orc, bits):
    """Same samples, same initial points, same stopping rule: the library's grid-accelerated
    trainer must walk the same path as the plain Lloyd iteration."""
    n = 1 << 14
    cb, mse, it = qamw.train_codebook(bits, n, seed=5, max_iters=40, tol=1e-6)
    xy = orc.gauss_samples(5, n)
    ref, ref_mse, ref_it = orc.lloyd(xy, 1 << bits, max_iters=40, tol=1e-6)
    assert it == ref_it
    assert abs(mse - ref_mse) <= 1e-12 * ref_mse
    assert np.array_equal(cb, ref.astype(np.float32)) or np.abs(cb - ref).max() < 1e-7


def test_trainer_single_iteration_returns_initial_points(orc):
    cb, mse, it = qamw.train_codebook(5, 4096, seed=1, max_iters=1, tol=0.0)
    assert it == 1
    assert np.array_equal(cb, orc.codebook_init(32).astype(np.float32))
    _, e = orc.assign(orc.gauss_samples(1, 4096), orc.codebook_init(32))
    assert abs(mse - e.mean()) < 1e-12


@pytest.fixture(scope="module")
def codebook_2048():
    return qamw.train_codebook(11, 1 << 20, seed=0, max_iters=200, tol=1e-7)


def test_trained_2048_point_codebook_satisfies_lloyd_conditions(orc, codebook_2048):
    """The benchmark codebook (K=2048, 2^20 samples, seed 0): nearest-neighbour and centroid
    conditions, checked with the oracle's brute-force assignment."""
    cb, mse, it = codebook_2048
    assert cb.shape == (2048, 2) and cb.dtype == np.float32 and 2 <= it <= 200
    assert cb.nbytes == 16384                                          # Sec. 3.5: at most 16 KB at B <= 11
    n = 1 << 18
    xy = orc.gauss_samples(0, n)                                       # a prefix of the training draw
    a, e = orc.assign(xy, cb.astype(np.float64), threads=8)
    assert abs(e.mean() / mse - 1.0) < 0.02
    G2 = 5 / (36 * np.sqrt(3))
    assert abs(mse / (2 * G2 * 8 * np.pi / 2048) - 1.0) < 0.25        # high-rate level for this source
    fresh = orc.gauss_samples(4242, n)
    a2, e2 = orc.assign(fresh, cb.astype(np.float64), threads=8)
    assert abs(e2.mean() / mse - 1.0) < 0.06                            # small cells over-fit a little
    cnt = np.bincount(a2, minlength=2048)
    big = cnt >= 30                       # the outermost cells of a sample-trained codebook hold a few draws each
    assert big.mean() > 0.8
    for ax in (0, 1):
        m = np.bincount(a2, weights=fresh[:, ax], minlength=2048)[big] / cnt[big]
        v = np.maximum(np.bincount(a2, weights=fresh[:, ax] ** 2, minlength=2048)[big] / cnt[big] - m ** 2, 1e-12)
        se = np.sqrt(v / cnt[big] + v / (4.0 * cnt[big]))              # fresh cell mean + training cell mean
        assert np.mean(np.abs(m - cb[big, ax]) < 4 * se) > 0.99
        assert np.all(np.abs(m - cb[big, ax]) < 8 * se + 1e-3)


def test_zador_slope_10_vs_11_bits(codebook_2048):
    cb10, mse10, _ = qamw.train_codebook(10, 1 << 20, seed=0, max_iters=200, tol=1e-7)
    assert abs(mse10 / codebook_2048[1] - 2.0) < 0.3


def test_trainer_is_deterministic_across_thread_counts(monkeypatch):
    monkeypatch.setenv("QAMW_NUM_THREADS", "1")
    a = qamw.train_codebook(6, 1 << 14, seed=9, max_iters=15, tol=0.0)
    monkeypatch.setenv("QAMW_NUM_THREADS", "7")
    b = qamw.train_codebook(6, 1 << 14, seed=9, max_iters=15, tol=0.0)
    assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2]
