"""ctypes front end of the QAM-W CPU oracle (oracle/qamw_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
CPU-baseline leg of the benchmark may import this module.  It never imports the
HIP library or its Python binding, and nothing here is used by them.

The arithmetic lives in the C file; this module only marshals numpy arrays.
`MODE_TRUTH` = all fp64 with the explicit Hadamard matrix, `MODE_SPEC` = the same
steps rounded to fp32 once each (see the header of the C file).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

MODE_TRUTH = 0
MODE_SPEC = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qamw_oracle.c")
_LIB = os.path.join(_HERE, "libqamw_oracle.so")

GCC_FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c99"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Rebuilds when the source is newer than the library."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", *GCC_FLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_bpw.restype = C.c_double
        _lib.orc_bpw.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        _lib.orc_paper_block_size.restype = C.c_int
        _lib.orc_packed_row_bytes.restype = C.c_int64
        _lib.orc_bf16_rne.restype = C.c_uint16
        _lib.orc_bf16_rne.argtypes = [C.c_float]
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int8)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------- helpers
def hadamard(b: int) -> np.ndarray:
    H = np.empty((b, b), dtype=np.int8)
    lib().orc_hadamard(C.c_int(b), _p(H, C.c_int8))
    return H


def paper_block_size(d_in: int) -> int:
    return int(lib().orc_paper_block_size(C.c_int(d_in)))


def bpw(d_in: int, d_out: int, bits: int, with_f16_scales: bool = False) -> float:
    return float(lib().orc_bpw(d_in, d_out, bits, int(with_f16_scales)))


def sign_mask(seed: int, d_in: int) -> np.ndarray:
    s = np.empty(d_in, dtype=np.int8)
    lib().orc_sign_mask(C.c_uint64(seed), C.c_int(d_in), _p(s, C.c_int8))
    return s


def gauss_samples(seed: int, n: int) -> np.ndarray:
    xy = np.empty((n, 2), dtype=np.float64)
    lib().orc_gauss_samples(C.c_uint64(seed), C.c_int64(n), _p(xy, C.c_double))
    return xy


def channel_scales(act_rms: np.ndarray, alpha: float) -> np.ndarray:
    a = _f32(act_rms)
    s = np.empty_like(a)
    lib().orc_channel_scales(_p(a, C.c_float), C.c_int(a.size), C.c_double(alpha), _p(s, C.c_float))
    return s


def bf16_rne(x: np.ndarray) -> np.ndarray:
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.uint16)
    f = lib().orc_bf16_rne
    flat, oflat = x.ravel(), out.ravel()
    for i in range(flat.size):
        oflat[i] = f(float(flat[i]))
    return out


def rotate_fwd_truth(v, block, signs=None):
    v = np.ascontiguousarray(v, dtype=np.float64)
    y = np.empty_like(v)
    sg = _i8(signs)
    lib().orc_rotate_fwd_truth(_p(v, C.c_double), C.c_int(v.size), C.c_int(block), _p(sg, C.c_int8),
                               _p(y, C.c_double))
    return y


def rotate_inv_truth(y, block, signs=None):
    y = np.ascontiguousarray(y, dtype=np.float64)
    u = np.empty_like(y)
    sg = _i8(signs)
    lib().orc_rotate_inv_truth(_p(y, C.c_double), C.c_int(y.size), C.c_int(block), _p(sg, C.c_int8),
                               _p(u, C.c_double))
    return u


def rotate_fwd_spec(u, block, signs=None):
    u = _f32(u)
    y = np.empty_like(u)
    sg = _i8(signs)
    lib().orc_rotate_fwd_spec(_p(u, C.c_float), C.c_int(u.size), C.c_int(block), _p(sg, C.c_int8),
                              _p(y, C.c_float))
    return y


def fwht_spec(t):
    t = np.array(t, dtype=np.float32, copy=True)
    lib().orc_fwht_spec(_p(t, C.c_float), C.c_int(t.size))
    return t


def packed_row_bytes(d_in: int, bits: int) -> int:
    return int(lib().orc_packed_row_bytes(C.c_int(d_in), C.c_int(bits)))


def pack(idx: np.ndarray, bits: int) -> np.ndarray:
    """idx [rows][P] int32 -> packed [rows][row_bytes] uint8."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows, P = idx.shape
    rb = packed_row_bytes(2 * P, bits)
    out = np.empty((rows, rb), dtype=np.uint8)
    for i in range(rows):
        lib().orc_pack_row(_p(idx[i], C.c_int32), C.c_int(P), C.c_int(bits), _p(out[i], C.c_uint8),
                           C.c_int64(rb))
    return out


def unpack(packed: np.ndarray, d_in: int, bits: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    P = d_in // 2
    out = np.empty((rows, P), dtype=np.int32)
    for i in range(rows):
        lib().orc_unpack_row(_p(packed[i], C.c_uint8), C.c_int(P), C.c_int(bits), _p(out[i], C.c_int32))
    return out


# --------------------------------------------------------------------------- codec
def _split(n_rows: int, threads: int):
    threads = max(1, min(threads, n_rows))
    edges = np.linspace(0, n_rows, threads + 1).astype(int)
    return [(int(edges[t]), int(edges[t + 1])) for t in range(threads) if edges[t] < edges[t + 1]]


def encode(W, codebook, bits, block, chan_scale=None, signs=None, pair_sigma=None, mode=MODE_SPEC,
           want_gaps=True, want_x=False, threads=1):
    """Encode every row of W (fp32 [d_out][d_in]).  Returns a dict with idx (int32 [d_out][P]),
    norms (fp64; in spec mode they are fp32 values), d1/d2 (two smallest squared distances) and
    optionally x (the normalised pairs).  `threads` only splits rows over independent calls."""
    W = _f32(W)
    d_out, d_in = W.shape
    P = d_in // 2
    cb = _f32(codebook)
    assert cb.shape == (1 << bits, 2)
    cs, sg, ps = _f32(chan_scale), _i8(signs), _f32(pair_sigma)
    idx = np.empty((d_out, P), dtype=np.int32)
    norms = np.empty(d_out, dtype=np.float64)
    d1 = np.empty((d_out, P), dtype=np.float64) if want_gaps else None
    d2 = np.empty((d_out, P), dtype=np.float64) if want_gaps else None
    x = np.empty((d_out, P, 2), dtype=np.float64) if want_x else None

    def run(rng):
        rc = lib().orc_encode_rows(_p(W, C.c_float), C.c_int64(d_in), C.c_int(rng[0]), C.c_int(rng[1]),
                                   C.c_int(d_in), _p(cs, C.c_float), _p(sg, C.c_int8), _p(ps, C.c_float),
                                   _p(cb, C.c_float), C.c_int(bits), C.c_int(block), C.c_int(mode),
                                   _p(idx, C.c_int32), _p(norms, C.c_double), _p(d1, C.c_double),
                                   _p(d2, C.c_double), _p(x, C.c_double))
        if rc != 0:
            raise ValueError("oracle encode: invalid arguments")

    parts = _split(d_out, threads)
    if len(parts) <= 1:
        for p in parts:
            run(p)
    else:
        with ThreadPoolExecutor(len(parts)) as ex:
            list(ex.map(run, parts))
    return {"idx": idx, "norms": norms, "d1": d1, "d2": d2, "x": x}


def decode(idx, norms, codebook, bits, block, chan_scale=None, signs=None, pair_sigma=None,
           mode=MODE_SPEC, want_yhat=False, threads=1):
    """Decode indices [d_out][P] with fp32 row norms.  Returns dict: w (fp64 view of the value
    before the bf16 cast), bf16 (uint16 bit patterns; spec mode only), yhat (optional)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    d_out, P = idx.shape
    d_in = 2 * P
    nr = _f32(norms)
    cb = _f32(codebook)
    cs, sg, ps = _f32(chan_scale), _i8(signs), _f32(pair_sigma)
    w = np.empty((d_out, d_in), dtype=np.float64)
    bf = np.empty((d_out, d_in), dtype=np.uint16) if mode == MODE_SPEC else None
    yh = np.empty((d_out, d_in), dtype=np.float64) if want_yhat else None

    def run(rng):
        rc = lib().orc_decode_rows(_p(idx, C.c_int32), C.c_int(rng[0]), C.c_int(rng[1]), C.c_int(d_in),
                                   _p(nr, C.c_float), _p(cs, C.c_float), _p(sg, C.c_int8),
                                   _p(ps, C.c_float), _p(cb, C.c_float), C.c_int(bits), C.c_int(block),
                                   C.c_int(mode), _p(w, C.c_double), _p(bf, C.c_uint16),
                                   _p(yh, C.c_double))
        if rc != 0:
            raise ValueError("oracle decode: invalid arguments")

    parts = _split(d_out, threads)
    if len(parts) <= 1:
        for p in parts:
            run(p)
    else:
        with ThreadPoolExecutor(len(parts)) as ex:
            list(ex.map(run, parts))
    return {"w": w, "bf16": bf, "yhat": yh}


def calibrate_sigma(W, block, chan_scale=None, signs=None, max_rows=1024, mode=MODE_SPEC):
    W = _f32(W)
    d_out, d_in = W.shape
    cs, sg = _f32(chan_scale), _i8(signs)
    out = np.empty(d_in // 2, dtype=np.float32)
    rc = lib().orc_calibrate_sigma(_p(W, C.c_float), C.c_int64(d_in), C.c_int(d_out), C.c_int(d_in),
                                   _p(cs, C.c_float), _p(sg, C.c_int8), C.c_int(block),
                                   C.c_int(max_rows), C.c_int(mode), _p(out, C.c_float))
    if rc != 0:
        raise ValueError("oracle calibrate_sigma: invalid arguments")
    return out


# --------------------------------------------------------------------------- codebook
def codebook_init(K: int) -> np.ndarray:
    cb = np.empty((K, 2), dtype=np.float64)
    lib().orc_codebook_init(C.c_int(K), _p(cb, C.c_double))
    return cb


def lloyd(samples, K, init=None, max_iters=200, tol=1e-7):
    """Plain Lloyd iterations.  Returns (codebook fp64 [K][2], mse, iterations)."""
    samples = np.ascontiguousarray(samples, dtype=np.float64)
    cb = codebook_init(K) if init is None else np.array(init, dtype=np.float64, copy=True)
    mse = C.c_double()
    iters = C.c_int()
    lib().orc_lloyd(_p(samples, C.c_double), C.c_int64(samples.shape[0]), C.c_int(K), _p(cb, C.c_double),
                    C.c_int(max_iters), C.c_double(tol), C.byref(mse), C.byref(iters))
    return cb, mse.value, iters.value


def assign(samples, codebook, threads=1):
    """Nearest codeword (fp64) of every sample: (assignment int32 [n], squared error [n])."""
    samples = np.ascontiguousarray(samples, dtype=np.float64)
    cb = np.ascontiguousarray(codebook, dtype=np.float64)
    n = samples.shape[0]
    a = np.empty(n, dtype=np.int32)
    e = np.empty(n, dtype=np.float64)

    def run(rng):
        lo, hi = rng
        lib().orc_assign(_p(samples[lo:hi], C.c_double), C.c_int64(hi - lo), _p(cb, C.c_double),
                         C.c_int(cb.shape[0]), _p(a[lo:hi], C.c_int32), _p(e[lo:hi], C.c_double))

    parts = _split(n, threads)
    if len(parts) <= 1:
        for p in parts:
            run(p)
    else:
        with ThreadPoolExecutor(len(parts)) as ex:
            list(ex.map(run, parts))
    return a, e


# ------------------------------------------------------------------------------ polar baseline
def rayleigh_lloyd_max(Na: int, rmax: float = 8.0, max_iters: int = 400000, tol: float = 1e-14):
    """Lloyd-Max levels of the unit Rayleigh density (Sec. 3 'Polar Baseline'), fp64; returns
    (levels, C_LM, iterations)."""
    levels = np.zeros(Na, dtype=np.float64)
    c = C.c_double()
    L = lib()
    L.orc_rayleigh_lloyd_max.restype = C.c_int
    it = L.orc_rayleigh_lloyd_max(C.c_int(Na), C.c_double(rmax), C.c_int(max_iters), C.c_double(tol),
                                  _p(levels, C.c_double), C.byref(c))
    return levels, float(c.value), int(it)


def rayleigh_distortion(levels) -> float:
    lv = np.ascontiguousarray(levels, dtype=np.float64)
    L = lib()
    L.orc_rayleigh_distortion.restype = C.c_double
    return float(L.orc_rayleigh_distortion(_p(lv, C.c_double), C.c_int(lv.size)))


def polar_table(levels, Np: int) -> np.ndarray:
    lv = _f32(levels)
    out = np.zeros((lv.size * Np, 2), dtype=np.float32)
    lib().orc_polar_table(_p(lv, C.c_float), C.c_int(lv.size), C.c_int(Np), _p(out, C.c_float))
    return out


def polar_quantize(x, levels, Np: int):
    """x: (..., 2) points.  Returns dict(idx, amp_margin, phase_margin) shaped like x[..., 0]."""
    xs = np.ascontiguousarray(x, dtype=np.float64)
    shape = xs.shape[:-1]
    n = int(np.prod(shape)) if shape else 1
    lv = _f32(levels)
    idx = np.zeros(n, dtype=np.int32)
    am = np.zeros(n, dtype=np.float64)
    pm = np.zeros(n, dtype=np.float64)
    lib().orc_polar_quantize(_p(xs, C.c_double), C.c_int64(n), _p(lv, C.c_float), C.c_int(lv.size), C.c_int(Np),
                             _p(idx, C.c_int32), _p(am, C.c_double), _p(pm, C.c_double))
    return dict(idx=idx.reshape(shape), amp_margin=am.reshape(shape), phase_margin=pm.reshape(shape))


def encode_polar(W, levels, bits_p, block, chan_scale=None, signs=None, pair_sigma=None, mode=MODE_SPEC, threads=1):
    """The encoder with the polar quantiser in place of the joint codebook: the same front half
    (channel scale, row norm, rotation, pair gain), then amplitude level and phase bin per pair.
    Index = amplitude_index * 2^bits_p + phase_index."""
    dummy = np.array([[0.0, 0.0], [1.0, 1.0]], dtype=np.float32)          # the front half does not depend on it
    front = encode(W, dummy, 1, block, chan_scale=chan_scale, signs=signs, pair_sigma=pair_sigma, mode=mode,
                   want_gaps=False, want_x=True, threads=threads)
    q = polar_quantize(front["x"], levels, 1 << bits_p)
    q["norms"] = front["norms"]
    q["x"] = front["x"]
    return q
