"""Thin ctypes binding of libqamw (include/qamw.h).  Argument marshalling only: every step of
the codec runs in the library's HIP kernels.  torch is used for device memory and streams.

There is no CPU fallback: importing works without a GPU (host helpers run anywhere), but the
device entry points raise if the library is missing or HIP reports an error.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_UNSUPPORTED, ERR_DEVICE = 0, 1, 2, 3, 4
DTYPE_F32, DTYPE_BF16 = 0, 1

EXPORTS = [
    "qamw_status_string", "qamw_packed_row_bytes", "qamw_paper_block_size", "qamw_bpw", "qamw_sign_mask",
    "qamw_channel_scales", "qamw_train_codebook", "qamw_calibrate_workspace_bytes", "qamw_calibrate_sigma", "qamw_encode", "qamw_decode",
    "qamw_decode_f32", "qamw_decode_batch", "qamw_set_kernel_path", "qamw_polar_codebook", "qamw_encode_polar",
    "qamw_matmul_workspace_bytes", "qamw_matmul", "qamw_matmul_batch", "qamw_encode_stats",
    "qamw_normalised_pairs", "qamw_lloyd_workspace_bytes", "qamw_lloyd_device",
    "qamw_search_grid_size", "qamw_search_grid_build", "qamw_encode_pruned", "qamw_calibrate_sigma_static", "qamw_decode_traffic_probe", "qamw_encode_batch", "qamw_calibrate_sigma_batch",
]


MAX_BATCH = 32


class MatmulItem(C.Structure):
    """qamw_matmul_item of include/qamw.h."""
    _fields_ = [("X", C.c_void_p), ("ldx", C.c_int64), ("packed", C.c_void_p), ("row_norms", C.c_void_p),
                ("chan_scale", C.c_void_p), ("signs", C.c_void_p), ("pair_sigma", C.c_void_p), ("Y", C.c_void_p),
                ("ldy", C.c_int64), ("d_out", C.c_int32), ("d_in", C.c_int32)]


class CalibrateItem(C.Structure):
    """qamw_calibrate_item of include/qamw.h."""
    _fields_ = [("W", C.c_void_p), ("ldw", C.c_int64), ("chan_scale", C.c_void_p), ("signs", C.c_void_p),
                ("sigma_out", C.c_void_p), ("d_out", C.c_int32), ("d_in", C.c_int32)]


class EncodeItem(C.Structure):
    """qamw_encode_item of include/qamw.h."""
    _fields_ = [("W", C.c_void_p), ("ldw", C.c_int64), ("chan_scale", C.c_void_p), ("signs", C.c_void_p),
                ("pair_sigma", C.c_void_p), ("packed_out", C.c_void_p), ("row_norms_out", C.c_void_p),
                ("d_out", C.c_int32), ("d_in", C.c_int32)]


class DecodeItem(C.Structure):
    """qamw_decode_item of include/qamw.h."""
    _fields_ = [("packed", C.c_void_p), ("row_norms", C.c_void_p), ("chan_scale", C.c_void_p), ("signs", C.c_void_p),
                ("pair_sigma", C.c_void_p), ("W_out", C.c_void_p), ("ldo", C.c_int64), ("d_out", C.c_int32),
                ("d_in", C.c_int32)]


class QamwError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Load libqamw.so (built in-tree).  Builds it only when no library exists at all."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime; it must be the one already loaded when libqamw's
        # dependency on libamdhip64 is resolved, or the two would not share streams and memory.
        import torch  # noqa: F401

        if not os.path.exists(_build.LIB):
            _build.build(verbose=False)
        L = C.CDLL(_build.LIB)
        L.qamw_status_string.restype = C.c_char_p
        L.qamw_status_string.argtypes = [C.c_int]
        vp, i32, i64, u64 = C.c_void_p, C.c_int, C.c_int64, C.c_uint64
        L.qamw_packed_row_bytes.argtypes = [i32, i32, C.POINTER(C.c_size_t)]
        L.qamw_paper_block_size.argtypes = [i32, C.POINTER(i32)]
        L.qamw_bpw.argtypes = [i32, i32, i32, i32, C.POINTER(C.c_double)]
        L.qamw_sign_mask.argtypes = [u64, i32, vp]
        L.qamw_channel_scales.argtypes = [vp, i32, C.c_float, vp]
        L.qamw_train_codebook.argtypes = [i32, u64, u64, i32, C.c_double, vp, C.POINTER(C.c_double), C.POINTER(i32)]
        L.qamw_calibrate_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(C.c_size_t)]
        L.qamw_calibrate_sigma.argtypes = [vp, i32, i32, i32, i64, vp, vp, i32, i32, vp, C.c_size_t, vp, vp]
        L.qamw_calibrate_sigma_static.argtypes = [vp, i32, i32, i32, i64, vp, vp, i32, i32, vp, vp]
        L.qamw_encode.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.qamw_encode_stats.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.qamw_decode.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, i64, vp]
        L.qamw_decode_f32.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, i64, vp]
        L.qamw_decode_batch.argtypes = [C.POINTER(DecodeItem), i32, vp, i32, i32, vp]
        L.qamw_decode_traffic_probe.argtypes = [C.POINTER(DecodeItem), i32, vp, i32, i32, vp]
        L.qamw_encode_batch.argtypes = [C.POINTER(EncodeItem), i32, i32, vp, i32, i32, vp]
        L.qamw_calibrate_sigma_batch.argtypes = [C.POINTER(CalibrateItem), i32, i32, i32, i32, vp, C.c_size_t, vp]
        L.qamw_set_kernel_path.argtypes = [i32]
        L.qamw_matmul_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(C.c_size_t)]
        L.qamw_matmul.argtypes = [vp, i32, i32, i64, vp, vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, C.c_size_t, vp, i64, vp]
        L.qamw_matmul_batch.argtypes = [C.POINTER(MatmulItem), i32, i32, i32, vp, i32, i32, vp, C.c_size_t, vp]
        L.qamw_normalised_pairs.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp, i32, vp, vp, vp]
        L.qamw_lloyd_workspace_bytes.argtypes = [i32, C.POINTER(C.c_size_t)]
        L.qamw_lloyd_device.argtypes = [vp, u64, i32, vp, i32, C.c_double, vp, C.c_size_t, C.POINTER(C.c_double), C.POINTER(i32), vp]
        L.qamw_polar_codebook.argtypes = [i32, i32, vp, vp, C.POINTER(C.c_double)]
        L.qamw_encode_polar.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp]
        L.qamw_search_grid_size.argtypes = [i32, C.POINTER(i32), C.POINTER(C.c_size_t)]
        L.qamw_search_grid_build.argtypes = [vp, i32, vp, C.c_size_t, C.POINTER(i32), C.POINTER(u64)]
        L.qamw_encode_pruned.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
        for name in EXPORTS:
            if name != "qamw_status_string":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().qamw_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise QamwError(status, where)


# ------------------------------------------------------------------------------ host helpers
def packed_row_bytes(d_in: int, bits: int) -> int:
    out = C.c_size_t()
    _check(lib().qamw_packed_row_bytes(d_in, bits, C.byref(out)), "qamw_packed_row_bytes")
    return int(out.value)


def paper_block_size(d_in: int) -> int:
    out = C.c_int()
    _check(lib().qamw_paper_block_size(d_in, C.byref(out)), "qamw_paper_block_size")
    return int(out.value)


def bpw(d_in: int, d_out: int, bits: int, with_f16_scales: bool = False) -> float:
    out = C.c_double()
    _check(lib().qamw_bpw(d_in, d_out, bits, int(with_f16_scales), C.byref(out)), "qamw_bpw")
    return float(out.value)


def sign_mask(seed: int, d_in: int) -> np.ndarray:
    out = np.empty(max(d_in, 0), dtype=np.int8)
    _check(lib().qamw_sign_mask(seed & (2**64 - 1), d_in, out.ctypes.data), "qamw_sign_mask")
    return out


def channel_scales(act_rms: np.ndarray, alpha: float) -> np.ndarray:
    a = np.ascontiguousarray(act_rms, dtype=np.float32)
    out = np.empty_like(a)
    _check(lib().qamw_channel_scales(a.ctypes.data, a.size, alpha, out.ctypes.data), "qamw_channel_scales")
    return out


def train_codebook(bits: int, n_samples: int = 1 << 20, seed: int = 0, max_iters: int = 200, tol: float = 1e-7):
    """Returns (codebook float32 [2^bits][2], mse, iterations)."""
    out = np.empty((1 << max(bits, 0) if 1 <= bits <= 12 else 1, 2), dtype=np.float32)
    mse, it = C.c_double(), C.c_int()
    _check(lib().qamw_train_codebook(bits, n_samples, seed & (2**64 - 1), max_iters, tol, out.ctypes.data,
                                     C.byref(mse), C.byref(it)), "qamw_train_codebook")
    return out, float(mse.value), int(it.value)


def normalised_pairs(W, block: int, chan_scale=None, signs=None, pair_sigma=None, stream=None):
    """The points the encoder quantises: (pairs float32 [d_out][d_in/2][2], row_norms float32 [d_out])."""
    import torch

    _require_cuda(W, chan_scale, signs, pair_sigma)
    if W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be 2-D with unit column stride")
    d_out, d_in = W.shape
    pairs = torch.empty((d_out, d_in // 2, 2), dtype=torch.float32, device=W.device)
    norms = torch.empty(d_out, dtype=torch.float32, device=W.device)
    _check(lib().qamw_normalised_pairs(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                       _ptr(pair_sigma), block, _ptr(pairs), _ptr(norms), _stream(stream)),
           "qamw_normalised_pairs")
    return pairs, norms


def lloyd_device(samples, init_codebook, bits: int, max_iters: int = 200, tol: float = 1e-7, stream=None):
    """Lloyd iterations on the device over samples (CUDA float32 [n][2]) from init_codebook ([2^bits][2]).
    Returns (codebook CUDA float32 [2^bits][2], mse, iterations).  Blocks until done."""
    import torch

    _require_cuda(samples, init_codebook)
    samples = samples.contiguous()
    cb = init_codebook.to(torch.float32).contiguous().clone()
    need = C.c_size_t()
    _check(lib().qamw_lloyd_workspace_bytes(bits, C.byref(need)), "qamw_lloyd_workspace_bytes")
    ws = torch.empty(need.value, dtype=torch.uint8, device=samples.device)
    mse, it = C.c_double(), C.c_int()
    _check(lib().qamw_lloyd_device(_ptr(samples), samples.shape[0], bits, _ptr(cb), max_iters, tol, _ptr(ws), need.value,
                                   C.byref(mse), C.byref(it), _stream(stream)), "qamw_lloyd_device")
    return cb, float(mse.value), int(it.value)


def polar_codebook(bits_a: int, bits_p: int):
    """Rayleigh Lloyd-Max amplitude levels and the lookup table of the polar baseline.
    Returns (levels float32 [2^bits_a], table float32 [2^(bits_a+bits_p)][2], C_LM)."""
    ok = 0 <= bits_a <= 6 and 0 <= bits_p <= 12 and 1 <= bits_a + bits_p <= 12
    levels = np.empty(1 << bits_a if ok else 1, dtype=np.float32)
    table = np.empty((1 << (bits_a + bits_p) if ok else 1, 2), dtype=np.float32)
    c_lm = C.c_double()
    _check(lib().qamw_polar_codebook(bits_a, bits_p, levels.ctypes.data_as(C.c_void_p), table.ctypes.data_as(C.c_void_p),
                                     C.byref(c_lm)), "qamw_polar_codebook")
    return levels, table, float(c_lm.value)


def set_kernel_path(path: int) -> int:
    return int(lib().qamw_set_kernel_path(path))


# ------------------------------------------------------------------------------ device entry points
def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dtype_code(W):
    import torch

    if W.dtype == torch.float32:
        return DTYPE_F32
    if W.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"W must be float32 or bfloat16, got {W.dtype}")


def _require_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("device entry points take CUDA (HIP) tensors")


def calibrate_workspace_bytes(d_in: int, d_out: int, max_rows: int = 1024) -> int:
    out = C.c_size_t()
    _check(lib().qamw_calibrate_workspace_bytes(d_in, d_out, max_rows, C.byref(out)), "qamw_calibrate_workspace_bytes")
    return int(out.value)


def calibrate_sigma(W, block: int, chan_scale=None, signs=None, max_rows: int = 1024, workspace=None, out=None,
                    stream=None):
    """Eq. 1 pair scales of matrix W (torch CUDA tensor [d_out][d_in]).  Returns float32 [d_in/2].
    `workspace` is a uint8 CUDA tensor of at least calibrate_workspace_bytes(); allocated if absent."""
    import torch

    _require_cuda(W, chan_scale, signs, workspace, out)
    d_out, d_in = W.shape
    if workspace is None:
        workspace = torch.empty(calibrate_workspace_bytes(d_in, d_out, max_rows), dtype=torch.uint8, device=W.device)
    if out is None:
        out = torch.empty(d_in // 2, dtype=torch.float32, device=W.device)
    _check(lib().qamw_calibrate_sigma(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                      block, max_rows, _ptr(workspace), workspace.numel(), _ptr(out), _stream(stream)),
           "qamw_calibrate_sigma")
    return out


STATIC_SCRATCH_BYTES = 8 * 1024 * 1024 + 4096


def calibrate_sigma_static(W, block: int, out, chan_scale=None, signs=None, max_rows: int = 1024, stream=None):
    """qamw_calibrate_sigma_static: the pair scales written into `out` (float32 CUDA [d_in/2]) with the library's own
    static scratch; this wrapper allocates nothing either."""
    _require_cuda(W, chan_scale, signs, out)
    d_out, d_in = W.shape
    _check(lib().qamw_calibrate_sigma_static(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                             block, max_rows, _ptr(out), _stream(stream)), "qamw_calibrate_sigma_static")
    return out


def encode(W, codebook, bits: int, block: int, chan_scale=None, signs=None, pair_sigma=None, out=None, stream=None,
           full_scans=None):
    """Encode W (torch CUDA tensor, fp32 or bf16, row-major, stride(1) == 1).
    Returns (packed uint8 [d_out][row_bytes], row_norms float32 [d_out]).  full_scans: optional int64 CUDA tensor of
    one element to which the number of pairs decided by the whole-codebook scan is added."""
    import torch

    _require_cuda(W, codebook, chan_scale, signs, pair_sigma)
    if W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be 2-D with unit column stride")
    d_out, d_in = W.shape
    rb = packed_row_bytes(d_in, bits)
    if out is None:
        packed = torch.empty((d_out, rb), dtype=torch.uint8, device=W.device)
        norms = torch.empty(d_out, dtype=torch.float32, device=W.device)
    else:
        packed, norms = out
    if full_scans is not None:
        _require_cuda(full_scans)
        _check(lib().qamw_encode_stats(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                       _ptr(pair_sigma), _ptr(codebook), bits, block, _ptr(packed), _ptr(norms),
                                       _ptr(full_scans), _stream(stream)), "qamw_encode_stats")
        return packed, norms
    _check(lib().qamw_encode(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                             _ptr(pair_sigma), _ptr(codebook), bits, block, _ptr(packed), _ptr(norms),
                             _stream(stream)), "qamw_encode")
    return packed, norms


def search_grid_size(bits: int):
    """(cells per side G, table bytes) of the pruned-search grid for 2^bits codewords."""
    g, n = C.c_int(), C.c_size_t()
    _check(lib().qamw_search_grid_size(bits, C.byref(g), C.byref(n)), "qamw_search_grid_size")
    return int(g.value), int(n.value)


def search_grid(codebook, bits: int):
    """Build the pruned-search table of a codebook (host array [2^bits][2] float32).
    Returns (table uint8 [bytes], longest candidate list, number of cells with more than 8 candidates)."""
    cb = np.ascontiguousarray(codebook, dtype=np.float32).reshape(-1)
    if cb.size != 2 << bits:
        raise ValueError("codebook must hold 2^bits pairs")
    _, n = search_grid_size(bits)
    table = np.zeros(n, dtype=np.uint8)
    mx, over = C.c_int(), C.c_uint64()
    _check(lib().qamw_search_grid_build(cb.ctypes.data, bits, table.ctypes.data, C.c_size_t(n), C.byref(mx), C.byref(over)),
           "qamw_search_grid_build")
    return table, int(mx.value), int(over.value)


def encode_pruned(W, codebook, grid, bits: int, block: int, chan_scale=None, signs=None, pair_sigma=None, out=None,
                  stream=None, full_scans=None):
    """qamw_encode with the pruned search: grid is the table of search_grid() as a CUDA uint8 tensor.
    Returns (packed uint8 [d_out][row_bytes], row_norms float32 [d_out])."""
    import torch

    _require_cuda(W, codebook, grid, chan_scale, signs, pair_sigma, full_scans)
    if W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be 2-D with unit column stride")
    if grid.numel() * grid.element_size() < search_grid_size(bits)[1]:
        raise ValueError("grid table too small for these bits")
    d_out, d_in = W.shape
    rb = packed_row_bytes(d_in, bits)
    if out is None:
        packed = torch.empty((d_out, rb), dtype=torch.uint8, device=W.device)
        norms = torch.empty(d_out, dtype=torch.float32, device=W.device)
    else:
        packed, norms = out
    _check(lib().qamw_encode_pruned(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                    _ptr(pair_sigma), _ptr(codebook), bits, block, _ptr(grid), _ptr(packed), _ptr(norms),
                                    _ptr(full_scans), _stream(stream)), "qamw_encode_pruned")
    return packed, norms


def encode_polar(W, levels, bits_a: int, bits_p: int, block: int, chan_scale=None, signs=None, pair_sigma=None, out=None,
                 stream=None):
    """Polar-baseline encode of W: index = amplitude level * 2^bits_p + phase bin, bits_a + bits_p bits per pair.
    Returns (packed uint8 [d_out][row_bytes], row_norms float32 [d_out])."""
    import torch

    _require_cuda(W, levels, chan_scale, signs, pair_sigma)
    if W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be 2-D with unit column stride")
    d_out, d_in = W.shape
    rb = packed_row_bytes(d_in, bits_a + bits_p)
    if out is None:
        packed = torch.empty((d_out, rb), dtype=torch.uint8, device=W.device)
        norms = torch.empty(d_out, dtype=torch.float32, device=W.device)
    else:
        packed, norms = out
    _check(lib().qamw_encode_polar(_ptr(W), _dtype_code(W), d_out, d_in, W.stride(0), _ptr(chan_scale), _ptr(signs),
                                   _ptr(pair_sigma), _ptr(levels), bits_a, bits_p, block, _ptr(packed), _ptr(norms),
                                   _stream(stream)), "qamw_encode_polar")
    return packed, norms


def decode(packed, row_norms, d_in: int, codebook, bits: int, block: int, chan_scale=None, signs=None,
           pair_sigma=None, out=None, f32: bool = False, stream=None):
    """Decode to bf16 [d_out][d_in] (or the fp32 value before the cast when f32=True)."""
    import torch

    _require_cuda(packed, row_norms, codebook, chan_scale, signs, pair_sigma)
    d_out = row_norms.shape[0]
    if out is None:
        out = torch.empty((d_out, d_in), dtype=torch.float32 if f32 else torch.bfloat16, device=packed.device)
    fn = lib().qamw_decode_f32 if f32 else lib().qamw_decode
    _check(fn(_ptr(packed), _ptr(row_norms), d_out, d_in, _ptr(chan_scale), _ptr(signs), _ptr(pair_sigma),
              _ptr(codebook), bits, block, _ptr(out), out.stride(0), _stream(stream)),
           "qamw_decode_f32" if f32 else "qamw_decode")
    return out


MATMUL_MAX_ROWS = 4096
MATMUL_TILE_ROWS = 64
MATMUL_VECTOR_ROWS = 8


def matmul_workspace_bytes(d_in: int, d_out: int, m: int) -> int:
    out = C.c_size_t()
    _check(lib().qamw_matmul_workspace_bytes(d_in, d_out, m, C.byref(out)), "qamw_matmul_workspace_bytes")
    return int(out.value)


def matmul(X, packed, row_norms, codebook, bits: int, block: int, chan_scale=None, signs=None, pair_sigma=None,
           workspace=None, out=None, stream=None):
    """Y = X W^T (fp32 [m][d_out]) for m <= 4096 rows of X (fp32 or bf16 [m][d_in]) against the packed matrix.
    Up to 8 rows: fp32 arithmetic throughout; more: bf16 operands on the matrix cores, fp32 accumulation, in tiles of at
    most 64 activation rows."""
    import torch

    _require_cuda(X, packed, row_norms, codebook, chan_scale, signs, pair_sigma)
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be 2-D with unit column stride")
    m, d_in = X.shape
    d_out = row_norms.shape[0]
    if workspace is None:
        workspace = torch.empty(matmul_workspace_bytes(d_in, d_out, m), dtype=torch.uint8, device=X.device)
    if out is None:
        out = torch.empty((m, d_out), dtype=torch.float32, device=X.device)
    _check(lib().qamw_matmul(_ptr(X), _dtype_code(X), m, X.stride(0), _ptr(packed), _ptr(row_norms), d_out, d_in,
                             _ptr(chan_scale), _ptr(signs), _ptr(pair_sigma), _ptr(codebook), bits, block,
                             _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out), out.stride(0),
                             _stream(stream)), "qamw_matmul")
    return out


def make_matmul_items(entries):
    """Host descriptor array for matmul_batch: each entry = (X, packed, row_norms, chan_scale, signs, pair_sigma, Y).
    Returns (array, keepalive, m, x dtype code, workspace bytes)."""
    arr = (MatmulItem * len(entries))()
    need, m, code = 0, None, None
    for i, (X, packed, norms, s, sg, sigma, Y) in enumerate(entries):
        _require_cuda(X, packed, norms, s, sg, sigma, Y)
        if X.dim() != 2 or X.stride(1) != 1 or Y.stride(1) != 1:
            raise ValueError("X and Y must be 2-D with unit column stride")
        if m is None:
            m, code = X.shape[0], _dtype_code(X)
        if X.shape[0] != m or _dtype_code(X) != code:
            raise ValueError("all items of a batch share the number of rows and the element type of X")
        d_in, d_out = X.shape[1], norms.shape[0]
        arr[i] = MatmulItem(X.data_ptr(), X.stride(0), packed.data_ptr(), norms.data_ptr(), None if s is None else s.data_ptr(),
                            None if sg is None else sg.data_ptr(), None if sigma is None else sigma.data_ptr(), Y.data_ptr(),
                            Y.stride(0), d_out, d_in)
        need += matmul_workspace_bytes(d_in, d_out, m)
    return arr, list(entries), m, code, need


def matmul_batch(items, codebook, bits: int, block: int, workspace, stream=None):
    arr, _keep, m, code, need = items
    _check(lib().qamw_matmul_batch(arr, len(arr), code, m, _ptr(codebook), bits, block, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "qamw_matmul_batch")


def make_decode_items(entries):
    """Build the host descriptor array for decode_batch from dicts/tuples of torch tensors:
    each entry = (packed, row_norms, d_in, chan_scale, signs, pair_sigma, out).  Returns (array, keepalive)."""
    arr = (DecodeItem * len(entries))()
    for i, (packed, norms, d_in, s, sg, sigma, out) in enumerate(entries):
        _require_cuda(packed, norms, s, sg, sigma, out)
        arr[i] = DecodeItem(packed.data_ptr(), norms.data_ptr(), None if s is None else s.data_ptr(),
                            None if sg is None else sg.data_ptr(), None if sigma is None else sigma.data_ptr(),
                            out.data_ptr(), out.stride(0), norms.shape[0], d_in)
    return arr, list(entries)


def decode_batch(items, codebook, bits: int, block: int, stream=None):
    """Decode up to MAX_BATCH matrices (a DecodeItem array from make_decode_items) in one launch."""
    arr = items[0] if isinstance(items, tuple) else items
    _check(lib().qamw_decode_batch(arr, len(arr), _ptr(codebook), bits, block, _stream(stream)), "qamw_decode_batch")


def decode_traffic_probe(items, codebook, bits: int, block: int, stream=None):
    """The loads and stores of decode_batch(items, ...) without the arithmetic: a measurement of the memory system.
    Every item's output is overwritten with meaningless values."""
    arr = items[0] if isinstance(items, tuple) else items
    _check(lib().qamw_decode_traffic_probe(arr, len(arr), _ptr(codebook), bits, block, _stream(stream)),
           "qamw_decode_traffic_probe")


def make_encode_items(entries):
    """Host descriptor array for encode_batch: each entry = (W, chan_scale, signs, pair_sigma, packed_out, row_norms_out).
    Returns (array, keepalive, dtype code)."""
    arr = (EncodeItem * len(entries))()
    code = None
    for i, (W, s, sg, sigma, packed, norms) in enumerate(entries):
        _require_cuda(W, s, sg, sigma, packed, norms)
        if W.dim() != 2 or W.stride(1) != 1:
            raise ValueError("W must be 2-D with unit column stride")
        if code is None:
            code = _dtype_code(W)
        if _dtype_code(W) != code:
            raise ValueError("all matrices of a batch share the element type")
        arr[i] = EncodeItem(W.data_ptr(), W.stride(0), None if s is None else s.data_ptr(), None if sg is None else sg.data_ptr(),
                            None if sigma is None else sigma.data_ptr(), packed.data_ptr(), norms.data_ptr(), W.shape[0], W.shape[1])
    return arr, list(entries), code


def encode_batch(items, codebook, bits: int, block: int, stream=None):
    """Encode up to MAX_BATCH matrices (an EncodeItem array from make_encode_items) in one launch."""
    arr, _keep, code = items
    _check(lib().qamw_encode_batch(arr, len(arr), code, _ptr(codebook), bits, block, _stream(stream)), "qamw_encode_batch")


def make_calibrate_items(entries, max_rows: int = 1024):
    """Host descriptor array for calibrate_sigma_batch: each entry = (W, chan_scale, signs, sigma_out).
    Returns (array, keepalive, dtype code, workspace bytes, max_rows)."""
    arr = (CalibrateItem * len(entries))()
    code, need = None, 0
    for i, (W, s, sg, sigma) in enumerate(entries):
        _require_cuda(W, s, sg, sigma)
        if W.dim() != 2 or W.stride(1) != 1:
            raise ValueError("W must be 2-D with unit column stride")
        if code is None:
            code = _dtype_code(W)
        if _dtype_code(W) != code:
            raise ValueError("all matrices of a batch share the element type")
        arr[i] = CalibrateItem(W.data_ptr(), W.stride(0), None if s is None else s.data_ptr(), None if sg is None else sg.data_ptr(),
                               sigma.data_ptr(), W.shape[0], W.shape[1])
        need += (calibrate_workspace_bytes(W.shape[1], W.shape[0], max_rows) + 255) // 256 * 256
    return arr, list(entries), code, need, max_rows


def calibrate_sigma_batch(items, block: int, workspace, stream=None):
    """Pair scales of up to MAX_BATCH matrices (a CalibrateItem array from make_calibrate_items) in two launches."""
    arr, _keep, code, need, max_rows = items
    _check(lib().qamw_calibrate_sigma_batch(arr, len(arr), code, block, max_rows, _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)),
           "qamw_calibrate_sigma_batch")
