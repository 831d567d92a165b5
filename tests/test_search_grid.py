"""CPU-side checks of the pruned-search table (qamw_search_grid_build): its layout, and that for every point
the codeword a whole-codebook search returns is among the candidates of the point's cell.  The search itself
is checked here by brute force in numpy, in the arithmetic the kernels use (fp32 differences, squares and one
fused multiply-add) and in fp64."""
import ctypes as C

import numpy as np
import pytest

from paper_2605_26339_amd import qamw


def parse(table):
    hdr = table[:32].view(np.uint32)
    G = int(hdr[2])
    assert hdr[0] == 0x44524751 and hdr[3] == 8 and hdr[6] == 0 and hdr[7] == 0
    inv_h = float(table[16:20].view(np.float32)[0])
    R = float(table[20:24].view(np.float32)[0])
    cells = table[32:].view(np.uint16).reshape(G, G, 8)
    return int(hdr[1]), G, inv_h, R, cells


def cell_of(x, inv_h, G):
    """floor(fma(x, inv_h, G/2)) in fp32: the product of two fp32 is exact in fp64; one rounding to fp32 follows."""
    t = (x.astype(np.float64) * np.float64(np.float32(inv_h)) + 0.5 * G).astype(np.float32)
    return np.floor(t).astype(np.int64)


def dist_fp32(x, c):
    """fma(e1, e1, e0 * e0) with e = fl32(x - c): x [n][1][2] against c [.][m][2].  The square of an fp32 is exact
    in fp64, so the fused multiply-add is one fp64 sum rounded to fp32."""
    e0 = (x[..., 0] - c[..., 0]).astype(np.float32)
    e1 = (x[..., 1] - c[..., 1]).astype(np.float32)
    return (e1.astype(np.float64) ** 2 + (e0 * e0).astype(np.float32).astype(np.float64)).astype(np.float32)


def nearest_fp32(x, cb, chunk=4096):
    """Whole-codebook argmin in the kernels' arithmetic, lowest index on ties."""
    return np.concatenate([dist_fp32(x[i:i + chunk, None, :], cb[None, :, :]).argmin(axis=1) for i in range(0, len(x), chunk)])


def nearest_fp64(x, cb, chunk=4096):
    out = []
    for i in range(0, len(x), chunk):
        d = ((x[i:i + chunk, None, :].astype(np.float64) - cb[None, :, :].astype(np.float64)) ** 2).sum(axis=2)
        out.append(d.argmin(axis=1))
    return np.concatenate(out)


def points_for(cb, inv_h, G, R, rng, n):
    h = 1.0 / inv_h
    gauss = rng.standard_normal((n, 2)).astype(np.float32)
    wide = (rng.standard_normal((n // 4, 2)) * 2.5).astype(np.float32)            # many near and beyond the border
    near = (cb[rng.integers(0, len(cb), n // 2)] + rng.standard_normal((n // 2, 2)) * 0.02).astype(np.float32)
    # points on and next to cell boundaries
    k = rng.integers(-G // 2, G // 2 + 1, (n // 2, 2)).astype(np.float64)
    edge = (k * h).astype(np.float32)
    edge_lo = np.nextafter(edge, np.float32(-np.inf))
    edge_hi = np.nextafter(edge, np.float32(np.inf))
    mixed = np.stack([edge[:, 0], gauss[: n // 2, 1]], axis=1)
    # midpoints between neighbouring codewords: the points where two distances tie
    i = rng.integers(0, len(cb), min(n // 2, 4096))
    dd = ((cb[i][:, None, :].astype(np.float64) - cb[None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    dd[np.arange(len(i)), i] = np.inf
    j = dd.argmin(axis=1)                                                         # the nearest other codeword
    mid = (0.5 * (cb[i].astype(np.float64) + cb[j].astype(np.float64))).astype(np.float32)
    return np.concatenate([gauss, wide, near, edge, edge_lo, edge_hi, mixed, mid]).astype(np.float32)


@pytest.mark.parametrize("bits", [11, 7, 3, 1])
def test_every_whole_codebook_winner_is_a_candidate_of_its_cell(bits):
    cb, _, _ = qamw.train_codebook(bits, 1 << 17, 5, 40, 1e-7)
    table, longest, overflow = qamw.search_grid(cb, bits)
    b, G, inv_h, R, cells = parse(table)
    assert b == bits and (G, len(table)) == qamw.search_grid_size(bits) and G == 1 << ((bits + 6) // 2)
    assert abs(R - 1.25 * np.abs(cb).max()) <= 1e-6 * R and abs(inv_h * 2 * R - G) <= 1e-5 * G
    K = 1 << bits
    # layout: ascending, padded with the first entry, or the overflow mark in the last slot
    over = cells[:, :, 7] == 0xFFFF
    assert int(over.sum()) == overflow
    body = cells.astype(np.int64)
    assert (body[~over] < K).all() and (body[over][:, :7] < K).all()
    full = body[~over].reshape(-1, 8)
    n_listed = 1 + (full[:, 1:] != full[:, :1]).sum(axis=1)                     # a list is padded with its first entry
    for rec, n in zip(full[:: max(1, len(full) // 4096)], n_listed[:: max(1, len(full) // 4096)]):
        assert (np.diff(rec[:n]) > 0).all() and (rec[n:] == rec[0]).all()
    assert (np.diff(body[over][:, :7], axis=1) > 0).all()
    assert longest == int(n_listed.max()) if overflow == 0 else longest > 8

    rng = np.random.default_rng(100 + bits)
    x = points_for(cb, inv_h, G, R, rng, 20000 if bits >= 7 else 4000)
    ix, iy = cell_of(x[:, 0], inv_h, G), cell_of(x[:, 1], inv_h, G)
    inside = (ix >= 0) & (ix < G) & (iy >= 0) & (iy < G)
    assert inside.sum() > 0.5 * len(x) and (~inside).sum() > 0          # both kinds are exercised
    x, ix, iy = x[inside], ix[inside], iy[inside]
    rec = cells[iy, ix].astype(np.int64)
    listed = rec[:, 7] != 0xFFFF
    for winner in (nearest_fp32(x, cb), nearest_fp64(x, cb)):
        hit = (rec == winner[:, None]).any(axis=1)
        assert (hit | ~listed).all(), f"{int((~hit & listed).sum())} winners missing from their cell's record"
    # and the record alone reproduces the whole-codebook search, ties included
    w32 = nearest_fp32(x, cb)
    d = dist_fp32(x[:, None, :], cb[np.where(rec == 0xFFFF, 0, rec)])           # [n][8]
    pick = rec[np.arange(len(x)), d.argmin(axis=1)]
    assert (pick[listed] == w32[listed]).all()


def test_degenerate_codebooks():
    # all codewords at the origin: every cell lists all of them (two fit a record; 16 do not)
    table, longest, overflow = qamw.search_grid(np.zeros((2, 2), np.float32), 1)
    _, G, inv_h, R, cells = parse(table)
    assert R == 1.0 and longest == 2 and overflow == 0 and (cells[:, :, :2] == [0, 1]).all()
    table, longest, overflow = qamw.search_grid(np.zeros((16, 2), np.float32), 4)
    _, G, _, _, cells = parse(table)
    assert longest == 16 and overflow == G * G and (cells[:, :, 7] == 0xFFFF).all()
    # duplicates of a nearest codeword are all listed (the lowest index must be able to win)
    cb = np.array([[1, 1], [-1, -1], [1, 1], [-1, 1]], np.float32)
    table, _, _ = qamw.search_grid(cb, 2)
    _, G, inv_h, _, cells = parse(table)
    ix = int(cell_of(np.array([0.9], np.float32), inv_h, G)[0])
    rec = set(cells[ix, ix].tolist())
    assert {0, 2} <= rec


def test_rejects_bad_arguments():
    L = qamw.lib()
    g, n = C.c_int(), C.c_size_t()
    assert L.qamw_search_grid_size(0, C.byref(g), C.byref(n)) == qamw.ERR_INVALID_ARG
    assert L.qamw_search_grid_size(13, C.byref(g), C.byref(n)) == qamw.ERR_INVALID_ARG
    assert L.qamw_search_grid_size(11, None, None) == qamw.OK
    assert L.qamw_search_grid_size(11, C.byref(g), C.byref(n)) == qamw.OK and g.value == 256 and n.value == 32 + 16 * 65536
    cb = np.zeros((8, 2), np.float32)
    buf = np.zeros(qamw.search_grid_size(3)[1], np.uint8)
    args = lambda **kw: [kw.get("cb", cb.ctypes.data), kw.get("bits", 3), kw.get("out", buf.ctypes.data),
                         kw.get("nbytes", len(buf)), None, None]
    assert L.qamw_search_grid_build(*args()) == qamw.OK
    assert L.qamw_search_grid_build(*args(cb=None)) == qamw.ERR_INVALID_ARG
    assert L.qamw_search_grid_build(*args(out=None)) == qamw.ERR_INVALID_ARG
    assert L.qamw_search_grid_build(*args(bits=0)) == qamw.ERR_INVALID_ARG
    assert L.qamw_search_grid_build(*args(nbytes=len(buf) - 1)) == qamw.ERR_INVALID_ARG
    bad = cb.copy()
    bad[3, 1] = np.inf
    assert L.qamw_search_grid_build(*args(cb=bad.ctypes.data)) == qamw.ERR_INVALID_ARG

    p = C.c_void_p(0x1000)

    def enc(**kw):
        a = dict(W=p, dtype=0, d_out=8, d_in=256, ldw=256, cb=p, bits=11, block=128, grid=p, packed=p, norms=p)
        a.update(kw)
        return L.qamw_encode_pruned(a["W"], a["dtype"], a["d_out"], a["d_in"], a["ldw"], None, None, None, a["cb"], a["bits"],
                                    a["block"], a["grid"], a["packed"], a["norms"], None, None)

    for k in ("W", "cb", "grid", "packed", "norms"):
        assert enc(**{k: None}) == qamw.ERR_INVALID_ARG
    assert enc(dtype=7) == qamw.ERR_INVALID_ARG
    assert enc(bits=0) == qamw.ERR_INVALID_ARG
    assert enc(grid=C.c_void_p(0x1008)) == qamw.ERR_INVALID_ARG
    assert enc(ldw=100) == qamw.ERR_SHAPE
    assert enc(block=96) == qamw.ERR_SHAPE
    assert enc(d_in=64, ldw=64, block=32) == qamw.ERR_UNSUPPORTED
    assert enc(W=C.c_void_p(0x1004)) == qamw.ERR_UNSUPPORTED
