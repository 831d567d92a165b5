"""Helpers shared by the GPU parity tests: case construction from the seeded generators, the
oracle run, and the acceptance checks (the tolerances live here, in the tests)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2605_26339_amd import qamw, synth

# Acceptance bars ------------------------------------------------------------------------------
NEAR_TIE_REL_GAP = 1e-6      # indices may differ from the oracle only where (d2 - d1) < 1e-6 * d2
DECODE_REL_TOL = 1e-5        # fp32 value before the cast: |gpu - spec oracle| <= 1e-5 * |oracle| per element
DECODE_ROW_TOL = 1e-5        # and vs the fp64 oracle: max_j |diff| <= 1e-5 * max_j |oracle| per row
BF16_ULPS = 1                # bf16 output: at most one unit in the last place from the oracle's cast


class Case:
    """One matrix with its side inputs on the host (numpy) and on the device (torch)."""

    def __init__(self, orc, seed, d_out, d_in, bits, block, dtype="f32", scale=True, signs=True, sigma="calibrated",
                 row_sigma=0.5, codebook=None, ldw=None, W=None):
        self.d_out, self.d_in, self.bits, self.block, self.dtype = d_out, d_in, bits, block, dtype
        W32 = synth.weight_host(seed, d_out, d_in, row_sigma) if W is None else np.asarray(W, dtype=np.float32)
        if dtype == "bf16":
            self.W_bits = synth.to_bf16_bits(W32)
            W32 = orc.bf16_bits_to_f32(self.W_bits)            # what the codec sees, widened exactly
        self.W = W32
        self.s = orc.channel_scales(synth.act_rms_host(seed + 1, d_in), 0.3) if scale else None
        self.sg = orc.sign_mask(seed + 2, d_in) if signs else None
        if isinstance(sigma, str) and sigma == "calibrated":
            self.sigma = orc.calibrate_sigma(self.W, block, chan_scale=self.s, signs=self.sg)
        else:
            self.sigma = sigma                                  # None or an explicit array
        self.cb = codebook
        self.ldw = d_in if ldw is None else ldw
        dev = "cuda"
        t = torch.from_numpy(self.W)
        if dtype == "bf16":
            t = torch.from_numpy(self.W_bits.view(np.int16)).view(torch.bfloat16)
        if self.ldw != d_in:
            full = torch.full((d_out, self.ldw), float("nan"), dtype=t.dtype)
            full[:, :d_in] = t
            self.W_dev = full.to(dev)[:, :d_in]
        else:
            self.W_dev = t.to(dev)
        self.s_dev = None if self.s is None else torch.from_numpy(self.s).to(dev)
        self.sg_dev = None if self.sg is None else torch.from_numpy(self.sg).to(dev)
        self.sigma_dev = None if self.sigma is None else torch.from_numpy(np.asarray(self.sigma, dtype=np.float32)).to(dev)
        self.cb_dev = torch.from_numpy(np.ascontiguousarray(codebook, dtype=np.float32)).to(dev)

    # ---- oracle side
    def oracle_encode(self, orc, mode=None, threads=8, rows=None):
        W = self.W if rows is None else self.W[rows]
        return orc.encode(W, self.cb, self.bits, self.block, chan_scale=self.s, signs=self.sg, pair_sigma=self.sigma,
                          mode=orc.MODE_SPEC if mode is None else mode, want_x=True, threads=threads)

    def oracle_decode(self, orc, idx, norms, mode=None, threads=8):
        return orc.decode(idx, norms, self.cb, self.bits, self.block, chan_scale=self.s, signs=self.sg,
                          pair_sigma=self.sigma, mode=orc.MODE_SPEC if mode is None else mode, threads=threads)

    # ---- device side (through the C ABI)
    def gpu_encode(self):
        packed, norms = qamw.encode(self.W_dev, self.cb_dev, self.bits, self.block, chan_scale=self.s_dev,
                                    signs=self.sg_dev, pair_sigma=self.sigma_dev)
        torch.cuda.synchronize()
        return packed.cpu().numpy(), norms.cpu().numpy()

    def gpu_decode(self, packed, norms, f32=False, ldo=None):
        pk = torch.from_numpy(np.ascontiguousarray(packed)).to("cuda")
        nr = torch.from_numpy(np.ascontiguousarray(norms, dtype=np.float32)).to("cuda")
        out = None
        if ldo is not None:
            full = torch.full((self.d_out, ldo), -7.0, dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
            out = full[:, :self.d_in]
        res = qamw.decode(pk, nr, self.d_in, self.cb_dev, self.bits, self.block, chan_scale=self.s_dev,
                          signs=self.sg_dev, pair_sigma=self.sigma_dev, out=out, f32=f32)
        torch.cuda.synchronize()
        if ldo is not None:
            assert bool((full[:, self.d_in:] == -7.0).all())   # nothing written beyond the row
        if f32:
            return res.cpu().numpy()
        return res.cpu().view(torch.int16).numpy().view(np.uint16)


# A row norm one ulp from the oracle's moves every point of the row: u = ws / r changes by at most 2^-23 relative and the
# butterflies add rounding differences of the same size per stage, so the kernel's point x' lies within
# eta = NORM_ULP_POINT_SHIFT * (1 + |x|) of the oracle's x (a bound with a wide margin; measured shifts are ~1e-7 |x|).
# If c' is nearest to x' then |x - c'| <= |x' - c'| + eta <= |x' - c1| + eta <= |x - c1| + 2 eta: that is asserted.
NORM_ULP_POINT_SHIFT = 2e-6


def check_encode(orc, case, packed, norms, ref, report=None, rows=None):
    """Indices bit-exact except at near-ties (counted); norms equal to the oracle's fp32 norms or one ulp off.  Rows
    whose norm is one ulp off (the fp64 summation order differs) are compared too: there an index may differ from the
    oracle's only if it is a near-tie or the chosen codeword is as near to the oracle's point as the best one up to
    the shift that one ulp of the norm can cause (needs ref["x"], the oracle's points)."""
    d_in, bits = case.d_in, case.bits
    rb = orc.packed_row_bytes(d_in, bits)
    assert packed.shape[1] == rb
    if rows is not None:
        packed, norms = packed[rows], norms[rows]
    ref_norms = ref["norms"].astype(np.float32)
    same_norm = norms == ref_norms
    ulp = np.abs(norms.view(np.int32).astype(np.int64) - ref_norms.view(np.int32).astype(np.int64))
    assert ulp.max(initial=0) <= 1, "row norm differs from the oracle by more than one ulp"
    n_norm_off = int((~same_norm).sum())
    assert n_norm_off <= max(1, int(1e-4 * norms.size))
    got = orc.unpack(packed, d_in, bits)
    assert got.min(initial=0) >= 0 and got.max(initial=0) < (1 << bits)
    # padding bits of every row are zero and the packed bytes equal the oracle's wherever indices agree
    mism = got != ref["idx"]
    diff = mism & same_norm[:, None]
    n_diff = int(diff.sum())
    if n_diff:
        d1, d2 = ref["d1"][diff], ref["d2"][diff]
        assert np.all((d2 - d1) < NEAR_TIE_REL_GAP * d2), "index mismatch away from a near-tie"
    # rows with a norm one ulp off: every mismatch is a near-tie or within the bound above
    off_diff = mism & ~same_norm[:, None]
    n_off_diff = int(off_diff.sum())
    if n_off_diff:
        assert ref.get("x") is not None, "rows with a one-ulp norm difference have index mismatches and the oracle's points were not kept"
        x = ref["x"][off_diff]                                         # [n][2] fp64, the oracle's points
        cbk = np.asarray(case.cb, dtype=np.float64)
        d_got = ((x - cbk[got[off_diff]]) ** 2).sum(-1)
        d1, d2 = ref["d1"][off_diff], ref["d2"][off_diff]
        eta = NORM_ULP_POINT_SHIFT * (1.0 + np.abs(x).max(-1))
        near_tie = (d2 - d1) < NEAR_TIE_REL_GAP * d2
        ok = near_tie | (np.sqrt(d_got) <= np.sqrt(d1) * (1 + 1e-6) + 2 * eta)
        assert np.all(ok), "index mismatch in a row whose norm is one ulp off, beyond what that ulp can cause"
    near = ((ref["d2"] - ref["d1"]) < NEAR_TIE_REL_GAP * ref["d2"])
    repack = orc.pack(got, bits)
    assert np.array_equal(repack, packed), "padding bits or field layout differ"
    if report is not None:
        report.update(pairs=int(got.size), mismatches=n_diff, near_ties=int(near.sum()), norm_ulp_rows=n_norm_off,
                      norm_ulp_row_mismatches=n_off_diff)
    return n_diff


def bf16_order(bits16: np.ndarray) -> np.ndarray:
    """Map bf16 bit patterns to integers that are monotone in the represented value."""
    b = bits16.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def check_decode(orc, case, idx, norms, got_f32=None, got_bf16=None, threads=8):
    spec = case.oracle_decode(orc, idx, norms, mode=orc.MODE_SPEC, threads=threads)
    truth = case.oracle_decode(orc, idx, norms, mode=orc.MODE_TRUTH, threads=threads)
    out = {}
    if got_f32 is not None:
        ref = spec["w"]
        err = np.abs(got_f32.astype(np.float64) - ref)
        assert np.all(err <= DECODE_REL_TOL * np.abs(ref) + 1e-37), float((err / (np.abs(ref) + 1e-300)).max())
        rowmax = np.abs(truth["w"]).max(1, keepdims=True)
        errt = np.abs(got_f32.astype(np.float64) - truth["w"])
        assert np.all(errt <= DECODE_ROW_TOL * rowmax + 1e-37), float((errt / (rowmax + 1e-300)).max())
        out["f32_exact_fraction"] = float((got_f32.astype(np.float64) == ref).mean())
        out["f32_max_rel"] = float((err / (np.abs(ref) + 1e-300)).max())
    if got_bf16 is not None:
        d = np.abs(bf16_order(got_bf16) - bf16_order(spec["bf16"]))
        assert d.max(initial=0) <= BF16_ULPS
        out["bf16_exact_fraction"] = float((d == 0).mean())
    return out
