#!/usr/bin/env python3
"""Benchmark of the QAM-W codec hot path on one MI355X.

A step is one pass of the whole hot path over one model-shaped synthetic weight set that is
already resident in HBM: for every matrix, pair-scale calibration (Eq. 1) and encode (row norms,
rotation, nearest codeword, bit-pack), then decode of every layer to bf16; a layer's matrices go
through each entry point together (qamw_calibrate_sigma_batch, qamw_encode_batch, qamw_decode_batch).
Rank 0 prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--layers L]
                    [--decode-passes N] [--also NAME,NAME | --also none]
                    [--matmul M [--matmul-calls both|layer|site] [--matmul-path P]]
                    [--polar] [--no-pruned] [--no-valu-path] [--no-cpu-baseline]

The headline record (`value`, `roofline`, `roofline_decode`) is the 7B-shaped set at 11 bits (`--workload`).  The
workloads named by `--also` (default: the 7B set at 7 bits and the 13B set) are then measured the same way with one
warm-up and two steps each and 10 decode-only passes, and reported as sub-records under their names.

Beside the step: N decode-only passes over the set; the decoder's loads and stores without its arithmetic
(`roofline_decode.ceiling_gb_per_s`: what the memory system gives that access pattern); one encode pass with the
shortlist on the vector ALU instead of the matrix cores (`roofline.valu_only`); one encode pass with the pruned
nearest-codeword search (`pruned_search`; same indices, not part of `value` or of a roofline fraction); the fused
dequantise-and-multiply for M activation rows, 1 by default (`fused_matmul`; `--matmul 0` skips it); on request the
polar baseline (`polar_baseline`).

Timing uses HIP events recorded on the stream the kernels are launched on.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "encode Gpairs/s + decode GB/s (BF16 out), 7B-shaped weights; % of roofline"
PEAK_FP32_TFLOPS = 157.3          # MI355X vector fp32 (published)
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E (published)
PEAK_BF16_TFLOPS = 2500.0         # MI355X dense bf16 matrix cores (published)
FLOPS_PER_EVAL = 4.0              # one distance evaluation = 2 FMA
SHORTLIST_UNIT = ("shortlist scores on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 operands split exactly into "
                  "three bf16 pieces); min-reduction, exact fp32 recheck and whole-codebook scans on the vector ALU")


def build_workload(wl, layers, device):
    """Synthetic weights and side inputs of every matrix, generated on the device."""
    import torch

    from paper_2605_26339_amd import qamw, synth

    mats = []
    for layer in range(layers):
        site_cache = {}
        for name, d_out, d_in, site in wl.matrices:
            if site not in site_cache:
                a = synth.act_rms_host(synth.seed_for(wl.config_id, layer, site), d_in)
                s = torch.from_numpy(qamw.channel_scales(a, wl.alpha)).to(device)
                sg = torch.from_numpy(qamw.sign_mask(synth.seed_for(wl.config_id, layer, "mask-" + site), d_in)).to(device)
                site_cache[site] = (s, sg)
            s, sg = site_cache[site]
            W = synth.weight_device(synth.seed_for(wl.config_id, layer, name), d_out, d_in, wl.row_sigma, wl.dtype, device)
            rb = qamw.packed_row_bytes(d_in, wl.bits)
            mats.append(dict(name=f"L{layer}.{name}", W=W, s=s, sg=sg, d_out=d_out, d_in=d_in,
                             sigma=torch.empty(d_in // 2, dtype=torch.float32, device=device),
                             packed=torch.empty((d_out, rb), dtype=torch.uint8, device=device),
                             norms=torch.empty(d_out, dtype=torch.float32, device=device),
                             out=torch.empty((d_out, d_in), dtype=torch.bfloat16, device=device)))
    return mats


def run_step(layers, batches, wl, cb, ws, timed):
    """One pass: for every layer, pair-scale calibration of its matrices (qamw_calibrate_sigma_batch), their encode
    (qamw_encode_batch), and after all layers the decode of the set (qamw_decode_batch, several layers per call): one
    launch per call (calibration: two).  Returns the event triples (before calibration, between, after encode)
    per layer and the event pairs of each decode launch."""
    import torch

    from paper_2605_26339_amd import qamw

    ev_enc, ev_dec = [], []
    for cal_items, enc_items in layers:
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if timed else None
        if timed:
            e[0].record()
        qamw.calibrate_sigma_batch(cal_items, wl.block, ws)
        if timed:
            e[1].record()
        qamw.encode_batch(enc_items, cb, wl.bits, wl.block)
        if timed:
            e[2].record()
            ev_enc.append(e)
    for dec_items in batches:
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)] if timed else None
        if timed:
            e[0].record()
        qamw.decode_batch(dec_items, cb, wl.bits, wl.block)
        if timed:
            e[1].record()
            ev_dec.append(e)
    return ev_enc, ev_dec


def timed_passes(fn, n):
    """Milliseconds of n calls of fn(), each bracketed by events on the current stream."""
    import torch

    out = []
    for _ in range(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        out.append(e0.elapsed_time(e1))
    return out


def median(xs):
    return sorted(xs)[len(xs) // 2]


def measured_traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this workload (or None)."""
    rel = os.path.join("profiles", f"{workload}_hbm_traffic.json")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            d = json.load(f)
        return (d, rel) if d.get("workload") == workload else (None, None)
    except OSError:
        return None, None


def measure_workload(wl, layers, steps, warmup, decode_passes, dev, cb, valu_path=True):
    """Builds the set, runs `warmup` + `steps` steps, the decode-only passes, the traffic-only passes and (valu_path)
    one encode pass with the vector-ALU shortlist.  Returns (record dict, mats, batches, workspace)."""
    import torch

    from paper_2605_26339_amd import qamw

    mats = build_workload(wl, layers, dev)
    per_layer = len(wl.matrices)
    by_layer = [mats[i:i + per_layer] for i in range(0, len(mats), per_layer)]
    # decode: as many whole layers per qamw_decode_batch call as its item limit takes (4 layers of 7 matrices): a launch
    # of one layer is ~100 us of HBM time, of which the ramp-up and the tail of the launch are a tenth
    lpd = max(1, qamw.MAX_BATCH // per_layer)
    batches = [qamw.make_decode_items([(m["packed"], m["norms"], m["d_in"], m["s"], m["sg"], m["sigma"], m["out"])
                                       for lm in by_layer[i:i + lpd] for m in lm]) for i in range(0, len(by_layer), lpd)]
    layer_items = [(qamw.make_calibrate_items([(m["W"], m["s"], m["sg"], m["sigma"]) for m in lm]),
                    qamw.make_encode_items([(m["W"], m["s"], m["sg"], m["sigma"], m["packed"], m["norms"]) for m in lm]))
                   for lm in by_layer]
    ws = torch.empty(max(li[0][3] for li in layer_items), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    for _ in range(warmup):
        run_step(layer_items, batches, wl, cb, ws, timed=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    all_enc, all_dec = [], []
    for _ in range(steps):
        ev_enc, ev_dec = run_step(layer_items, batches, wl, cb, ws, timed=True)
        all_enc.extend(ev_enc)
        all_dec.extend(ev_dec)
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    total_ms = start.elapsed_time(stop)

    def decode_pass():
        for items in batches:
            qamw.decode_batch(items, cb, wl.bits, wl.block)

    def traffic_pass():
        for items in batches:
            qamw.decode_traffic_probe(items, cb, wl.bits, wl.block)

    # decode-only passes over the whole set (what a dequantise-before-matmul pipeline repeats), each timed as a whole
    pass_ms = timed_passes(decode_pass, decode_passes)
    # the decoder's loads and stores without its arithmetic: what the memory system gives this access pattern.  It
    # overwrites the decoded matrices with meaningless values, so the set is decoded again afterwards.
    probe_ms = timed_passes(traffic_pass, 1 + 5)[1:]
    decode_pass()

    # how often the encoder's shortlist could not decide and the whole codebook was scanned (first layer)
    scans = torch.zeros(1, dtype=torch.int64, device=dev)
    for m in mats[:per_layer]:
        qamw.encode(m["W"], cb, wl.bits, wl.block, chan_scale=m["s"], signs=m["sg"], pair_sigma=m["sigma"],
                    out=(m["packed"], m["norms"]), full_scans=scans)
    pairs_step = sum(m["d_out"] * m["d_in"] // 2 for m in mats)
    full_scan_fraction = float(scans.item()) / sum(m["d_out"] * m["d_in"] // 2 for m in mats[:per_layer])

    # the same encode with the shortlist on the vector ALU (no matrix cores): the path the fp32-ALU roofline describes
    valu = None
    if valu_path:
        prev = qamw.set_kernel_path(2)
        try:
            def encode_pass():
                for m in mats:
                    qamw.encode(m["W"], cb, wl.bits, wl.block, chan_scale=m["s"], signs=m["sg"], pair_sigma=m["sigma"],
                                out=(m["packed"], m["norms"]))
            ms = min(timed_passes(encode_pass, 2))
        finally:
            qamw.set_kernel_path(prev)
        tf = pairs_step * wl.K * FLOPS_PER_EVAL / (ms * 1e-3) / 1e12
        valu = {"kernel": "qamw_encode with qamw_set_kernel_path(2): shortlist, recheck and scans all on the vector ALU",
                "gpairs_per_s": pairs_step / (ms * 1e-3) / 1e9, "achieved": tf, "peak": PEAK_FP32_TFLOPS,
                "unit": "TFLOP/s", "frac": tf / PEAK_FP32_TFLOPS, "ms_per_pass": ms}

    cal_ms = sum(e[0].elapsed_time(e[1]) for e in all_enc)
    enc_ms = sum(e[1].elapsed_time(e[2]) for e in all_enc)
    dec_ms = sum(e[0].elapsed_time(e[1]) for e in all_dec)
    n_launch, n_dec_launch = len(all_enc), len(all_dec)
    pairs = pairs_step * steps
    evals = pairs * wl.K
    dec_bytes_step = pairs_step * (wl.bits / 8.0 + 4.0) + sum(4 * m["d_out"] for m in mats)
    dec_bytes = dec_bytes_step * steps
    enc_in_bytes = pairs * ((8 if wl.dtype == "f32" else 4) + wl.bits / 8.0)
    enc_tflops = evals * FLOPS_PER_EVAL / (enc_ms * 1e-3) / 1e12
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9
    ceiling_gbs = dec_bytes_step / (median(probe_ms) * 1e-3) / 1e9
    traffic, traffic_source = measured_traffic(wl.name) if layers == wl.layers else (None, None)
    mfma_tf = evals * 32.0 / (enc_ms * 1e-3) / 1e12
    rec = {
        "value": pairs / ((enc_ms + cal_ms) * 1e-3) / 1e9,
        "unit": "Gpairs/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": total_ms / steps,
        "config": {"workload": wl.name, "layers": layers, "matrices": len(mats), "weights": 2 * pairs_step,
                   "input_dtype": wl.dtype, "bits": wl.bits, "K": wl.K, "hadamard_block": wl.block},
        "encode": {"gpairs_per_s_kernels_only": pairs / (enc_ms * 1e-3) / 1e9,
                   "gpairs_per_s_with_calibration": pairs / ((enc_ms + cal_ms) * 1e-3) / 1e9,
                   "ms_per_step": enc_ms / steps, "calibration_ms_per_step": cal_ms / steps,
                   "hbm_gb_per_s": enc_in_bytes / (enc_ms * 1e-3) / 1e9,
                   "full_scan_fraction": full_scan_fraction},
        "decode": {"value": dec_gbs, "unit": "GB/s", "ms_per_step": dec_ms / steps,
                   "gpairs_per_s": pairs / (dec_ms * 1e-3) / 1e9,
                   "whole_set_passes": len(pass_ms),
                   "pass_gb_per_s_median": pass_ms and dec_bytes_step / (median(pass_ms) * 1e-3) / 1e9,
                   "pass_gb_per_s_best": pass_ms and dec_bytes_step / (min(pass_ms) * 1e-3) / 1e9,
                   "pass_frac_of_peak_median": pass_ms and dec_bytes_step / (median(pass_ms) * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "roofline": {"kernel": "qamw_encode_batch (one launch per layer, %d matrices: row norms + nearest-codeword search)" % per_layer, "bound": "alu",
                     "unit_doing_the_work": SHORTLIST_UNIT,
                     "achieved": enc_tflops, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                     "frac": enc_tflops / PEAK_FP32_TFLOPS,
                     "strict_roofline_gpairs_per_s": PEAK_FP32_TFLOPS * 1e3 / FLOPS_PER_EVAL / wl.K,
                     "traffic": traffic and traffic["encode"] * per_layer, "traffic_source": traffic_source,
                     "avg_launch_ms": enc_ms / n_launch,
                     "algorithmic_flops_per_launch": evals * FLOPS_PER_EVAL / n_launch,
                     # what the shortlist spends on the matrix cores to get there: one 32x32x16 bf16 tile
                     # (32768 flop) per 1024 evaluations, against the dense bf16 peak
                     "matrix_core": {"instruction": "v_mfma_f32_32x32x16_bf16", "tflops": mfma_tf,
                                     "peak": PEAK_BF16_TFLOPS, "frac": mfma_tf / PEAK_BF16_TFLOPS},
                     "valu_only": valu},
        "roofline_decode": {"kernel": "qamw_decode_batch (one launch per %d layers, %d matrices)" % (lpd, lpd * per_layer), "bound": "hbm",
                            "achieved": dec_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dec_gbs / PEAK_HBM_GBS,
                            "ceiling_gb_per_s": ceiling_gbs, "ceiling_frac_of_peak": ceiling_gbs / PEAK_HBM_GBS,
                            "frac_of_ceiling": dec_gbs / ceiling_gbs,
                            "ceiling_source": "qamw_decode_traffic_probe in this run: the same launches with every load and "
                                              "store of the decoder and none of its arithmetic, median of 5 whole-set passes",
                            "traffic": traffic and traffic["decode"] * (len(mats) / len(batches)),
                            "traffic_source": traffic_source,
                            "avg_launch_ms": dec_ms / n_dec_launch,
                            "algorithmic_bytes_per_launch": dec_bytes / n_dec_launch},
        "wall_s_timed_region": wall,
    }
    return rec, mats, batches, ws


def cpu_baseline(wl, mats, cb_host):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload (the first 4096 rows
    of the first matrix, about 16 core-seconds of encode at K = 2048) and on the small single-matrix configuration
    (2048 x 2048 fp32, the same codebook size), on all cores and on one."""
    import numpy as np

    from oracle import qamw_oracle as orc
    from paper_2605_26339_amd import qamw, synth

    m = mats[0]
    rows = min(4096, m["d_out"])
    W = m["W"][:rows].float().cpu().numpy()
    s, sg = m["s"].cpu().numpy(), m["sg"].cpu().numpy()
    cores = min(os.cpu_count() or 1, 16)
    sigma = orc.calibrate_sigma(W, wl.block, chan_scale=s, signs=sg)
    t0 = time.perf_counter()
    enc = orc.encode(W, cb_host, wl.bits, wl.block, chan_scale=s, signs=sg, pair_sigma=sigma, want_gaps=False, threads=cores)
    t1 = time.perf_counter()
    dec = orc.decode(enc["idx"], enc["norms"], cb_host, wl.bits, wl.block, chan_scale=s, signs=sg, pair_sigma=sigma,
                     threads=cores)
    t2 = time.perf_counter()
    pairs = rows * m["d_in"] // 2
    dec_bytes = pairs * (wl.bits / 8.0 + 4.0)
    del dec
    # the same on one core, on a sample 16 times smaller
    rows1 = max(1, rows // 16)
    t3 = time.perf_counter()
    enc1 = orc.encode(W[:rows1], cb_host, wl.bits, wl.block, chan_scale=s, signs=sg, pair_sigma=sigma, want_gaps=False, threads=1)
    t4 = time.perf_counter()
    orc.decode(enc1["idx"], enc1["norms"], cb_host, wl.bits, wl.block, chan_scale=s, signs=sg, pair_sigma=sigma, threads=1)
    t5 = time.perf_counter()
    pairs1 = rows1 * m["d_in"] // 2
    out = {"value": pairs / (t1 - t0) / 1e9, "unit": "Gpairs/s", "cores": cores, "kind": "oracle",
           "sample": f"first {rows} rows of {m['name']} ({m['d_out']}x{m['d_in']}) of {wl.name}, fp32 spec mode, "
                     f"encode {t1 - t0:.2f}s decode {t2 - t1:.2f}s; one core: first {rows1} rows, "
                     f"encode {t4 - t3:.2f}s decode {t5 - t4:.2f}s",
           "decode_value": dec_bytes / (t2 - t1) / 1e9, "decode_unit": "GB/s",
           "one_core_value": pairs1 / (t4 - t3) / 1e9,
           "one_core_decode_value": pairs1 * (wl.bits / 8.0 + 4.0) / (t5 - t4) / 1e9}
    # the small configuration, whole: one 2048 x 2048 fp32 matrix, block 128 (only if the codebook size is the same)
    c0 = synth.WORKLOADS["c0_single_2048"]
    if c0.bits == wl.bits:
        W0 = synth.weight_host(synth.seed_for(0, 0, "q"), 2048, 2048, c0.row_sigma)
        s0 = orc.channel_scales(synth.act_rms_host(synth.seed_for(0, 0, "attn_in"), 2048), c0.alpha)
        sg0 = orc.sign_mask(synth.seed_for(0, 0, "mask-attn_in"), 2048)
        sig0 = orc.calibrate_sigma(W0, c0.block, chan_scale=s0, signs=sg0)
        t0 = time.perf_counter()
        e0 = orc.encode(W0, cb_host, c0.bits, c0.block, chan_scale=s0, signs=sg0, pair_sigma=sig0, want_gaps=False, threads=cores)
        t1 = time.perf_counter()
        orc.decode(e0["idx"], e0["norms"], cb_host, c0.bits, c0.block, chan_scale=s0, signs=sg0, pair_sigma=sig0, threads=cores)
        t2 = time.perf_counter()
        p0 = 2048 * 1024
        out["c0_single_2048"] = {"value": p0 / (t1 - t0) / 1e9, "unit": "Gpairs/s", "cores": cores,
                                 "decode_value": p0 * (c0.bits / 8.0 + 4.0) / (t2 - t1) / 1e9, "decode_unit": "GB/s",
                                 "sample": f"the whole 2048x2048 matrix, encode {t1 - t0:.2f}s decode {t2 - t1:.2f}s"}
    return out


def fused_matmul_leg(args, wl, mats, cb, dev):
    """Y = X W^T for every matrix of the set without materialising W (what generating one token batch reads), next to
    the same products with the decoded bf16 matrices through torch."""
    import torch

    from paper_2605_26339_amd import qamw

    per_layer = len(wl.matrices)
    mm = args.matmul
    xs = {d: torch.randn((mm, d), device=dev, dtype=torch.float32).to(torch.bfloat16) for d in {m["d_in"] for m in mats}}
    ys = [torch.empty((mm, m["d_out"]), device=dev, dtype=torch.float32) for m in mats[:per_layer]]
    # one call per layer: its projections as independent products (a kernel benchmark; in a model some of
    # them depend on each other and would go in separate calls)
    mm_batches = [qamw.make_matmul_items([(xs[m["d_in"]], m["packed"], m["norms"], m["s"], m["sg"], m["sigma"], y)
                                          for m, y in zip(mats[i:i + per_layer], ys)]) for i in range(0, len(mats), per_layer)]
    # ... and as a forward pass has to issue them: one call per activation site (the products that share an
    # input: q/k/v, o, gate/up, down), each call depending on the one before
    site_batches = []
    for i in range(0, len(mats), per_layer):
        sites = []
        for (_, _, _, site), m, y in zip(wl.matrices, mats[i:i + per_layer], ys):
            if not sites or sites[-1][0] != site:
                sites.append((site, []))
            sites[-1][1].append((xs[m["d_in"]], m["packed"], m["norms"], m["s"], m["sg"], m["sigma"], y))
        site_batches += [qamw.make_matmul_items(entries) for _, entries in sites]
    ws_mm = torch.empty(max(b[4] for b in mm_batches + site_batches), dtype=torch.uint8, device=dev)
    times = {}
    prev_path = qamw.set_kernel_path(args.matmul_path)
    for kind in ("fused", "by_site", "bf16"):
        if (kind == "fused" and args.matmul_calls == "site") or (kind == "by_site" and args.matmul_calls == "layer"):
            times[kind] = None
            continue

        def one_pass():
            if kind != "bf16":
                for b in (mm_batches if kind == "fused" else site_batches):
                    qamw.matmul_batch(b, cb, wl.bits, wl.block, ws_mm)
            else:
                for m in mats:
                    torch.matmul(xs[m["d_in"]], m["out"].t())
        times[kind] = median(timed_passes(one_pass, 1 + 5)[1:])
    qamw.set_kernel_path(prev_path)
    pairs_set = sum(m["d_out"] * m["d_in"] // 2 for m in mats)
    fused_bytes = pairs_set * wl.bits / 8.0 + sum(4 * m["d_out"] + mm * (2 * m["d_in"] + 4 * m["d_out"]) for m in mats)
    bf16_bytes = pairs_set * 4.0 + sum(mm * 2 * (m["d_in"] + m["d_out"]) for m in mats)
    rate = lambda ms: ms and fused_bytes / (ms * 1e-3) / 1e9
    return {"rows": mm, "ms_per_pass": times["fused"], "gb_per_s": rate(times["fused"]),
            "frac_of_hbm_peak": times["fused"] and rate(times["fused"]) / PEAK_HBM_GBS,
            "algorithmic_bytes_per_pass": fused_bytes,
            "ms_per_pass_one_call_per_site": times["by_site"], "gb_per_s_one_call_per_site": rate(times["by_site"]),
            "calls_per_pass_by_site": len(site_batches),
            "bf16_matmul_ms_per_pass": times["bf16"], "bf16_matmul_gb_per_s": bf16_bytes / (times["bf16"] * 1e-3) / 1e9,
            "speedup_vs_bf16_matmul": times["fused"] and times["bf16"] / times["fused"],
            "speedup_vs_bf16_matmul_one_call_per_site": times["by_site"] and times["bf16"] / times["by_site"],
            "note": "median of 5 passes over the whole set, one qamw_matmul_batch call per layer (ms_per_pass) or one per activation site, the products that share an input (ms_per_pass_one_call_per_site); the bf16 leg is torch.matmul on the decoded matrices, one call per matrix"}


def polar_leg(wl, mats, dev):
    """The polar baseline at the same rate (amplitude bits + phase bits = B): one encode pass over the set."""
    import torch

    from paper_2605_26339_amd import qamw

    bits_a = wl.bits // 2
    bits_p = wl.bits - bits_a
    levels = torch.from_numpy(qamw.polar_codebook(bits_a, bits_p)[0]).to(dev)

    def one_pass():
        for m in mats:
            qamw.encode_polar(m["W"], levels, bits_a, bits_p, wl.block, chan_scale=m["s"], signs=m["sg"],
                              pair_sigma=m["sigma"], out=(m["packed"], m["norms"]))
    pol_ms = timed_passes(one_pass, 2)[1]
    pairs_set = sum(m["d_out"] * m["d_in"] // 2 for m in mats)
    in_bytes = pairs_set * ((8 if wl.dtype == "f32" else 4) + wl.bits / 8.0)
    return {"bits_amplitude": bits_a, "bits_phase": bits_p, "encode_gpairs_per_s": pairs_set / (pol_ms * 1e-3) / 1e9,
            "encode_ms_per_pass": pol_ms, "encode_hbm_gb_per_s": in_bytes / (pol_ms * 1e-3) / 1e9,
            "note": "same decoder as the joint code (table lookup); packed buffers are overwritten by this pass"}


def pruned_leg(wl, mats, cb, cb_host, dev):
    """The encoder with the pruned nearest-codeword search (same indices, far fewer distance evaluations): one encode
    pass over the set with the pair scales already calibrated.  Not part of `value` or the roofline: the roofline
    accounts a search over all K codewords."""
    import torch

    from paper_2605_26339_amd import qamw

    per_layer = len(wl.matrices)
    t_b = time.perf_counter()
    table, longest, overflow = qamw.search_grid(cb_host, wl.bits)
    build_s = time.perf_counter() - t_b
    grid = torch.from_numpy(table).to(dev)
    first = [qamw.encode(m["W"], cb, wl.bits, wl.block, chan_scale=m["s"], signs=m["sg"], pair_sigma=m["sigma"])
             for m in mats[:per_layer]]                          # the whole-codebook encoder's output, first layer
    scans_p = torch.zeros(1, dtype=torch.int64, device=dev)
    for m in mats[:per_layer]:
        qamw.encode_pruned(m["W"], cb, grid, wl.bits, wl.block, chan_scale=m["s"], signs=m["sg"], pair_sigma=m["sigma"],
                           out=(m["packed"], m["norms"]), full_scans=scans_p)
    same = all(torch.equal(m["packed"], f[0]) and torch.equal(m["norms"], f[1]) for m, f in zip(mats[:per_layer], first))

    def one_pass():
        for m in mats:
            qamw.encode_pruned(m["W"], cb, grid, wl.bits, wl.block, chan_scale=m["s"], signs=m["sg"], pair_sigma=m["sigma"],
                               out=(m["packed"], m["norms"]))
    pr = median(timed_passes(one_pass, 3))
    pairs_set = sum(m["d_out"] * m["d_in"] // 2 for m in mats)
    in_bytes = pairs_set * ((8 if wl.dtype == "f32" else 4) + wl.bits / 8.0)
    return {"encode_gpairs_per_s": pairs_set / (pr * 1e-3) / 1e9, "encode_ms_per_pass": pr,
            "encode_hbm_gb_per_s": in_bytes / (pr * 1e-3) / 1e9,
            "identical_to_whole_codebook_search": bool(same),
            "whole_codebook_scan_fraction": float(scans_p.item()) / sum(m["d_out"] * m["d_in"] // 2 for m in mats[:per_layer]),
            "grid_cells_per_side": qamw.search_grid_size(wl.bits)[0], "table_bytes": int(table.size),
            "longest_candidate_list": longest, "overflowing_cells": overflow, "table_build_s": build_s,
            "note": "median of 3 passes over the set (pruned-search kernel per matrix, pair scales given); "
                    "first layer compared byte for byte with qamw_encode's output"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c2_llama2_7b_b11")
    ap.add_argument("--layers", type=int, default=0, help="0 = the workload's own layer count")
    ap.add_argument("--decode-passes", type=int, default=10,
                    help="extra decode-only passes over the whole weight set after the timed steps (median and best reported)")
    ap.add_argument("--also", default="c3_llama2_7b_b7,c4_llama2_13b_b11",
                    help="comma-separated workloads measured after the headline one (1 warm-up + 2 steps + 10 decode-only passes each), "
                         "reported as sub-records; 'none' skips them")
    ap.add_argument("--matmul", type=int, default=1, metavar="M",
                    help="also time the fused dequantise-and-multiply with M activation rows over the whole set; 0 skips it")
    ap.add_argument("--matmul-calls", default="both", choices=("both", "layer", "site"),
                    help="fused-matmul leg: one call per layer, one per activation site, or both (default)")
    ap.add_argument("--matmul-path", type=int, default=0, choices=(0, 1, 2),
                    help="qamw_set_kernel_path() value during the fused-matmul leg (1 / 2: activations rotated by their own launch / inside the product kernel)")
    ap.add_argument("--polar", action="store_true", help="also time the polar-baseline encoder at the same bits per pair")
    ap.add_argument("--no-pruned", action="store_true", help="skip the pruned-search encoder leg")
    ap.add_argument("--no-valu-path", action="store_true", help="skip the encode pass with the shortlist on the vector ALU")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this codec benchmark runs on exactly one GPU (rows and matrices are independent; "
              "nothing is exchanged between devices). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_26339_amd import qamw, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    wl = synth.WORKLOADS[args.workload]
    layers = args.layers or wl.layers
    codebooks = {}

    def codebook_for(bits):
        if bits not in codebooks:
            host, mse, iters = qamw.train_codebook(bits, 1 << 20, seed=0)
            codebooks[bits] = (host, torch.from_numpy(host).to(dev), f"Lloyd, 2^20 samples, seed 0, mse {mse:.6f}, {iters} iterations")
        return codebooks[bits]

    cb_host, cb, cb_note = codebook_for(wl.bits)

    # a plain copy of known size: the reference the HBM byte counters are scaled by (rocprofv3 --pmc runs)
    probe_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    probe_dst = torch.empty_like(probe_src)
    probe_dst.copy_(probe_src)
    del probe_src, probe_dst

    rec, mats, batches, ws = measure_workload(wl, layers, args.steps, args.warmup, args.decode_passes, dev, cb,
                                              valu_path=not args.no_valu_path)
    rec["config"]["codebook"] = cb_note
    result = {"metric": METRIC, "value": rec["value"], "unit": rec["unit"], "n_gpus": 1, "steps": args.steps,
              "warmup": args.warmup, "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    for k in ("config", "encode", "decode", "roofline", "roofline_decode", "wall_s_timed_region"):
        result[k] = rec[k]
    if args.matmul:
        result["fused_matmul"] = fused_matmul_leg(args, wl, mats, cb, dev)
    if args.polar:
        result["polar_baseline"] = polar_leg(wl, mats, dev)
    if not args.no_pruned:
        result["pruned_search"] = pruned_leg(wl, mats, cb, cb_host, dev)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, mats, cb_host)

    # the other workloads of the metric: the headline set's buffers are released first (the 13B set needs ~61 GB)
    also = [] if args.also.strip().lower() in ("", "none") else [w.strip() for w in args.also.split(",") if w.strip()]
    del mats, batches, ws
    for name in also:
        if name == wl.name:
            continue
        gc.collect()
        torch.cuda.empty_cache()
        wl2 = synth.WORKLOADS[name]
        _, cb2, note2 = codebook_for(wl2.bits)
        rec2, mats2, batches2, ws2 = measure_workload(wl2, wl2.layers, 2, 1, 10, dev, cb2, valu_path=not args.no_valu_path)
        rec2["config"]["codebook"] = note2
        del mats2, batches2, ws2
        result[name] = rec2
    print(json.dumps(result))


if __name__ == "__main__":
    main()
