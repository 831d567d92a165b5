"""The calibration entry point that allocates nothing (qamw_calibrate_sigma_static) against the entry point it is
a variant of (qamw_calibrate_sigma, caller workspace): same pair scales bit for bit, on two calls in a row, the
second with a smaller input, so that whatever the first call left in the library's static scratch is there when the
second one runs."""
import sys

import numpy as np
import pytest
import torch

from paper_2605_26339_amd import qamw, synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _one(orc, seed, d_out, d_in, block, dtype, max_rows=1024):
    W = synth.weight_device(seed, d_out, d_in, 0.5, dtype)
    s_h = qamw.channel_scales(synth.act_rms_host(seed + 1, d_in), 0.3)
    sg_h = qamw.sign_mask(seed + 2, d_in)
    s, sg = torch.from_numpy(s_h).cuda(), torch.from_numpy(sg_h).cuda()
    want = qamw.calibrate_sigma(W, block, chan_scale=s, signs=sg, max_rows=max_rows)
    got = torch.full((d_in // 2,), -1.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    qamw.calibrate_sigma_static(W, block, got, chan_scale=s, signs=sg, max_rows=max_rows)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got, want), f"{d_out}x{d_in}: static-scratch result differs from the workspace entry point"
    # and both are the oracle's pair scales (the bar of the calibration parity test)
    head = W[:max_rows].float().cpu().numpy()
    ref = orc.calibrate_sigma(head, block, chan_scale=s_h, signs=sg_h, max_rows=max_rows)
    assert np.allclose(got.cpu().numpy(), ref, rtol=1e-6, atol=0)


def test_static_scratch_calibration_two_calls_second_smaller(orc):
    say("[no-alloc] 1500x4096 b=128 bf16, then 300x1280 b=256 f32, then 40x96 b=32 (general kernels)")
    _one(orc, 901, 1500, 4096, 128, "bf16")
    _one(orc, 902, 300, 1280, 256, "f32")                 # smaller: fewer rows, fewer pairs, other block
    _one(orc, 903, 40, 96, 32, "f32")                     # a shape the general kernels serve: only the norms use the scratch
    _one(orc, 904, 2000, 11008, 256, "bf16", max_rows=700)


def test_static_scratch_limit_and_errors():
    W = torch.zeros((4, 32768), dtype=torch.float32, device="cuda")
    out = torch.zeros(16384, dtype=torch.float32, device="cuda")
    # 4 rows of 32768 columns still fit (one partial-sum chunk); 1024 rows of them do not
    qamw.calibrate_sigma_static(W, 128, out)
    W2 = torch.zeros((1024, 32768), dtype=torch.bfloat16, device="cuda")
    assert qamw.calibrate_workspace_bytes(32768, 1024) > qamw.STATIC_SCRATCH_BYTES
    with pytest.raises(qamw.QamwError) as ei:
        qamw.calibrate_sigma_static(W2, 128, out)
    assert ei.value.status == qamw.ERR_UNSUPPORTED
    with pytest.raises(qamw.QamwError) as ei:
        qamw.calibrate_sigma_static(W, 96, out)           # block not a power of two
    assert ei.value.status == qamw.ERR_SHAPE
    torch.cuda.synchronize()
