"""The MFMA-only measurement aid: it runs, fills its sink, and computes what it says it computes
(checked against torch on the CPU for one wave's accumulators summed per lane)."""
import numpy as np
import pytest
import torch

from paper_2604_22782_amd import calib as skv

pytestmark = pytest.mark.gpu


def test_mfma_calibration_kernel_result():
    g = torch.Generator().manual_seed(5)
    ops = torch.randn(16, 64, 8, generator=g).to(torch.bfloat16)      # [operand][lane][8 values]
    blocks, iters = 3, 2
    sink = torch.full((blocks * 256,), float("nan"), dtype=torch.float32, device="cuda")
    skv.skv_calib_mfma_bf16(ops.cuda(), sink, blocks, iters)
    got = sink.cpu().double().numpy().reshape(blocks * 4, 64)
    # v_mfma_f32_32x32x16: lane l holds row (A) / column (B) l % 32, k values 8 (l / 32) .. + 7 of the step
    o = ops.double().numpy()
    def mat(i):           # operand block -> [32][16]
        return o[i].reshape(2, 32, 8).transpose(1, 0, 2).reshape(32, 16)
    total = np.zeros(64)
    for j in range(4):
        acc = np.zeros((32, 32))
        for i in range(8):
            acc += mat(2 * i) @ mat(2 * ((i + j) % 8) + 1).T
        acc *= iters
        # accumulator layout: lane l, register r holds row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
        for l in range(64):
            rows = [8 * (r // 4) + 4 * (l // 32) + r % 4 for r in range(16)]
            total[l] += acc[rows, l % 32].sum()
    assert np.allclose(got, total[None, :], rtol=1e-4, atol=1e-3)
    # the variants with vector and LDS work between the MFMAs compute the same thing
    for mix in (0, 1, 2, 3):
        other = torch.full_like(sink, float("nan"))
        skv.skv_calib_mfma_mix_bf16(ops.cuda(), other, blocks, iters, mix)
        assert torch.equal(other, sink), mix
    with pytest.raises(RuntimeError):
        skv.skv_calib_mfma_mix_bf16(ops.cuda(), sink, blocks, iters, 4)
    with pytest.raises(RuntimeError):
        skv.skv_calib_mfma_bf16(ops.cuda(), sink, blocks, 0)
