"""Parity at the full benchmark sizes, in the launch configuration bench.py times (PATH_AUTO).

The GPU computes the whole workload; the oracle checks every token of the rotate + quantize stage
(a token sample for the largest workload) and a random sample of token rows of the GEMM, each row
against all N outputs: int32 accumulators bit-exact, bf16 outputs within 1e-2 relative."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_17513_amd as pme
from parity_util import check_bf16, check_codes, check_scales, to_device, unpack_gpu
from workloads import SPECS, make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ("C2", "C3", "C4", "C5"))
def test_full_workload(name):
    wl = make_workload(name)
    sp = wl.spec
    xd = to_device(wl.x, sp.in_dtype)
    wd = pme.pack_int4_codes(torch.from_numpy(wl.qw)).cuda()
    swd = torch.from_numpy(wl.sw).cuda()
    assert pme.get_path() == pme.PATH_AUTO
    y = pme.expanded_linear(xd, sp.d_e, wd, swd)
    qx, sx = pme.hadamard_expand_quant(xd, sp.d_e)
    acc = pme.w4a4_gemm_i32(qx, wd)
    torch.cuda.synchronize()

    rng = np.random.default_rng(123)
    # rotate + quantize: every token, or 512 sampled tokens (first and last included) for the largest
    if sp.T * sp.d_e > 2048 * 8704:
        rows = np.unique(np.concatenate([[0, sp.T - 1], rng.choice(sp.T, 510, replace=False)]))
    else:
        rows = np.arange(sp.T)
    ref_x = oracle.rotate_structured(wl.x[rows], sp.d_e)
    q_ref, s_ref = oracle.quantize_sym_int4(ref_x)
    q_gpu_all = unpack_gpu(qx)
    sx_all = sx.cpu().numpy()
    check_scales(sx_all[rows], s_ref)
    check_codes(q_gpu_all[rows], q_ref, ref_x, s_ref)

    # GEMM: sampled token rows against all N outputs, from the library's own codes
    grow = np.unique(np.concatenate([[0, sp.T - 1], rng.choice(sp.T, min(sp.T, 62), replace=False)]))
    acc_ref = oracle.int_gemm(q_gpu_all[grow], wl.qw)
    assert np.array_equal(acc.cpu().numpy()[grow], acc_ref)
    y_ref = oracle.dequant_bf16(acc_ref, sx_all[grow], wl.sw)
    check_bf16(y.to(torch.float32).cpu().numpy()[grow], y_ref)
    # properties that hold at any size: every non-zero token reaches +-7, nothing leaves [-7, 7]
    assert q_gpu_all.min() >= -7 and q_gpu_all.max() <= 7
    assert np.all(np.abs(q_gpu_all).max(axis=1) == 7)
