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
from workloads import SPECS, custom_spec, make_workload

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


def test_code_matrix_beyond_4_gib():
    """Maximum sizes: activations whose packed codes exceed 4 GiB (the matrix-core GEMM addresses operand rows with
    32-bit byte offsets and takes such operands in token slices).  Sampled tokens, among them the first, the last
    and those either side of the slice boundary, against the oracle: codes, accumulators, outputs."""
    T, d, d_e, N = 262144 + 300, 96, 32768, 192
    assert T * (d_e // 2) > 1 << 32
    wl = make_workload(custom_spec(T, d, d_e, N, in_dtype="bf16", act_dist="student_t3", outlier_frac=0.02,
                                   outlier_gain=30.0, seed=11))
    xd = to_device(wl.x, "bf16")
    wd = pme.pack_int4_codes(torch.from_numpy(wl.qw)).cuda()
    swd = torch.from_numpy(wl.sw).cuda()
    y = pme.expanded_linear(xd, d_e, wd, swd)
    qx, sx = pme.hadamard_expand_quant(xd, d_e)
    acc = pme.w4a4_gemm_i32(qx, wd)
    torch.cuda.synchronize()

    edge = ((1 << 32) - 1) // (d_e // 2) // 256 * 256          # first token of the second slice
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, edge - 1, edge, edge + 1, T - 2, T - 1], rng.choice(T, 41, replace=False)]))
    idx = torch.from_numpy(rows).cuda()
    ref_x = oracle.rotate_structured(wl.x[rows], d_e)
    q_ref, s_ref = oracle.quantize_sym_int4(ref_x)
    q_gpu = unpack_gpu(qx[idx])
    s_gpu = sx[idx].cpu().numpy()
    check_scales(s_gpu, s_ref)
    check_codes(q_gpu, q_ref, ref_x, s_ref)
    acc_ref = oracle.int_gemm(q_gpu, wl.qw)
    assert np.array_equal(acc[idx].cpu().numpy(), acc_ref)
    check_bf16(y[idx].to(torch.float32).cpu().numpy(), oracle.dequant_bf16(acc_ref, s_gpu, wl.sw))
    # every token was written: a code of magnitude 7 in each row, also in the second slice
    tail = unpack_gpu(qx[edge - 64:])
    assert np.all(np.abs(tail).max(axis=1) == 7)


def test_weight_matrix_beyond_4_gib():
    """The same limit on the other operand: packed weights above 4 GiB go through the GEMM in slices of output
    channels.  Random codes drawn on the device (seeded); sampled output channels, among them those either side
    of the slice boundary, against the oracle."""
    T, d_e, N = 100, 32768, 262144 + 200
    g = torch.Generator(device="cuda").manual_seed(3)
    qw = torch.randint(0, 256, (N, d_e // 2), dtype=torch.uint8, device="cuda", generator=g)
    qx = torch.randint(0, 256, (T, d_e // 2), dtype=torch.uint8, device="cuda", generator=g)
    sw = torch.rand(N, device="cuda", generator=g) * 0.02 + 0.001
    sx = torch.rand(T, device="cuda", generator=g) * 0.5 + 0.01
    assert qw.numel() > 1 << 32
    acc = pme.w4a4_gemm_i32(qx, qw)
    y = pme.w4a4_gemm(qx, sx, qw, sw)
    torch.cuda.synchronize()
    edge = ((1 << 32) - 1) // (d_e // 2) // 256 * 256
    rng = np.random.default_rng(6)
    cols = np.unique(np.concatenate([[0, 1, edge - 1, edge, edge + 1, N - 2, N - 1], rng.choice(N, 57, replace=False)]))
    idx = torch.from_numpy(cols).cuda()
    acc_ref = oracle.int_gemm(unpack_gpu(qx), unpack_gpu(qw[idx]))
    assert np.array_equal(acc[:, idx].cpu().numpy(), acc_ref)
    y_ref = oracle.dequant_bf16(acc_ref, sx.cpu().numpy(), sw[idx].cpu().numpy())
    check_bf16(y[:, idx].to(torch.float32).cpu().numpy(), y_ref)
