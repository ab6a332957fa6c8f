"""Parity at the full benchmark sizes, in the launch configuration bench.py times (PATH_AUTO).

The GPU computes the whole workload; the oracle checks every token of the rotate + quantize stage
(a token sample for the largest workload) and a random sample of token rows of the GEMM, each row
against all N outputs: int32 accumulators bit-exact, bf16 outputs within 1e-2 relative."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_17513_amd as pme
from parity_util import check_bf16, check_codes, check_mx_gemm, check_mx_quant, check_scales, to_device, unpack_gpu
from workloads import SPECS, custom_spec, make_workload

pytestmark = pytest.mark.gpu


def _sample_tokens(sp, rng):
    """Every token, or 512 sampled tokens (first and last included) for the largest workload."""
    if sp.T * sp.d_e > 2048 * 8704:
        return np.unique(np.concatenate([[0, sp.T - 1], rng.choice(sp.T, 510, replace=False)]))
    return np.arange(sp.T)


def _sample_gemm_rows(sp, rng):
    return np.unique(np.concatenate([[0, sp.T - 1], rng.choice(sp.T, min(sp.T, 62), replace=False)]))


@pytest.mark.parametrize("name", ("C2", "C3", "C4", "C5"))
def test_full_workload(name):
    wl = make_workload(name)
    sp = wl.spec
    xd = to_device(wl.x, sp.in_dtype)
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
    swd = torch.from_numpy(wl.sw).cuda()
    assert pme.get_path() == pme.PATH_AUTO
    y = pme.expanded_linear(xd, sp.d_e, wd, swd)
    qx, sx = pme.hadamard_expand_quant(xd, sp.d_e)
    acc = pme.w4a4_gemm_i32(qx, wd)
    torch.cuda.synchronize()

    rng = np.random.default_rng(123)
    rows = _sample_tokens(sp, rng)
    ref_x = oracle.rotate_structured(wl.x[rows], sp.d_e)
    q_ref, s_ref = oracle.quantize_sym_int4(ref_x)
    q_gpu_all = unpack_gpu(qx)
    sx_all = sx.cpu().numpy()
    check_scales(sx_all[rows], s_ref)
    check_codes(q_gpu_all[rows], q_ref, ref_x, s_ref)

    # GEMM: sampled token rows against all N outputs, from the library's own codes
    grow = _sample_gemm_rows(sp, rng)
    acc_ref = oracle.int_gemm(q_gpu_all[grow], wl.qw)
    assert np.array_equal(acc.cpu().numpy()[grow], acc_ref)
    y_ref = oracle.dequant_bf16(acc_ref, sx_all[grow], wl.sw)
    check_bf16(y.to(torch.float32).cpu().numpy()[grow], y_ref)
    # properties that hold at any size: every non-zero token reaches +-7, nothing leaves [-7, 7]
    assert q_gpu_all.min() >= -7 and q_gpu_all.max() <= 7
    assert np.all(np.abs(q_gpu_all).max(axis=1) == 7)


@pytest.mark.parametrize("name", ("C2", "C3", "C4", "C5"))
def test_full_workload_asymmetric(name):
    """The layer with the paper's own activation quantizer (Section 4: per-token asymmetric int4) at the
    benchmark sizes, automatic kernel and tile choice: scales, zero points and codes of the sampled tokens
    against the oracle's quantizer, the fused call bit-equal to the chain of its parts, and sampled token rows
    of the output against the oracle's GEMM and epilogue evaluated on the library's codes."""
    wl = make_workload(name)
    sp = wl.spec
    xd = to_device(wl.x, sp.in_dtype)
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
    swd = torch.from_numpy(wl.sw).cuda()
    assert pme.get_path() == pme.PATH_AUTO
    wsum = pme.weight_rowsum(wd)
    assert np.array_equal(wsum.cpu().numpy(), wl.qw.astype(np.int64).sum(axis=1))
    y = pme.expanded_linear_asym(xd, sp.d_e, wd, swd, wsum)
    qx, sx, zx = pme.hadamard_expand_quant_asym(xd, sp.d_e)
    y2 = pme.w4a4_gemm_asym(qx, sx, zx, wd, swd, wsum)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))

    rng = np.random.default_rng(321)
    rows = _sample_tokens(sp, rng)
    ref_x = oracle.rotate_structured(wl.x[rows], sp.d_e)
    q_ref, s_ref, z_ref = oracle.quantize_asym_int4(ref_x)
    q_gpu_all = unpack_gpu(qx, signed=False)
    sx_all, zx_all = sx.cpu().numpy(), zx.cpu().numpy()
    check_scales(sx_all[rows], s_ref)
    # a zero point may differ by one only where -lo / s sits at a rounding tie; such a token's codes are all
    # shifted with it and are left out of the code comparison
    zdiff = zx_all[rows] != z_ref
    if zdiff.any():
        lo = np.minimum(ref_x.min(axis=1), 0.0)
        scaled = -lo / s_ref.astype(np.float64)
        assert np.all(np.abs(np.abs(scaled - np.floor(scaled)) - 0.5)[zdiff] < 5e-5)
        assert np.all(np.abs(zx_all[rows] - z_ref)[zdiff] == 1) and zdiff.sum() <= 1
    keep = ~zdiff
    check_codes(q_gpu_all[rows][keep], q_ref[keep], ref_x[keep], s_ref[keep])
    assert q_gpu_all.max() <= 15 and np.all(q_gpu_all.max(axis=1) - q_gpu_all.min(axis=1) == 15)

    grow = _sample_gemm_rows(sp, rng)
    acc_ref = oracle.int_gemm(q_gpu_all[grow], wl.qw)
    y_ref = oracle.dequant_asym_bf16(acc_ref, sx_all[grow], zx_all[grow], wl.qw, wl.sw)
    check_bf16(y.to(torch.float32).cpu().numpy()[grow], y_ref)


@pytest.mark.parametrize("name", ("C2", "C3", "C4", "C5"))
def test_full_workload_mxfp4(name):
    """The MXFP4 layer (Section 4, second setting) at the benchmark sizes, automatic kernel and tile choice.
    Weights: seeded Gaussian W^T [N, d] on the bf16 grid, expanded and quantized by the library's own
    weight-side call and checked on sampled channels against the oracle's quantizer; activations: the
    workload's.  Sampled token rows of the output against the oracle's block-scaled GEMM on the library's codes."""
    wl = make_workload(name, weights=False)
    sp = wl.spec
    rng = np.random.default_rng(77)
    wt = torch.from_numpy(rng.standard_normal((sp.N, sp.d), dtype=np.float32) / np.float32(np.sqrt(sp.d)))
    wt = wt.to(torch.bfloat16).to(torch.float32).numpy()
    xd = to_device(wl.x, sp.in_dtype)
    wtd = to_device(wt, "bf16")
    assert pme.get_path() == pme.PATH_AUTO
    qw, ew = pme.hadamard_expand_quant_mxfp4(wtd, sp.d_e)
    y = pme.expanded_linear_mxfp4(xd, sp.d_e, qw, ew)
    qx, ex = pme.hadamard_expand_quant_mxfp4(xd, sp.d_e)
    y2 = pme.mxfp4_gemm(qx, ex, qw, ew)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))

    rows = _sample_tokens(sp, rng)
    if rows.size > 512:
        rows = np.unique(np.concatenate([[0, sp.T - 1], rng.choice(sp.T, 510, replace=False)]))
    idx = torch.from_numpy(rows).cuda()
    check_mx_quant(qx[idx], ex[idx], oracle.rotate_structured(wl.x[rows], sp.d_e))
    chans = np.unique(np.concatenate([[0, sp.N - 1], rng.choice(sp.N, 254, replace=False)]))
    cidx = torch.from_numpy(chans).cuda()
    check_mx_quant(qw[cidx], ew[cidx], oracle.rotate_structured(wt[chans], sp.d_e))

    grow = _sample_gemm_rows(sp, rng)
    gidx = torch.from_numpy(grow).cuda()
    check_mx_gemm(y[gidx].to(torch.float32).cpu().numpy(), oracle.unpack_fp4(qx[gidx].cpu().numpy()), ex[gidx].cpu().numpy(),
                  oracle.unpack_fp4(qw.cpu().numpy()), ew.cpu().numpy())


def test_code_matrix_beyond_4_gib():
    """Maximum sizes: activations whose packed codes exceed 4 GiB (the matrix-core GEMM addresses operand rows with
    32-bit byte offsets and takes such operands in token slices).  Sampled tokens, among them the first, the last
    and those either side of the slice boundary, against the oracle: codes, accumulators, outputs."""
    T, d, d_e, N = 262144 + 300, 96, 32768, 192
    assert T * (d_e // 2) > 1 << 32
    wl = make_workload(custom_spec(T, d, d_e, N, in_dtype="bf16", act_dist="student_t3", outlier_frac=0.02,
                                   outlier_gain=30.0, seed=11))
    xd = to_device(wl.x, "bf16")
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
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
