"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Sizes are small enough for the oracle to finish in seconds yet span several MFMA
tiles, several waves per token and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_17513_amd as pme
from parity_util import check_bf16, check_codes, check_scales, check_xhat, to_device, unpack_gpu
from workloads import custom_spec, make_workload

pytestmark = pytest.mark.gpu

GENERIC, MFMA = pme.PATH_GENERIC, pme.PATH_MFMA


@pytest.fixture(autouse=True)
def _reset_path():
    yield
    pme.set_path(pme.PATH_AUTO)
    pme.set_gemm_tile(0)


# (name, T, d, d_e, in_dtype, paths)
ROTATE_CASES = [
    ("tiny_c1", 16, 64, 80, "f32", (GENERIC,)),
    ("b68_k5", 37, 2048, 2176, "bf16", (GENERIC, MFMA)),
    ("b68_k7", 9, 8192, 8704, "bf16", (GENERIC, MFMA)),
    ("b132_k6", 8, 8192, 8448, "bf16", (GENERIC, MFMA)),
    ("b60_k8", 5, 14336, 15360, "bf16", (GENERIC, MFMA)),
    ("b68_k5_many_tokens", 700, 2048, 2176, "bf16", (MFMA,)),
    ("b68_k7_many_tokens", 600, 8192, 8704, "bf16", (MFMA,)),
    ("b60_k8_many_tokens", 520, 14336, 15360, "bf16", (MFMA,)),
    ("ragged_d_inside_base_row", 6, 2000, 2176, "bf16", (GENERIC, MFMA)),
    ("ragged_d_small", 6, 304, 2176, "bf16", (GENERIC, MFMA)),
    ("ragged_d_not_multiple_of_8", 6, 300, 2176, "bf16", (GENERIC,)),
    ("odd_d", 4, 301, 2176, "bf16", (GENERIC,)),
    ("f32_b68_k5", 7, 2048, 2176, "f32", (GENERIC, MFMA)),
    ("f32_b132_k6", 3, 8192, 8448, "f32", (GENERIC, MFMA)),
    ("pow2_ratio_one", 5, 256, 256, "bf16", (GENERIC, MFMA)),
    ("pow2_padded", 5, 200, 256, "f32", (GENERIC, MFMA)),
    # 2^k > 128 with a small block (required beyond 512): the matrix-core kernel folds the first butterfly stages
    # into the base block (4096 runs as 32 x 128, 12288 as 48 x 256, 32768 as 64 x 512, 40960 as 80 x 512)
    ("pow2_k12", 3, 4096, 4096, "bf16", (GENERIC, MFMA)),
    ("pow2_k10_ragged_d", 5, 1000, 1024, "bf16", (GENERIC, MFMA)),
    ("pow2_k13_f32", 3, 8192, 8192, "f32", (GENERIC, MFMA)),
    ("pow2_k15", 2, 30000, 32768, "bf16", (GENERIC, MFMA)),
    ("b12_k10_many_tokens", 300, 8192, 12288, "bf16", (MFMA,)),
    ("b20_k11", 3, 36000, 40960, "bf16", (MFMA,)),          # 160 KB of fp32: beyond the generic kernel's LDS buffer
    ("b12_k6", 4, 696, 768, "bf16", (GENERIC, MFMA)),
    ("b20_k5", 4, 600, 640, "bf16", (GENERIC, MFMA)),
    ("b72_k5", 4, 2104, 2304, "bf16", (GENERIC, MFMA)),
    ("b140_k6", 3, 8192, 8960, "bf16", (GENERIC, MFMA)),
    ("b152_k6", 3, 8192, 9728, "bf16", (GENERIC, MFMA)),
    # 20 column tiles on 7 waves, P fragments read from device memory
    ("b312_k6", 3, 14336, 19968, "bf16", (GENERIC, MFMA)),
    ("b312_k6_many_tokens_ragged_d", 290, 14000, 19968, "bf16", (MFMA,)),
    ("b344_k6", 3, 14336, 22016, "bf16", (GENERIC, MFMA)),          # block over GF(7^3), 22 tiles on 8 waves
    ("b344_k6_many_tokens", 270, 14336, 22016, "bf16", (MFMA,)),
    ("b20_k9", 3, 8192, 10240, "bf16", (GENERIC, MFMA)),
    ("b12_k10", 2, 8192, 12288, "bf16", (GENERIC, MFMA)),
    ("single_token", 1, 2048, 2176, "bf16", (GENERIC, MFMA)),
    ("b140_k6_three_tiles_per_wave", 3080, 8192, 8960, "bf16", (MFMA,)),          # the launch for 3072 tokens and more
    # 1024 tokens or more at 2^k = 32: workgroups whose waves each rotate tokens of their own (token counts
    # that do not divide by the waves of a workgroup, one- and five-tile blocks, ragged d)
    ("b68_k5_token_per_wave", 1030, 2048, 2176, "bf16", (MFMA,)),
    ("b20_k5_token_per_wave", 1027, 600, 640, "bf16", (MFMA,)),
    ("b72_k5_token_per_wave_ragged_d", 1025, 2104, 2304, "bf16", (MFMA,)),
]


def _acts(T, d, d_e, in_dtype, seed=0):
    spec = custom_spec(T, d, d_e, 8, in_dtype=in_dtype, act_dist="student_t3", outlier_frac=0.01,
                       outlier_gain=50.0, seed=seed)
    return make_workload(spec, weights=False).x


@pytest.mark.parametrize("name,T,d,d_e,in_dtype,paths", ROTATE_CASES, ids=[c[0] for c in ROTATE_CASES])
def test_rotate_and_quantize(name, T, d, d_e, in_dtype, paths):
    x = _acts(T, d, d_e, in_dtype, seed=len(name))
    x[0, : min(d, 7)] = 0.0
    if T > 2:
        x[1] = 0.0                      # an all-zero token
        x[2] = 0.0
        x[2, d // 2] = 1.0              # a one-hot token: every code is +-7
    xd = to_device(x, in_dtype)
    ref = oracle.rotate_structured(x, d_e)
    q_ref, s_ref = oracle.quantize_sym_int4(ref)
    for path in paths:
        pme.set_path(path)
        xhat = pme.hadamard_expand_f32(xd, d_e).cpu().numpy()
        check_xhat(xhat, ref)
        qx, sx = pme.hadamard_expand_quant(xd, d_e)
        torch.cuda.synchronize()
        check_scales(sx.cpu().numpy(), s_ref)
        check_codes(unpack_gpu(qx), q_ref, ref, s_ref)
        if T > 2:
            assert sx[1].item() == 1.0 and int(qx[1].max()) == 0
            assert np.all(np.abs(unpack_gpu(qx)[2]) == 7)


@pytest.mark.parametrize("path", (GENERIC, MFMA))
def test_rotate_strided_rows(path):
    # ldx > d: rows of a wider buffer
    T, d, d_e = 6, 2048, 2176
    x = _acts(T, 2560, 2560, "bf16", seed=5)
    xd_full = to_device(x, "bf16")
    xd = xd_full[:, :d]
    pme.set_path(path)
    ref = oracle.rotate_structured(x[:, :d], d_e)
    check_xhat(pme.hadamard_expand_f32(xd, d_e).cpu().numpy(), ref)


@pytest.mark.parametrize("d_h,d_he", ((64, 80), (128, 160), (128, 192)))
def test_per_head_expansion_of_the_value_and_output_projections(d_h, d_he):
    # Section 4, compute graph details: the head-wise rotation between the value and output projections is merged
    # into their weights, so expanding it is weight-side work only: each head's d_h columns of W_v and of W_o^T
    # (slices of wider matrices, hence the row pitch) go through X H_hat, and the product of the pair is unchanged
    d_model, heads = 192, 3
    rng = np.random.default_rng(7)
    wv = rng.standard_normal((d_model, heads * d_h)).astype(np.float32)          # x W_v: head h = columns h d_h ..
    wo_t = rng.standard_normal((d_model, heads * d_h)).astype(np.float32)        # W_o^T, same column layout
    wv_d, wo_d = torch.from_numpy(wv).cuda(), torch.from_numpy(wo_t).cuda()
    for h in range(heads):
        cols = slice(h * d_h, (h + 1) * d_h)
        a = pme.hadamard_expand_f32(wv_d[:, cols], d_he).cpu().numpy()
        b = pme.hadamard_expand_f32(wo_d[:, cols], d_he).cpu().numpy()
        check_xhat(a, oracle.rotate_structured(wv[:, cols], d_he))
        check_xhat(b, oracle.rotate_structured(wo_t[:, cols], d_he))
        exact = wv[:, cols].astype(np.float64) @ wo_t[:, cols].astype(np.float64).T
        assert np.max(np.abs(a.astype(np.float64) @ b.astype(np.float64).T - exact)) <= 1e-5 * np.max(np.abs(exact))


ASYM_CASES = [("tiny", 16, 64, 80, "f32", (GENERIC,)), ("b68_k5", 9, 2048, 2176, "bf16", (GENERIC, MFMA)),
              ("b60_k8", 4, 14336, 15360, "bf16", (GENERIC, MFMA)),
              ("b68_k5_token_per_wave", 1026, 2048, 2176, "bf16", (MFMA,)),
              ("b12_k10_folded", 5, 8192, 12288, "bf16", (GENERIC, MFMA)),
              ("b312_k6", 5, 14336, 19968, "bf16", (GENERIC, MFMA))]


@pytest.mark.parametrize("name,T,d,d_e,in_dtype,paths", ASYM_CASES, ids=[c[0] for c in ASYM_CASES])
def test_rotate_and_quantize_asymmetric(name, T, d, d_e, in_dtype, paths):
    x = _acts(T, d, d_e, in_dtype, seed=3) + np.float32(0.25)
    if in_dtype == "bf16":
        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    x[1] = 0.0
    xd = to_device(x, in_dtype)
    ref = oracle.rotate_structured(x, d_e)
    q_ref, s_ref, z_ref = oracle.quantize_asym_int4(ref)
    for path in paths:
        pme.set_path(path)
        qx, sx, zx = pme.hadamard_expand_quant_asym(xd, d_e)
        check_scales(sx.cpu().numpy(), s_ref)
        assert np.array_equal(zx.cpu().numpy(), z_ref)
        check_codes(unpack_gpu(qx, signed=False), q_ref, ref, s_ref)


# (name, T, N, d_e, paths)
GEMM_CASES = [
    ("tiny_c1", 16, 64, 80, (GENERIC,)),
    ("ragged_generic", 77, 130, 262, (GENERIC,)),
    ("one_k_step", 40, 72, 128, (GENERIC, MFMA)),
    ("small_tile_ragged", 100, 200, 2176, (GENERIC, MFMA)),
    ("tile_64x128", 500, 1100, 384, (MFMA,)),
    ("tile_128x128", 1000, 2100, 256, (MFMA,)),
    ("tile_128x192", 2048, 3072, 256, (MFMA,)),
    ("tile_128x256", 2000, 4200, 256, (MFMA,)),
    ("tile_256x256", 4000, 4100, 128, (MFMA,)),
    ("single_row_col", 1, 1, 2176, (GENERIC, MFMA)),
    ("decode_shape", 8, 2048, 8448, (GENERIC, MFMA)),
    ("decode_16_tokens_ragged_n", 16, 100, 384, (GENERIC, MFMA)),
    ("decode_one_chunk", 3, 40, 128, (GENERIC, MFMA)),
    ("decode_one_token_long_k", 1, 520, 15360, (GENERIC, MFMA)),
    ("decode_five_tokens_odd_chunks_ragged_n", 5, 36, 640, (GENERIC, MFMA)),
    ("decode_nine_tokens", 9, 50, 640, (GENERIC, MFMA)),
    # 17 .. 64 tokens: the weight-streaming kernel with 2, 3 or 4 groups of 16 tokens
    ("decode_17_tokens", 17, 64, 256, (GENERIC, MFMA)),
    ("decode_33_tokens_odd_chunks_ragged_n", 33, 100, 640, (GENERIC, MFMA)),
    ("decode_48_tokens", 48, 40, 384, (GENERIC, MFMA)),
    ("decode_64_tokens_shape", 64, 2048, 8448, (GENERIC, MFMA)),
    ("sixty_five_tokens_use_the_tiled_kernel", 65, 72, 256, (GENERIC, MFMA)),
]


@pytest.mark.parametrize("name,T,N,d_e,paths", GEMM_CASES, ids=[c[0] for c in GEMM_CASES])
def test_gemm_accumulators_and_epilogue(name, T, N, d_e, paths):
    rng = np.random.default_rng(len(name) + T)
    q = rng.integers(-7, 8, size=(T, d_e), dtype=np.int8)
    qw = rng.integers(-8, 8, size=(N, d_e), dtype=np.int8)
    if T > 1 and N > 1:
        q[0] = 7                         # extreme rows: the accumulator reaches its bound
        qw[0] = -8
        qw[N - 1] = 7
    sx = rng.uniform(0.01, 2.0, T).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    acc_ref = oracle.int_gemm(q, qw)
    y_ref = oracle.dequant_bf16(acc_ref, sx, sw)
    qd = torch.from_numpy(oracle.pack_int4(q)).cuda()
    wd = torch.from_numpy(oracle.pack_int4(qw)).cuda()
    sxd, swd = torch.from_numpy(sx).cuda(), torch.from_numpy(sw).cuda()
    for path in paths:
        pme.set_path(path)
        acc = pme.w4a4_gemm_i32(qd, wd).cpu().numpy()
        assert np.array_equal(acc, acc_ref), f"path {path}: {np.count_nonzero(acc != acc_ref)} accumulators differ"
        y = pme.w4a4_gemm(qd, sxd, wd, swd).to(torch.float32).cpu().numpy()
        check_bf16(y, y_ref)


@pytest.mark.parametrize("d_e", (1280, 1152, 128))
@pytest.mark.parametrize("tile", range(1, 29))
def test_gemm_every_tile_configuration(tile, d_e):
    # every entry of the MFMA kernel's tile table, forced through the tuning hook: ragged T and N; K of
    # 5 whole steps of 128 bytes, of 4.5 (a half-length last step), and of a single half step; extreme rows
    rng = np.random.default_rng(tile)
    T, N = 300, 520
    q = rng.integers(-7, 8, size=(T, d_e), dtype=np.int8)
    qw = rng.integers(-8, 8, size=(N, d_e), dtype=np.int8)
    q[0] = -7
    qw[1] = -8
    sx = rng.uniform(0.01, 2.0, T).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    acc_ref = oracle.int_gemm(q, qw)
    qd = torch.from_numpy(oracle.pack_int4(q)).cuda()
    wd = torch.from_numpy(oracle.pack_int4(qw)).cuda()
    pme.set_path(MFMA)
    pme.set_gemm_tile(tile)
    try:
        acc = pme.w4a4_gemm_i32(qd, wd).cpu().numpy()
        y = pme.w4a4_gemm(qd, torch.from_numpy(sx).cuda(), wd, torch.from_numpy(sw).cuda())
        y = y.to(torch.float32).cpu().numpy()
    finally:
        pme.set_gemm_tile(0)
    assert np.array_equal(acc, acc_ref)
    check_bf16(y, oracle.dequant_bf16(acc_ref, sx, sw))


@pytest.mark.parametrize("tm,tn", [(8, 1), (1, 8), (4, 2), (2, 4), (16, 16), (3, 5), (24, 8)])
def test_gemm_tile_map_is_a_bijection(tm, tn):
    # The workgroup -> tile map hands each XCD a block of tiles; the split (8x1, 4x2, 2x4, 1x8 XCDs, or none
    # when the tile counts do not divide) depends on the tile grid.  Every output must be written exactly
    # once and exactly: 64 x 64 and 64 x 128 tiles, one short K step.  A block of the output's size is
    # poisoned and released first, so that the allocator does not hand back an earlier, correct result.
    rng = np.random.default_rng(100 * tm + tn)
    T, N, d_e = 64 * tm, 64 * tn, 128
    q = rng.integers(-7, 8, size=(T, d_e), dtype=np.int8)
    qw = rng.integers(-8, 8, size=(N, d_e), dtype=np.int8)
    acc_ref = oracle.int_gemm(q, qw)
    qd = torch.from_numpy(oracle.pack_int4(q)).cuda()
    wd = torch.from_numpy(oracle.pack_int4(qw)).cuda()
    pme.set_path(MFMA)
    for tile in (7, 6):
        poison = torch.full((T, N), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
        del poison
        pme.set_gemm_tile(tile)
        try:
            acc = pme.w4a4_gemm_i32(qd, wd).cpu().numpy()
        finally:
            pme.set_gemm_tile(0)
        assert np.array_equal(acc, acc_ref), f"tile {tile}: {np.count_nonzero(acc != acc_ref)} accumulators differ"


@pytest.mark.parametrize("tile", (9, 11, 13, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28))
def test_gemm_asymmetric_on_the_default_tiles(tile):
    # the asymmetric epilogue (zero points, weight row sums) on the tiles the automatic choice uses,
    # K split included; 4.5 K steps of 128 bytes, ragged T and N
    rng = np.random.default_rng(tile)
    T, N, d_e = 300, 520, 1152
    q = rng.integers(0, 16, size=(T, d_e), dtype=np.uint8)
    z = rng.integers(0, 16, size=T).astype(np.int32)
    qw = rng.integers(-8, 8, size=(N, d_e), dtype=np.int8)
    sx = rng.uniform(0.01, 2.0, T).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    y_ref = oracle.dequant_asym_bf16(oracle.int_gemm(q, qw), sx, z, qw, sw)
    wd = torch.from_numpy(oracle.pack_int4(qw)).cuda()
    wsum = pme.weight_rowsum(wd)
    pme.set_path(MFMA)
    pme.set_gemm_tile(tile)
    try:
        y = pme.w4a4_gemm_asym(torch.from_numpy(oracle.pack_int4(q)).cuda(), torch.from_numpy(sx).cuda(),
                               torch.from_numpy(z).cuda(), wd, torch.from_numpy(sw).cuda(), wsum)
    finally:
        pme.set_gemm_tile(0)
    check_bf16(y.to(torch.float32).cpu().numpy(), y_ref)


@pytest.mark.parametrize("T", (150, 8, 40))
@pytest.mark.parametrize("path", (GENERIC, MFMA))
def test_gemm_asymmetric(path, T):
    rng = np.random.default_rng(8)
    N, d_e = 260, 384
    q = rng.integers(0, 16, size=(T, d_e), dtype=np.uint8)
    z = rng.integers(0, 16, size=T).astype(np.int32)
    qw = rng.integers(-8, 8, size=(N, d_e), dtype=np.int8)
    sx = rng.uniform(0.01, 2.0, T).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    y_ref = oracle.dequant_asym_bf16(oracle.int_gemm(q, qw), sx, z, qw, sw)
    pme.set_path(path)
    wd = torch.from_numpy(oracle.pack_int4(qw)).cuda()
    wsum = pme.weight_rowsum(wd)
    assert np.array_equal(wsum.cpu().numpy(), qw.astype(np.int64).sum(axis=1))
    y = pme.w4a4_gemm_asym(torch.from_numpy(oracle.pack_int4(q)).cuda(), torch.from_numpy(sx).cuda(),
                           torch.from_numpy(z).cuda(), wd, torch.from_numpy(sw).cuda(), wsum)
    check_bf16(y.to(torch.float32).cpu().numpy(), y_ref)


LAYER_CASES = [("C1", None), ("mid_b68_k5", (300, 2048, 2176, 520)), ("mid_b132_k6", (8, 8192, 8448, 2048)),
               ("mid_b60_k8", (130, 14336, 15360, 260)),
               # decode: at most 16 tokens through the fused call (weight-streaming GEMM)
               ("decode_b68_k7", (16, 8192, 8704, 530)), ("decode_b60_k8_one_token", (1, 14336, 15360, 300)),
               ("decode_b132_k5", (5, 4096, 4224, 200)), ("decode_folded_b20_k9", (3, 8192, 10240, 100)),
               ("decode_folded_b12_k10", (4, 8192, 12288, 64)), ("decode_b152_k6_ragged_d", (9, 8000, 9728, 1000))]


@pytest.mark.parametrize("name,shape", LAYER_CASES, ids=[c[0] for c in LAYER_CASES])
def test_expanded_linear_end_to_end(name, shape):
    if shape is None:
        wl = make_workload("C1")
    else:
        T, d, d_e, N = shape
        wl = make_workload(custom_spec(T, d, d_e, N, act_dist="student_t3", outlier_frac=0.005,
                                       outlier_gain=100.0, seed=1))
    sp = wl.spec
    ref = oracle.expanded_linear(wl.x, sp.d_e, wl.qw, wl.sw)
    xd = to_device(wl.x, sp.in_dtype)
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
    assert np.array_equal(wd.cpu().numpy(), oracle.pack_int4(wl.qw))
    swd = torch.from_numpy(wl.sw).cuda()
    y = pme.expanded_linear(xd, sp.d_e, wd, swd).to(torch.float32).cpu().numpy()
    # stage by stage with the library's own codes: the fused call must equal the chain of its parts
    qx, sx = pme.hadamard_expand_quant(xd, sp.d_e)
    q_gpu = unpack_gpu(qx)
    nflip = check_codes(q_gpu, ref["qx"], ref["xhat"], ref["sx"])
    check_scales(sx.cpu().numpy(), ref["sx"])
    y_chain = oracle.dequant_bf16(oracle.int_gemm(q_gpu, wl.qw), sx.cpu().numpy(), wl.sw)
    check_bf16(y, y_chain)
    y2 = pme.w4a4_gemm(qx, sx, wd, swd).to(torch.float32).cpu().numpy()
    assert np.array_equal(y, y2)
    # against the oracle's own end-to-end output: tokens whose codes all agree meet the bf16 bound outright
    same = np.all(q_gpu == ref["qx"], axis=1) & (sx.cpu().numpy() == ref["sx"])
    if same.any():
        check_bf16(y[same], ref["y"][same])
    assert np.linalg.norm(y - ref["y"]) <= 2e-3 * np.linalg.norm(ref["y"])
    assert nflip <= max(1, int(1e-4 * q_gpu.size))


@pytest.mark.parametrize("shape", ((300, 2048, 2176, 520), (8, 8192, 8448, 2048), (130, 14336, 15360, 260)))
def test_expanded_linear_asymmetric_end_to_end(shape):
    # the paper's own activation quantizer (per-token asymmetric int4) through the fused call
    T, d, d_e, N = shape
    wl = make_workload(custom_spec(T, d, d_e, N, act_dist="student_t3", outlier_frac=0.005, outlier_gain=100.0, seed=2))
    x = wl.x + np.float32(0.125)                  # an offset, so that the zero points are not all mid-range
    x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    ref = oracle.expanded_linear(x, d_e, wl.qw, wl.sw, asymmetric=True)
    xd = to_device(x, "bf16")
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
    swd = torch.from_numpy(wl.sw).cuda()
    wsum = pme.weight_rowsum(wd)
    y = pme.expanded_linear_asym(xd, d_e, wd, swd, wsum)
    # the fused call equals the chain of its parts, bit for bit
    qx, sx, zx = pme.hadamard_expand_quant_asym(xd, d_e)
    y2 = pme.w4a4_gemm_asym(qx, sx, zx, wd, swd, wsum)
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    # and the chain evaluated by the oracle on the library's codes
    q_gpu = unpack_gpu(qx, signed=False)
    y_chain = oracle.dequant_asym_bf16(oracle.int_gemm(q_gpu, wl.qw), sx.cpu().numpy(), zx.cpu().numpy(), wl.qw, wl.sw)
    check_bf16(y.to(torch.float32).cpu().numpy(), y_chain)
    same = np.all(q_gpu == ref["qx"], axis=1) & (sx.cpu().numpy() == ref["sx"]) & (zx.cpu().numpy() == ref["zx"])
    if same.any():
        check_bf16(y.to(torch.float32).cpu().numpy()[same], ref["y"][same])
    yf = y.to(torch.float32).cpu().numpy()
    assert np.linalg.norm(yf - ref["y"]) <= 2e-3 * np.linalg.norm(ref["y"])


@pytest.mark.parametrize("d,d_e,N,dtype", ((64, 80, 48, "f32"), (2048, 2176, 300, "f32"), (8192, 8704, 130, "bf16")))
def test_offline_weight_expansion_and_whole_layer_from_real_weights(d, d_e, N, dtype):
    # W_hat = H_hat^T W then per-channel round-to-nearest int4 (Sections 3 and 4), on the GPU, against the
    # oracle; then the whole quantized layer built from those weights tracks the unquantized X W.
    rng = np.random.default_rng(d + N)
    W = (rng.standard_normal((d, N)) / np.sqrt(d)).astype(np.float32)
    if dtype == "bf16":
        W = torch.from_numpy(W).to(torch.bfloat16).to(torch.float32).numpy()
    What = oracle.expand_weight(W, d_e)
    q_ref, s_ref = oracle.quantize_weight_rtn(What)
    wt = to_device(np.ascontiguousarray(W.T), dtype)
    qw, sw = pme.expand_quantize_weights(wt, d_e)
    check_scales(sw.cpu().numpy(), s_ref)
    check_codes(unpack_gpu(qw), q_ref, What.T, s_ref)
    T = 24
    x = _acts(T, d, d_e, dtype, seed=9)
    y = pme.expanded_linear(to_device(x, dtype), d_e, qw, sw).to(torch.float32).cpu().numpy()
    ref = x.astype(np.float64) @ W.astype(np.float64)
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) < 0.25
    y_or = oracle.expanded_linear(x, d_e, unpack_gpu(qw), sw.cpu().numpy())["y"]
    assert np.linalg.norm(y - y_or) <= 2e-3 * np.linalg.norm(y_or)


def test_run_twice_is_bit_identical():
    wl = make_workload(custom_spec(257, 2048, 2176, 384, seed=4))
    xd = to_device(wl.x, "bf16")
    wd = pme.pack_int4(torch.from_numpy(wl.qw))
    swd = torch.from_numpy(wl.sw).cuda()
    outs = []
    for _ in range(2):
        qx, sx = pme.hadamard_expand_quant(xd, 2176)
        acc = pme.w4a4_gemm_i32(qx, wd)
        y = pme.expanded_linear(xd, 2176, wd, swd)
        torch.cuda.synchronize()
        outs.append((qx.clone(), sx.clone(), acc.clone(), y.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_empty_inputs_are_no_ops():
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    qx, sx = pme.hadamard_expand_quant(x, 80)
    assert qx.shape == (0, 40) and sx.shape == (0,)
    qw = torch.zeros((0, 40), dtype=torch.uint8, device="cuda")
    y = pme.w4a4_gemm(qx, sx, qw, torch.zeros(0, device="cuda"))
    assert y.shape == (0, 0)


def test_forced_mfma_path_refuses_unsupported_shape():
    pme.set_path(MFMA)
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(pme.PmeError) as e:
        pme.hadamard_expand_quant(x, 80)      # 2^k = 4 is below the MFMA kernel's range
    assert e.value.status == 8
    q = torch.zeros((4, 40), dtype=torch.uint8, device="cuda")
    with pytest.raises(pme.PmeError):
        pme.w4a4_gemm_i32(q, q)               # d_e = 80 is not a multiple of 128


def test_pack_int4_matches_the_oracle_packing():
    rng = np.random.default_rng(9)
    for rows, K in ((1, 2), (7, 80), (300, 2176), (64, 15360)):
        codes = rng.integers(-8, 8, size=(rows, K), dtype=np.int8)
        got = pme.pack_int4(torch.from_numpy(codes)).cpu().numpy()
        assert np.array_equal(got, oracle.pack_int4(codes))
    assert pme.pack_int4(torch.zeros((0, 8), dtype=torch.int8)).shape == (0, 4)


@pytest.mark.parametrize("T,tile", ((8, 0), (40, 0), (70, 0), (300, 8), (300, 11), (300, 16), (300, 21)),
                         ids=("decode_kernel", "decode_kernel_three_groups", "auto_small_tile", "tile_256x256_64B", "tile_256x256_128B", "tile_128x256", "tile_128x192_loader"))
@pytest.mark.parametrize("d_e", ((1 << 17) - 128, 1 << 17), ids=("largest_matrix_core_d_e", "first_plain_alu_d_e"))
def test_gemm_extreme_codes_either_side_of_the_accumulator_bound(T, tile, d_e):
    """Every code -8 on both sides gives the largest sum, 64 d_e.  The matrix-core kernels hold 256 x the sum in
    int32: 2^31 - 2^23 at d_e = 2^17 - 128, and 2^31 (a wrap) at d_e = 2^17, which therefore runs on the plain-ALU
    kernel.  Asymmetric extremes (codes 15 with zero point 0, codes 0 with zero point 15, weights -8) reach
    -+120 d_e after the zero-point correction, which is formed after the factor 256 has been removed.
    Expected sums are the closed forms; the oracle supplies the epilogue."""
    N = 272
    big = d_e >= 1 << 17
    if big and tile:
        pytest.skip("the plain-ALU kernel has no tile table")
    pme.set_gemm_tile(tile)
    assert pme.gemm_plan(T, d_e, N).startswith("k_gemm_generic" if big else ("k_gemm_decode" if T <= 64 else "k_gemm_mfma"))
    qx = torch.full((T, d_e // 2), 0x88, dtype=torch.uint8, device="cuda")
    qw = torch.full((N, d_e // 2), 0x88, dtype=torch.uint8, device="cuda")
    qx[1] = 0x77                                   # one token of all +7: the most negative sum, -56 d_e
    acc = pme.w4a4_gemm_i32(qx, qw).cpu().numpy()
    want = np.full((T, N), 64 * d_e, dtype=np.int64)
    want[1] = -56 * d_e
    assert np.array_equal(acc, want)
    sx = torch.linspace(0.5, 1.5, T, device="cuda")
    sw = torch.linspace(1e-3, 2e-3, N, device="cuda")
    y = pme.w4a4_gemm(qx, sx, qw, sw).to(torch.float32).cpu().numpy()
    check_bf16(y, oracle.dequant_bf16(want, sx.cpu().numpy(), sw.cpu().numpy()))
    # asymmetric: unsigned codes 15 with zero point 0 (even tokens) and codes 0 with zero point 15 (odd tokens)
    qa = torch.full((T, d_e // 2), 0xFF, dtype=torch.uint8, device="cuda")
    qa[1::2] = 0
    zx = torch.zeros(T, dtype=torch.int32, device="cuda")
    zx[1::2] = 15
    wsum = pme.weight_rowsum(qw)
    assert np.array_equal(wsum.cpu().numpy(), np.full(N, -8 * d_e))
    ya = pme.w4a4_gemm_asym(qa, sx, zx, qw, sw, wsum).to(torch.float32).cpu().numpy()
    corr = np.full((T, N), -120 * d_e, dtype=np.int64)          # sum_j (15 - 0) (-8)
    corr[1::2] = 120 * d_e                                        # sum_j (0 - 15) (-8)
    check_bf16(ya, oracle.dequant_bf16(corr, sx.cpu().numpy(), sw.cpu().numpy()))


def test_plain_alu_gemm_beyond_a_million_tokens():
    """The plain-ALU kernels put blocks of 16 tokens on the grid's y axis, which ends at 65535: more tokens are
    walked by the same workgroups.  Sampled rows around that boundary and at both ends, int4 and MXFP4."""
    T, d_e, N = 65535 * 16 + 40, 64, 24
    rng = np.random.default_rng(12)
    g = torch.Generator(device="cuda").manual_seed(12)
    qx = torch.randint(0, 256, (T, d_e // 2), dtype=torch.uint8, device="cuda", generator=g)
    qw = torch.randint(0, 256, (N, d_e // 2), dtype=torch.uint8, device="cuda", generator=g)
    rows = np.unique(np.concatenate([[0, 1, 65535 * 16 - 1, 65535 * 16, 65535 * 16 + 17, T - 1], rng.choice(T, 50, replace=False)]))
    idx = torch.from_numpy(rows).cuda()
    assert pme.gemm_plan(T, d_e, N) == "k_gemm_generic"
    acc = pme.w4a4_gemm_i32(qx, qw)
    assert np.array_equal(acc[idx].cpu().numpy(), oracle.int_gemm(unpack_gpu(qx[idx]), unpack_gpu(qw)))
    ex = torch.randint(120, 130, (T, d_e // 32), dtype=torch.uint8, device="cuda", generator=g)
    ew = torch.randint(120, 130, (N, d_e // 32), dtype=torch.uint8, device="cuda", generator=g)
    assert pme.gemm_plan(T, d_e, N, variant=2) == "k_mxgemm_generic"
    y = pme.mxfp4_gemm(qx, ex, qw, ew)
    y_ref, abs_sum = oracle.gemm_mxfp4(oracle.unpack_fp4(qx[idx].cpu().numpy()), ex[idx].cpu().numpy(),
                                       oracle.unpack_fp4(qw.cpu().numpy()), ew.cpu().numpy(), return_abs=True)
    err = np.abs(y[idx].to(torch.float32).cpu().numpy().astype(np.float64) - y_ref)
    assert np.all(err <= 1e-2 * np.abs(y_ref) + 2.0 ** -18 * abs_sum)


def test_fused_layer_refused_by_a_forced_path_launches_nothing():
    """Under the forced matrix-core path the rotation takes this shape but the GEMM does not (its weight rows are
    only 4-byte aligned): the fused call must return the status without having run the rotation."""
    T, d, d_e, N = 40, 2048, 2176, 64
    x = torch.randn((T, d), device="cuda").to(torch.bfloat16)
    store = torch.zeros((N * (d_e // 2) + 16,), dtype=torch.uint8, device="cuda")
    qw = store[4:4 + N * (d_e // 2)].view(N, d_e // 2)
    assert qw.data_ptr() % 16 == 4
    sw = torch.ones(N, device="cuda")
    ws = torch.full((pme.workspace_bytes(T, d, d_e, N),), 0xA5, dtype=torch.uint8, device="cuda")
    y = torch.full((T, N), 3.0, dtype=torch.bfloat16, device="cuda")
    wsum = torch.zeros(N, dtype=torch.int32, device="cuda")
    pme.set_path(MFMA)
    for call in (lambda: pme.expanded_linear(x, d_e, qw, sw, y, ws),
                 lambda: pme.expanded_linear_asym(x, d_e, qw, sw, wsum, y, ws),
                 lambda: pme.expanded_linear_mxfp4(x, d_e, qw, torch.zeros((N, d_e // 32), dtype=torch.uint8, device="cuda"), y, ws)):
        with pytest.raises(pme.PmeError) as e:
            call()
        assert e.value.status == 8
    torch.cuda.synchronize()
    assert bool((ws == 0xA5).all()) and bool((y == 3.0).all())
    pme.set_path(pme.PATH_AUTO)                     # the automatic path serves the same call on the plain-ALU GEMM
    pme.expanded_linear(x, d_e, qw, sw, y, ws)
    torch.cuda.synchronize()
    assert not bool((ws == 0xA5).all())


_POOL_SCRIPT = """
import sys, torch
sys.path.insert(0, sys.argv[1])
import paper_2503_17513_amd as pme
torch.manual_seed(0)
x = torch.randn(2, 152 * 64, device="cuda").to(torch.bfloat16)
pme.set_path(pme.PATH_MFMA)
first = pme.hadamard_expand_quant(x[:, :64].contiguous(), 9728)
served, refused = 0, None
for d_e, b in ((9728, 152), (8960, 140)):          # every count of real base rows is a table of its own
    for rows in range(1, b + 1):
        try:
            pme.hadamard_expand_quant(x[:, :64 * rows].contiguous(), d_e)
            served += 1
        except pme.PmeError as e:
            assert e.status == 8, e.status
            refused = (64 * rows, d_e)
            break
    if refused:
        break
assert refused is not None and served > 200, (served, refused)
xs = x[:, :refused[0]].contiguous()
pme.set_path(pme.PATH_AUTO)
qa, sa = pme.hadamard_expand_quant(xs, refused[1])
pme.set_path(pme.PATH_GENERIC)
qg, sg = pme.hadamard_expand_quant(xs, refused[1])
assert torch.equal(qa, qg) and torch.equal(sa, sg)
pme.set_path(pme.PATH_MFMA)                          # tables handed out earlier keep working
again = pme.hadamard_expand_quant(x[:, :64].contiguous(), 9728)
torch.cuda.synchronize()
assert torch.equal(again[0], first[0]) and torch.equal(again[1], first[1])
print("POOL_OK", served)
"""


def test_fragment_pool_exhaustion_falls_back_to_the_generic_kernel():
    # in a process of its own: the pool is never given back, and the other tests need it
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", _POOL_SCRIPT, root], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "POOL_OK" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


def test_decode_layer_calls_sharing_a_workspace():
    # back-to-back decode calls with changing token counts on one workspace: each equals the chain of its parts
    d, d_e, N = 8192, 8448, 1000
    wl = make_workload(custom_spec(16, d, d_e, N, act_dist="student_t3", seed=9))
    x = torch.from_numpy(wl.x).to(torch.bfloat16).cuda()
    qw = pme.pack_int4(torch.from_numpy(wl.qw))
    sw = torch.from_numpy(wl.sw).cuda()
    ws = torch.empty((pme.workspace_bytes(16, d, d_e, N),), dtype=torch.uint8, device="cuda")
    for T in (16, 3, 16, 1, 8, 8):
        xt = x[:T].contiguous()
        y = torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        pme.expanded_linear(xt, d_e, qw, sw, y, ws)
        qx, sx = pme.hadamard_expand_quant(xt, d_e)
        y_parts = pme.w4a4_gemm(qx, sx, qw, sw)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_parts.view(torch.int16)), f"T = {T}"


@pytest.mark.parametrize("shape", ((300, 2048, 2176, 520), (8, 8192, 8448, 2048)), ids=("prefill", "decode"))
def test_layer_in_a_hip_graph_replays_identically(shape):
    # the library only enqueues kernels (no memset nodes, no allocation, no synchronisation once a shape is
    # warm), so a captured layer call must give the eager result on every replay, with eager work between
    T, d, d_e, N = shape
    wl = make_workload(custom_spec(T, d, d_e, N, seed=5))
    x = torch.from_numpy(wl.x).to(torch.bfloat16).cuda()
    qw = pme.pack_int4(torch.from_numpy(wl.qw))
    sw = torch.from_numpy(wl.sw).cuda()
    ws = torch.empty((pme.workspace_bytes(T, d, d_e, N),), dtype=torch.uint8, device="cuda")
    y_eager = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda")
    pme.expanded_linear(x, d_e, qw, sw, y_eager, ws)                 # also warms the shape (and this workspace)
    y = torch.zeros_like(y_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        pme.expanded_linear(x, d_e, qw, sw, y, ws)
    for rep in range(4):
        y.fill_(float("nan"))                                        # eager work on the outputs between replays
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_eager.view(torch.int16)), f"replay {rep} differs from the eager result"


def test_first_use_of_a_shape_under_graph_capture_is_refused_and_the_capture_survives():
    """The first rotation of a shape fills its base-block table and waits for it once; on a capturing stream that
    wait would break the capture, so the call returns PME_ERR_COLD_SHAPE with nothing enqueued.  After one call
    outside a capture the same call is captured and replays with identical results."""
    d, d_e, T = 8000, 8960, 6                       # 125 real base rows of the order-140 block: no other test uses it
    x = (torch.randn((T, d), device="cuda") * 3).to(torch.bfloat16)
    qx = torch.zeros((T, d_e // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((T,), dtype=torch.float32, device="cuda")
    marker = torch.zeros(8, device="cuda")
    pme.set_path(MFMA)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    status = None
    with torch.cuda.graph(g, stream=side):
        marker.add_(1.0)
        try:
            pme.hadamard_expand_quant(x, d_e, qx, sx)
        except pme.PmeError as e:
            status = e.status
    assert status == 9
    g.replay()
    torch.cuda.synchronize()
    assert float(marker[0]) == 1.0 and int(qx.max()) == 0          # the captured work ran, the refused call left no trace
    pme.hadamard_expand_quant(x, d_e, qx, sx)                       # outside a capture: fills the table
    torch.cuda.synchronize()
    want_q, want_s = qx.clone(), sx.clone()
    ref_x = oracle.rotate_structured(x.to(torch.float32).cpu().numpy(), d_e)
    q_ref, s_ref = oracle.quantize_sym_int4(ref_x)
    check_scales(want_s.cpu().numpy(), s_ref)
    check_codes(unpack_gpu(want_q), q_ref, ref_x, s_ref)
    qx.zero_()
    sx.zero_()
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2, stream=side):
        pme.hadamard_expand_quant(x, d_e, qx, sx)
    g2.replay()
    torch.cuda.synchronize()
    assert torch.equal(qx, want_q) and torch.equal(sx, want_s)


def test_probe_mfma():
    # every accumulator grows by the same amount per instruction: the checksum is linear in iters
    out = torch.zeros(512 * 256, dtype=torch.int32, device="cuda")
    assert pme.probe_mfma(0, out, 10) == 512 * 16 * 10 * 65536.0
    one = out.clone()
    assert pme.probe_mfma(0, out, 30) == 512 * 16 * 30 * 65536.0
    assert one.abs().sum().item() > 0 and torch.equal(out, 3 * one)
    assert pme.probe_mfma(1, out, 10) == 512 * 16 * 10 * 131072.0
    f10 = out.view(torch.float32).clone()
    pme.probe_mfma(1, out, 20)
    assert f10.abs().sum().item() > 0 and torch.equal(out.view(torch.float32), 2 * f10)


def test_probe_mfma_on_random_codes():
    out = torch.zeros(512 * 256, dtype=torch.int32, device="cuda")
    assert pme.probe_mfma(2, out, 8) == 512 * 16 * 8 * 65536.0
    # the operand sets rotate with a period of four iterations: equal runs of 8 iterations add equal sums
    one = out.clone()
    pme.probe_mfma(2, out, 24)
    assert one.abs().sum().item() > 0 and torch.equal(out, 3 * one)
    assert pme.probe_mfma(3, out, 8) == 512 * 16 * 8 * 131072.0
    assert torch.isfinite(out.view(torch.float32)).all()


def test_probe_copy():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    pme.probe_copy(src, dst)
    assert torch.equal(src, dst)
