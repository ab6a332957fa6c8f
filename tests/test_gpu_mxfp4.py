"""GPU parity of the MXFP4 path (paper Section 4, second quantization setting) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_17513_amd as pme
from parity_util import check_mx_gemm, check_mx_quant, to_device
from workloads import custom_spec, make_workload

pytestmark = pytest.mark.gpu
GENERIC, MFMA = pme.PATH_GENERIC, pme.PATH_MFMA


@pytest.fixture(autouse=True)
def _reset():
    yield
    pme.set_path(pme.PATH_AUTO)
    pme.set_gemm_tile(0)


def _acts(T, d, d_e, in_dtype="bf16", seed=0):
    spec = custom_spec(T, d, d_e, 8, in_dtype=in_dtype, act_dist="student_t3", outlier_frac=0.01, outlier_gain=50.0, seed=seed)
    return make_workload(spec, weights=False).x


QUANT_CASES = [
    ("b12_k3_generic", 9, 80, 96, "f32", (GENERIC,)),
    ("b68_k5", 21, 2048, 2176, "bf16", (GENERIC, MFMA)),
    ("b132_k6", 8, 8192, 8448, "bf16", (GENERIC, MFMA)),
    ("b68_k7", 9, 8192, 8704, "bf16", (GENERIC, MFMA)),
    ("b60_k8", 5, 14336, 15360, "bf16", (GENERIC, MFMA)),
    ("b20_k9", 3, 8192, 10240, "bf16", (GENERIC, MFMA)),
    ("f32_b68_k5", 6, 2048, 2176, "f32", (GENERIC, MFMA)),
    ("many_tokens_k7", 530, 8192, 8704, "bf16", (MFMA,)),
    ("b68_k5_token_per_wave", 1029, 2048, 2176, "bf16", (MFMA,)),
    ("b12_k10_folded", 5, 8192, 12288, "bf16", (GENERIC, MFMA)),
    ("b312_k6", 5, 14336, 19968, "bf16", (GENERIC, MFMA)),
]


@pytest.mark.parametrize("name,T,d,d_e,in_dtype,paths", QUANT_CASES, ids=[c[0] for c in QUANT_CASES])
def test_rotate_and_quantize_mxfp4(name, T, d, d_e, in_dtype, paths):
    x = _acts(T, d, d_e, in_dtype, seed=len(name))
    if T > 2:
        x[1] = 0.0
        x[2] = 0.0
        x[2, d // 3] = 1.0
    xd = to_device(x, in_dtype)
    ref = oracle.rotate_structured(x, d_e)
    for path in paths:
        pme.set_path(path)
        qx, ex = pme.hadamard_expand_quant_mxfp4(xd, d_e)
        torch.cuda.synchronize()
        check_mx_quant(qx, ex, ref)
        if T > 2:
            assert int(ex[1].max()) == 0 and int(qx[1].max()) == 0     # all-zero token: smallest scale, zero codes


def test_mxfp4_rejects_d_e_not_multiple_of_32():
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(pme.PmeError) as e:
        pme.hadamard_expand_quant_mxfp4(x, 80)
    assert e.value.status == 2


GEMM_CASES = [("small_ragged", 50, 70, 96, (GENERIC,)), ("one_k_step", 40, 72, 128, (GENERIC, MFMA)),
              ("ragged_tiles", 300, 200, 2176, (GENERIC, MFMA)), ("wide_rows", 260, 520, 1280, (GENERIC, MFMA)),
              ("c2_shape_rows", 2048, 384, 2176, (MFMA,)), ("big_tile", 1024, 4096, 512, (MFMA,)),
              # at most 32 tokens: the weight-streaming kernel, 1 or 2 groups of 16 tokens; beyond: tiles
              ("decode_shape", 8, 2048, 8448, (GENERIC, MFMA)), ("decode_one_token_one_chunk", 1, 24, 128, (GENERIC, MFMA)),
              ("decode_16_ragged_n", 16, 100, 384, (GENERIC, MFMA)), ("decode_33_odd_chunks", 33, 40, 640, (GENERIC, MFMA)),
              ("decode_48", 48, 72, 1280, (MFMA,)), ("decode_64", 64, 130, 2176, (GENERIC, MFMA)),
              ("sixty_five_tokens_tiled", 65, 72, 256, (MFMA,))]


@pytest.mark.parametrize("name,T,N,d_e,paths", GEMM_CASES, ids=[c[0] for c in GEMM_CASES])
def test_mxfp4_gemm(name, T, N, d_e, paths):
    rng = np.random.default_rng(T + N)
    qx = rng.integers(0, 16, size=(T, d_e), dtype=np.uint8)
    qw = rng.integers(0, 16, size=(N, d_e), dtype=np.uint8)
    ex = rng.integers(118, 132, size=(T, d_e // 32), dtype=np.uint8)
    ew = rng.integers(118, 130, size=(N, d_e // 32), dtype=np.uint8)
    args = [torch.from_numpy(a).cuda() for a in (oracle.pack_fp4(qx), ex, oracle.pack_fp4(qw), ew)]
    for path in paths:
        pme.set_path(path)
        y = pme.mxfp4_gemm(*args).to(torch.float32).cpu().numpy()
        check_mx_gemm(y, qx, ex, qw, ew)


@pytest.mark.parametrize("tile", range(1, 12))
def test_mxfp4_gemm_every_tile(tile):
    rng = np.random.default_rng(tile)
    T, N, d_e = 300, 520, 1280
    qx = rng.integers(0, 16, size=(T, d_e), dtype=np.uint8)
    qw = rng.integers(0, 16, size=(N, d_e), dtype=np.uint8)
    ex = rng.integers(120, 130, size=(T, d_e // 32), dtype=np.uint8)
    ew = rng.integers(120, 130, size=(N, d_e // 32), dtype=np.uint8)
    args = [torch.from_numpy(a).cuda() for a in (oracle.pack_fp4(qx), ex, oracle.pack_fp4(qw), ew)]
    pme.set_path(MFMA)
    pme.set_gemm_tile(100 + tile)
    y = pme.mxfp4_gemm(*args).to(torch.float32).cpu().numpy()
    check_mx_gemm(y, qx, ex, qw, ew)


@pytest.mark.parametrize("shape", ((40, 2048, 2176, 200), (130, 8192, 8704, 300)))
def test_mxfp4_layer_end_to_end(shape):
    T, d, d_e, N = shape
    rng = np.random.default_rng(5)
    x = _acts(T, d, d_e, "bf16", seed=2)
    W = (rng.standard_normal((d, N)) / np.sqrt(d)).astype(np.float32)
    xd = to_device(x, "bf16")
    wt = torch.from_numpy(np.ascontiguousarray(W.T)).cuda()
    qw, ew = pme.hadamard_expand_quant_mxfp4(wt, d_e)          # offline weight side: rows of W^T
    check_mx_quant(qw, ew, oracle.expand_weight(W, d_e).T)
    y = pme.expanded_linear_mxfp4(xd, d_e, qw, ew).to(torch.float32).cpu().numpy()
    qx, ex = pme.hadamard_expand_quant_mxfp4(xd, d_e)
    check_mx_quant(qx, ex, oracle.rotate_structured(x, d_e))
    check_mx_gemm(y, oracle.unpack_fp4(qx.cpu().numpy()), ex.cpu().numpy(), oracle.unpack_fp4(qw.cpu().numpy()), ew.cpu().numpy())
    ref = x.astype(np.float64) @ W.astype(np.float64)
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) < 0.25
