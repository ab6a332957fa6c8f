"""Host-side tests of the C-ABI library that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments with the documented status before any HIP call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2503_17513_amd as pme

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, ORDER, ALIGN, WORKSPACE, DTYPE, HIP, PATH, COLD = range(10)
FAKE = 0x10000   # a non-null, 64 KiB aligned address that is never dereferenced: every call below fails validation


def test_header_symbols_are_exported():
    with open(os.path.join(ROOT, "include", "pme.h")) as f:
        text = f.read()
    declared = set(re.findall(r"\b(pme_[a-z0-9_]+)\s*\(", text))
    assert declared == set(pme.EXPORTS)
    L = pme.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert pme.version() >= 100
    assert L.pme_status_string(OK) == b"ok"
    for s in range(1, 10):
        assert L.pme_status_string(s) not in (b"ok", b"unknown status")


def test_factor_order_matches_oracle():
    for M in (80, 2176, 8704, 8448, 15360, 64, 8960, 9728, 10240, 12288, 18432, 19968, 22016, 24, 40):
        assert pme.factor_order(M) == oracle.factor_order(M)
    for bad in (7, 100, 11264, 0, -4):
        with pytest.raises(pme.PmeError) as e:
            pme.factor_order(bad)
        assert e.value.status == ORDER


def test_base_block_matches_oracle():
    for b in oracle.SUPPORTED_BASE:
        assert np.array_equal(pme.base_block(b), oracle.paley_block(b))
    out = np.zeros((16, 16), np.int8)
    assert pme.lib().pme_base_block(16, out.ctypes.data) == ORDER
    assert pme.lib().pme_base_block(20, None) == NULL


def test_rotate_argument_errors():
    f = pme.lib().pme_hadamard_expand_quant
    good = dict(x=FAKE, xt=1, T=4, d=64, ldx=64, d_e=80, qx=FAKE, sx=FAKE, stream=None)

    def call(**kw):
        a = dict(good, **kw)
        return f(a["x"], a["xt"], a["T"], a["d"], a["ldx"], a["d_e"], a["qx"], a["sx"], a["stream"])

    assert call(x=None) == NULL
    assert call(qx=None) == NULL
    assert call(sx=None) == NULL
    assert call(xt=5) == DTYPE
    assert call(T=-1) == SHAPE
    assert call(d=0) == SHAPE
    assert call(d=81) == SHAPE            # d > d_e
    assert call(ldx=63) == SHAPE          # pitch smaller than d
    assert call(d_e=81, d=64) == SHAPE    # odd d_e
    assert call(d_e=100) == ORDER
    assert call(d_e=11264, d=64) == ORDER
    assert call(x=FAKE + 1) == ALIGN
    assert call(xt=0, x=FAKE + 2) == ALIGN
    assert call(qx=FAKE + 2) == ALIGN
    assert call(sx=FAKE + 2) == ALIGN
    assert call(T=0, x=None, qx=None, sx=None) == OK      # empty input: no-op


def test_gemm_argument_errors():
    f = pme.lib().pme_w4a4_gemm

    def call(qx=FAKE, sx=FAKE, qw=FAKE, sw=FAKE, T=4, d_e=80, N=8, y=FAKE, ldy=8):
        return f(qx, sx, qw, sw, T, d_e, N, y, ldy, None)

    assert call(qx=None) == NULL
    assert call(qw=None) == NULL
    assert call(sx=None) == NULL
    assert call(sw=None) == NULL
    assert call(y=None) == NULL
    assert call(T=-2) == SHAPE
    assert call(N=-1) == SHAPE
    assert call(d_e=0) == SHAPE
    assert call(d_e=81) == SHAPE
    assert call(ldy=7) == SHAPE
    assert call(qx=FAKE + 1) == ALIGN
    assert call(qw=FAKE + 3) == ALIGN
    assert call(y=FAKE + 1) == ALIGN
    assert call(T=0) == OK
    assert call(N=0, ldy=0) == OK
    g = pme.lib().pme_w4a4_gemm_i32
    assert g(FAKE, FAKE, 4, 80, 8, None, None) == NULL
    assert g(FAKE, FAKE, 4, 81, 8, FAKE, None) == SHAPE


def test_expanded_linear_argument_errors():
    f = pme.lib().pme_expanded_linear
    need = pme.workspace_bytes(4, 64, 80, 8)
    assert need == 256 + 256 + 256
    # codes + MXFP4 scale bytes (the larger of the two scale kinds) + zero points of the asymmetric variant
    assert pme.workspace_bytes(2048, 2048, 2176, 3072) == 2048 * 1088 + 2048 * 68 + 2048 * 4
    assert pme.workspace_bytes(4, 81, 80, 8) == 0

    def call(x=FAKE, xt=1, T=4, d=64, ldx=64, d_e=80, qw=FAKE, sw=FAKE, N=8, y=FAKE, ldy=8, ws=FAKE, wsb=need):
        return f(x, xt, T, d, ldx, d_e, qw, sw, N, y, ldy, ws, wsb, None)

    assert call(wsb=need - 1) == WORKSPACE
    assert call(ws=None) == NULL
    assert call(ws=FAKE + 64) == ALIGN
    assert call(qw=None) == NULL
    assert call(d_e=100) == ORDER
    assert call(xt=9) == DTYPE
    assert call(ldy=4) == SHAPE
    assert call(T=0, x=None, ws=None, wsb=0) == OK


def test_mxfp4_and_weight_argument_errors():
    L = pme.lib()
    f = L.pme_hadamard_expand_quant_mxfp4
    assert f(None, 1, 4, 64, 64, 96, FAKE, FAKE, None) == NULL
    assert f(FAKE, 1, 4, 64, 64, 96, None, FAKE, None) == NULL
    assert f(FAKE, 1, 4, 64, 64, 96, FAKE, None, None) == NULL
    assert f(FAKE, 1, 4, 64, 64, 80, FAKE, FAKE, None) == SHAPE           # d_e not a multiple of 32
    assert f(FAKE, 1, 4, 64, 64, 100, FAKE, FAKE, None) == ORDER
    assert f(FAKE, 3, 4, 64, 64, 96, FAKE, FAKE, None) == DTYPE
    assert f(None, 1, 0, 64, 64, 96, None, None, None) == OK
    g = L.pme_mxfp4_gemm
    assert g(None, FAKE, FAKE, FAKE, 4, 96, 8, FAKE, 8, None) == NULL
    assert g(FAKE, None, FAKE, FAKE, 4, 96, 8, FAKE, 8, None) == NULL
    assert g(FAKE, FAKE, FAKE, None, 4, 96, 8, FAKE, 8, None) == NULL
    assert g(FAKE, FAKE, FAKE, FAKE, 4, 80, 8, FAKE, 8, None) == SHAPE
    assert g(FAKE, FAKE, FAKE, FAKE, 4, 96, 8, FAKE, 7, None) == SHAPE
    assert g(FAKE + 1, FAKE, FAKE, FAKE, 4, 96, 8, FAKE, 8, None) == ALIGN
    assert g(FAKE, FAKE, FAKE, FAKE, 0, 96, 8, FAKE, 8, None) == OK
    h = L.pme_expanded_linear_mxfp4
    need = pme.workspace_bytes(4, 64, 96, 8)
    assert h(FAKE, 1, 4, 64, 64, 96, FAKE, FAKE, 8, FAKE, 8, FAKE, need - 1, None) == WORKSPACE
    assert h(FAKE, 1, 4, 64, 64, 96, FAKE, None, 8, FAKE, 8, FAKE, need, None) == NULL
    assert h(FAKE, 1, 4, 64, 64, 80, FAKE, FAKE, 8, FAKE, 8, FAKE, need, None) == SHAPE
    w = L.pme_expand_quantize_weights
    assert w(None, 0, 8, 64, 64, 80, FAKE, FAKE, None) == NULL
    assert w(FAKE, 0, 8, 64, 60, 80, FAKE, FAKE, None) == SHAPE
    r = L.pme_weight_rowsum
    assert r(None, 8, 80, FAKE, None) == NULL
    assert r(FAKE, 8, 81, FAKE, None) == SHAPE
    a = L.pme_w4a4_gemm_asym
    assert a(FAKE, FAKE, None, FAKE, FAKE, FAKE, 4, 80, 8, FAKE, 8, None) == NULL
    assert a(FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, 80, 8, FAKE, 8, None) == NULL
    q = L.pme_hadamard_expand_quant_asym
    assert q(FAKE, 1, 4, 64, 64, 80, FAKE, FAKE, None, None) == NULL


def test_expanded_linear_asym_argument_errors():
    f = pme.lib().pme_expanded_linear_asym
    need = pme.workspace_bytes(4, 64, 80, 8)

    def call(x=FAKE, xt=1, T=4, d=64, ldx=64, d_e=80, qw=FAKE, sw=FAKE, wsum=FAKE, N=8, y=FAKE, ldy=8, ws=FAKE, wsb=need):
        return f(x, xt, T, d, ldx, d_e, qw, sw, wsum, N, y, ldy, ws, wsb, None)

    assert call(wsum=None) == NULL
    assert call(wsum=FAKE + 2) == ALIGN
    assert call(wsb=need - 1) == WORKSPACE
    assert call(ws=FAKE + 128) == ALIGN
    assert call(d_e=11264) == ORDER
    assert call(ldy=7) == SHAPE
    assert call(T=0) == OK


def test_probe_copy_errors():
    f = pme.lib().pme_probe_copy
    assert f(None, FAKE, 16, None) == NULL
    assert f(FAKE, FAKE, 24, None) == SHAPE
    assert f(FAKE + 8, FAKE, 32, None) == ALIGN
    assert f(FAKE, FAKE, 0, None) == OK


def test_probe_mfma_errors():
    f = pme.lib().pme_probe_mfma
    n = 512 * 256
    assert f(0, None, n, 10, None, None) == NULL
    assert f(4, FAKE, n, 10, None, None) == DTYPE
    assert f(-1, FAKE, n, 10, None, None) == DTYPE
    assert f(0, FAKE, n - 1, 10, None, None) == SHAPE
    assert f(1, FAKE, n, -1, None, None) == SHAPE
    assert f(0, FAKE + 2, n, 10, None, None) == ALIGN


def test_binding_has_no_fallback():
    # The binding refuses host tensors instead of computing anything itself.
    import torch
    x = torch.zeros(2, 64)
    with pytest.raises(ValueError):
        pme.hadamard_expand_quant(x, 80)


def test_gemm_plan_names_the_kernel_without_launching():
    """pme_gemm_plan is a dry run of the dispatch: it needs no GPU and names the instantiation a profiler would print."""
    assert pme.gemm_plan(4096, 15360, 4096) == "k_gemm_mfma<256, 256, 2, 2, 128, 2, 0, 1, false>"
    assert pme.gemm_plan(4096, 15360, 4096, variant=1) == "k_gemm_mfma<256, 256, 2, 2, 128, 2, 1, 1, false>"
    assert pme.gemm_plan(2048, 2176, 3072) == "k_gemm_mfma<128, 192, 2, 2, 64, 3, 0, 1, true>"
    assert pme.gemm_plan(2048, 8704, 2048) == "k_gemm_mfma<128, 128, 2, 2, 128, 3, 0, 1, true>"
    assert pme.gemm_plan(8, 8448, 2048) == "k_gemm_decode"
    assert pme.gemm_plan(4096, 15360, 4096, variant=2).startswith("k_mxgemm_mfma<256, 256, ")
    assert pme.gemm_plan(8, 8448, 2048, variant=2) == "k_mxgemm_decode"
    assert pme.gemm_plan(16, 80, 64) == "k_gemm_generic"                 # d_e not a multiple of 128
    # the x256 accumulator of the matrix-core kernels: 256 * 64 * d_e < 2^31 holds below d_e = 2^17 only
    assert pme.gemm_plan(300, (1 << 17) - 128, 256).startswith("k_gemm_mfma<")
    assert pme.gemm_plan(300, 1 << 17, 256) == "k_gemm_generic"
    assert pme.gemm_plan(8, (1 << 17) - 128, 256) == "k_gemm_decode"
    assert pme.gemm_plan(8, 1 << 17, 256) == "k_gemm_generic"
    f = pme.lib().pme_gemm_plan
    buf = C.create_string_buffer(64)
    assert f(0, 8, 256, 8, None, 64) == NULL
    assert f(3, 8, 256, 8, buf, 64) == DTYPE
    assert f(0, 0, 256, 8, buf, 64) == SHAPE
    assert f(0, 8, 255, 8, buf, 64) == SHAPE
    assert f(2, 8, 80, 8, buf, 64) == SHAPE                              # MXFP4 needs whole blocks of 32
    try:
        pme.set_path(pme.PATH_MFMA)
        assert f(0, 16, 80, 64, buf, 64) == PATH                         # forced matrix-core path, shape it does not take
    finally:
        pme.set_path(pme.PATH_AUTO)


def test_pack_int4_argument_errors():
    f = pme.lib().pme_pack_int4
    assert f(None, 4, 8, FAKE, None) == NULL
    assert f(FAKE, 4, 8, None, None) == NULL
    assert f(FAKE, 4, 7, FAKE, None) == SHAPE
    assert f(FAKE, -1, 8, FAKE, None) == SHAPE
    assert f(None, 0, 8, None, None) == OK


def test_static_scratch_layer_argument_errors():
    """pme_expanded_linear_static validates like pme_expanded_linear and refuses, before any HIP call, a shape whose
    quantized activations do not fit its static scratch."""
    f = pme.lib().pme_expanded_linear_static

    def call(x=FAKE, xt=1, T=8, d=8192, ldx=8192, d_e=8448, qw=FAKE, sw=FAKE, N=2048, y=FAKE, ldy=2048):
        return f(x, xt, T, d, ldx, d_e, qw, sw, N, y, ldy, None)

    assert call(x=None) == NULL
    assert call(qw=None) == NULL
    assert call(y=None) == NULL
    assert call(ldy=2047) == SHAPE
    assert call(d_e=8450) == ORDER
    assert call(y=FAKE + 1) == ALIGN
    assert call(T=0, x=None) == OK
    # 4096 tokens of 15360 expanded features need 31.5 MB of codes: beyond the 16 MiB scratch
    assert pme.workspace_bytes(4096, 14336, 15360, 4096) > pme.STATIC_SCRATCH_BYTES
    assert call(T=4096, d=14336, ldx=14336, d_e=15360, N=4096, ldy=4096) == WORKSPACE
    assert pme.workspace_bytes(2048, 14336, 15360, 4096) <= pme.STATIC_SCRATCH_BYTES
