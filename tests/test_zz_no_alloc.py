"""The entry point that allocates nothing (pme_expanded_linear_static) against pme_expanded_linear: same
outputs bit for bit, on two calls in a row that share the library's static scratch, the second one smaller."""
import numpy as np
import pytest
import torch

import paper_2503_17513_amd as pme
from parity_util import to_device
from workloads import custom_spec, make_workload

pytestmark = pytest.mark.gpu


def _operands(T, d, d_e, N, seed):
    wl = make_workload(custom_spec(T, d, d_e, N, act_dist="student_t3", outlier_frac=0.005, outlier_gain=100.0, seed=seed))
    return to_device(wl.x, "bf16"), pme.pack_int4(torch.from_numpy(wl.qw)), torch.from_numpy(wl.sw).cuda()


def test_static_scratch_layer_equals_the_workspace_layer_on_two_calls_in_a_row():
    assert pme.get_path() == pme.PATH_AUTO
    shapes = ((700, 2048, 2176, 520, 21), (9, 8192, 8448, 2048, 22))      # the second input is the smaller one
    ops = [_operands(*s) for s in shapes]
    want = []
    for (T, d, d_e, N, _), (x, qw, sw) in zip(shapes, ops):
        want.append(pme.expanded_linear(x, d_e, qw, sw))
    torch.cuda.synchronize()
    got = [torch.full((s[0], s[3]), float("nan"), dtype=torch.bfloat16, device="cuda") for s in shapes]
    # set-up: the first call on a device resolves the static array's address (the runtime places the array then)
    pme.expanded_linear_static(ops[1][0], shapes[1][2], ops[1][1], ops[1][2], got[1])
    torch.cuda.synchronize()
    got[1].fill_(float("nan"))
    free_before = torch.cuda.mem_get_info()[0]
    for (T, d, d_e, N, _), (x, qw, sw), y in zip(shapes, ops, got):       # back to back on one stream, no sync between
        pme.expanded_linear_static(x, d_e, qw, sw, y)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before                   # the calls took and gave back no device memory
    for w, g in zip(want, got):
        assert torch.equal(w.view(torch.int16), g.view(torch.int16))
    # once more in the other order: the large call runs over what the small one left in the scratch
    for i in (1, 0):
        T, d, d_e, N, _ = shapes[i]
        got[i].fill_(float("nan"))
        pme.expanded_linear_static(ops[i][0], d_e, ops[i][1], ops[i][2], got[i])
    torch.cuda.synchronize()
    for w, g in zip(want, got):
        assert torch.equal(w.view(torch.int16), g.view(torch.int16))


def test_static_scratch_layer_rejects_sizes_beyond_its_maximum():
    T, d, d_e, N = 4096, 14336, 15360, 64
    assert pme.workspace_bytes(T, d, d_e, N) > pme.STATIC_SCRATCH_BYTES
    x = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    qw = torch.zeros((N, d_e // 2), dtype=torch.uint8, device="cuda")
    sw = torch.ones(N, device="cuda")
    y = torch.full((T, N), 2.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pme.PmeError) as e:
        pme.expanded_linear_static(x, d_e, qw, sw, y)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((y == 2.0).all())
    # the largest token count that fits is accepted
    T_fit = (pme.STATIC_SCRATCH_BYTES - 512) // (d_e // 2 + 4) // 256 * 256
    assert pme.workspace_bytes(T_fit, d, d_e, N) <= pme.STATIC_SCRATCH_BYTES < pme.workspace_bytes(T_fit + 512, d, d_e, N)
    pme.expanded_linear_static(x[:T_fit], d_e, qw, sw, y[:T_fit])
    torch.cuda.synchronize()
    assert bool((y[:T_fit] == 0.0).all()) and bool((y[T_fit:] == 2.0).all())
