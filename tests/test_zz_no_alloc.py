"""psd_sync_fc_sfb_static (the entry point that allocates nothing) against psd_sync_fc_sfb with a
caller workspace: same kernels, same split, so the results must be identical bit for bit; two calls in a
row on the shared fixed array, the second with a smaller layer; and the host-side refusals."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import psd_oracle as orc
from paper_1512_06216_amd import binding as psd
from paper_1512_06216_amd import inputs

DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _layer_on_gpu(d, dtype):
    plan = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], d["P"])
    U, ldu, V, ldv = psd.alloc_factors(plan, dtype, DEV)
    psd.pack_factors(plan, [_dev(x) for x in d["delta"]], [_dev(x) for x in d["act"]], dtype, U, ldu, V, ldv)
    return plan, U, ldu, V, ldv


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [psd.BF16, psd.F32])
def test_static_scratch_entry_equals_workspace_entry_on_two_calls_in_a_row(dtype):
    # first a layer that splits in four (64 tiles), then a smaller one that splits in two: the second
    # call finds the first call's partials in the array and must not be affected by them
    shapes = [(1024, 1000, 256, 8), (520, 300, 220, 5)]
    name = "f32" if dtype == psd.F32 else "bf16"
    for call, (M, N, B, P) in enumerate(shapes):
        d = inputs.fc_layer(M, N, B, P, seed=M + N + 1, mom_std=1e-4)
        plan, U, ldu, V, ldv = _layer_on_gpu(d, dtype)
        need = psd.sfb_workspace_bytes(plan, dtype)
        assert 0 < need <= psd.STATIC_SCRATCH_BYTES
        ws = psd.alloc_workspace(plan, dtype, DEV)
        W1, M1 = _dev(d["W"]), _dev(d["Mom"])
        psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W1, M1, inputs.LR, inputs.MU, wd=5e-4, workspace=ws)
        W2, M2 = _dev(d["W"]), _dev(d["Mom"])
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()          # what the driver has left (torch's own cache does not move it)
        psd.sync_fc_sfb_static(plan, dtype, U, ldu, V, ldv, W2, M2, inputs.LR, inputs.MU, wd=5e-4)
        torch.cuda.synchronize()
        # The first call on a device looks the array's address up, which makes the runtime load the code
        # object that holds it; from then on a call takes no device memory from the driver.
        if call > 0:
            assert torch.cuda.mem_get_info()[0] >= free_before
        assert np.array_equal(W1.cpu().numpy(), W2.cpu().numpy()) and np.array_equal(M1.cpu().numpy(), M2.cpu().numpy())
        # and both are right: against the oracle
        Uo, Vo = orc.pack_factors(d["delta"], d["act"], name)
        Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], inputs.LR, inputs.MU, wd=5e-4)
        assert orc.rel_frob(M2.cpu().numpy(), Mr) <= 1e-5 and orc.rel_frob(W2.cpu().numpy(), Wr) <= 1e-5


@pytest.mark.gpu
def test_static_scratch_entry_runs_unsplit_layers_without_scratch():
    d = inputs.fc_layer_integer(384, 1000, 16, 8, seed=5)          # K = 128: never split
    plan, U, ldu, V, ldv = _layer_on_gpu(d, psd.BF16)
    assert psd.sfb_workspace_bytes(plan, psd.BF16) == 0
    W, Mom = _dev(d["W"]), _dev(d["Mom"])
    psd.sync_fc_sfb_static(plan, psd.BF16, U, ldu, V, ldv, W, Mom, 0.25, 0.5)
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)


def test_static_scratch_entry_refuses_layers_beyond_its_array_on_the_host():
    L = psd.lib()
    fake = lambda a: ctypes.c_void_p(a)
    # with the 128 x 256 tile pinned, a 4096 -> 1024 layer has 128 tiles and splits in two: 2 x 16 MiB of partials
    psd.tune_set(psd.TUNE_SFB_BF16_TILE, 0)
    try:
        big = psd.plan_layer(psd.LAYER_FC, 4096, 1024, 256, 8)
        need = psd.sfb_workspace_bytes(big, psd.BF16)
        assert need == 2 * 4096 * 1024 * 4 and need > psd.STATIC_SCRATCH_BYTES
        ldu, ldv = psd.factor_ld(big.N, psd.BF16), psd.factor_ld(big.M, psd.BF16)
        st = L.psd_sync_fc_sfb_static(ctypes.byref(big), psd.BF16, fake(0x10000000), ldu, fake(0x20000000), ldv,
                                      fake(0x30000000), fake(0x40000000), 0.01, 0.9, 0.0, None)
        assert st == psd.E_WORKSPACE
        assert L.psd_sync_fc_sfb_static(None, psd.BF16, fake(0x10000000), ldu, fake(0x20000000), ldv, fake(0x30000000),
                                        fake(0x40000000), 0.01, 0.9, 0.0, None) == psd.E_NULL
    finally:
        psd.tune_set(psd.TUNE_SFB_BF16_TILE, -1)
