"""The entry point that allocates nothing (mt_k_rmsnorm_bwd_noalloc) against the entry point it is a variant
of (mt_k_rmsnorm_bwd with a caller workspace) and against the oracle, through the C ABI: two calls in a row
on the same device, the second with a smaller input, so the second call runs over the first call's leftovers
in the library's static workspace."""
import numpy as np
import pytest
import torch

import paper_2604_05091_amd as mt
from gpu_util import bf16_round, dev_bf16, host, ok, rel_l2

pytestmark = pytest.mark.gpu

BF16_TOL = 6e-3   # one bf16 rounding per stored element (2^-9 each) plus fp32 sums


def _case(orc64, L, n, d, seed, with_residual):
    rng = np.random.default_rng(seed)
    x, g = bf16_round(rng.standard_normal((n, d)) * 1.7), bf16_round(1 + 0.3 * rng.standard_normal(d))
    dy, dres = bf16_round(rng.standard_normal((n, d))), bf16_round(rng.standard_normal((n, d)))
    X, G, DY, DR = dev_bf16(x), dev_bf16(g), dev_bf16(dy), dev_bf16(dres)
    res_ptr = DR.data_ptr() if with_residual else None
    # the existing entry point, workspace from the caller
    ws = torch.empty(L.mt_k_rmsnorm_bwd_ws_bytes(d) // 4, dtype=torch.float32, device="cuda")
    DX0 = torch.empty_like(X)
    DG0 = torch.empty(d, dtype=torch.float32, device="cuda")
    ok(L.mt_k_rmsnorm_bwd(DX0.data_ptr(), DG0.data_ptr(), DY.data_ptr(), X.data_ptr(), G.data_ptr(), res_ptr,
                          ws.data_ptr(), n, d, 1e-5, None))
    # the variant: outputs allocated by the caller beforehand, nothing else
    DX1 = torch.full_like(X, 3.0)
    DG1 = torch.full((d,), -5.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    ok(L.mt_k_rmsnorm_bwd_noalloc(DX1.data_ptr(), DG1.data_ptr(), DY.data_ptr(), X.data_ptr(), G.data_ptr(), res_ptr,
                                  n, d, 1e-5, None))
    # same kernels, same launch, same summation order: bit for bit
    assert torch.equal(DX0.view(torch.int16), DX1.view(torch.int16))
    assert torch.equal(DG0.view(torch.int32), DG1.view(torch.int32))
    # and both against the oracle
    dx_ref, dg_ref = orc64.rmsnorm_bwd(dy, x, g, 1e-5)
    if with_residual:
        dx_ref = dx_ref + dres
    assert rel_l2(host(DX1), dx_ref) < BF16_TOL
    assert rel_l2(host(DG1), dg_ref) < 1e-5
    # per element: a bf16 result is within one rounding step of the reference at the row's scale
    err = np.abs(host(DX1) - dx_ref)
    assert (err <= 2.0 ** -7 * np.abs(dx_ref).max(axis=1, keepdims=True) + 1e-6).all()


def test_no_alloc_rmsnorm_backward_two_calls_second_smaller(orc64):
    assert torch.cuda.is_available(), "needs the MI355X"
    L = mt.lib()
    # first call: more rows than the grid has waves and the widest supported row, so every partial row of
    # the static workspace is written; second call: fewer rows (a smaller grid) and narrower rows
    _case(orc64, L, 2600, 8192, 11, True)
    _case(orc64, L, 150, 4096, 12, False)
    _case(orc64, L, 7, 264, 13, True)


def test_no_alloc_rejects_rows_wider_than_the_static_workspace():
    L = mt.lib()
    d = 8192 + 8
    X = torch.zeros((2, d), dtype=torch.bfloat16, device="cuda")
    DG = torch.zeros(d, dtype=torch.float32, device="cuda")
    st = L.mt_k_rmsnorm_bwd_noalloc(X.data_ptr(), DG.data_ptr(), X.data_ptr(), X.data_ptr(), X.data_ptr(), None, 2, d,
                                    1e-5, None)
    assert st == -2   # MT_ERR_UNSUPPORTED, nothing launched
    assert L.mt_k_rmsnorm_bwd_noalloc(X.data_ptr(), DG.data_ptr(), X.data_ptr(), X.data_ptr(), X.data_ptr(), None, 0,
                                      256, 1e-5, None) == -1
    torch.cuda.synchronize()
