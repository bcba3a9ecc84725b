"""GPU parity of every kernel against the CPU oracle, element by element, through the C ABI.

Inputs are rounded to bf16 first and the oracle (fp64) is fed exactly those values, so the
differences measured here are the kernels' own arithmetic: fp32 accumulation order and one
bf16 rounding of each stored output (relative 2^-9 per element)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2604_05091_amd as mt
from gpu_util import assert_rows_close, bf16_round, cosine, dev_bf16, dev_f32, dev_i32, host, ok, rel_l2

pytestmark = pytest.mark.gpu
L = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global L
    assert torch.cuda.is_available(), "these tests need the MI355X"
    L = mt.lib()
    yield


BF16_TOL = 6e-3   # rel. L2 of a tensor whose elements carry one bf16 rounding (2^-9 = 2e-3 each) plus fp32 sums
# Per-row bounds (gpu_util.rows_close), as a fraction of the row's largest reference element: one bf16 rounding of
# that element is 2^-9; 2^-7 leaves room for fp32 summation order.  Two roundings deep (an input of the last step
# was itself rounded): 2^-6.  Attention backward (P, dS and O each pass through bf16): 2^-5 plus 2^-9 of the
# tensor's largest element for rows that are nearly zero by cancellation.
ROW1, ROW2, ROW_ATT_BWD, ROW_FLOOR = 2.0 ** -7, 2.0 ** -6, 2.0 ** -5, 2.0 ** -9


# ----------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,N,K", [(256, 1376, 256), (256, 256, 688), (300, 200, 136), (72, 1024, 264),
                                   (4000, 3100, 200), (4096, 3072, 128)])
def test_gemm_nt_bf16_out(orc64, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a, b = bf16_round(rng.standard_normal((M, K))), bf16_round(rng.standard_normal((N, K)))
    ref = orc64.linear_fwd(a, b)
    A, B = dev_bf16(a), dev_bf16(b)
    C = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, 0, M, N, K, 0, 0, None))
    got = host(C)
    assert rel_l2(got, ref) < BF16_TOL
    assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * np.max(np.abs(ref)) + 1e-3 * np.sqrt(K)


def test_gemm_nt_residual_strides_fp32_accumulate(orc64):
    rng = np.random.default_rng(1)
    M, N, K, lda, ldb, ldc = 328, 200, 88, 96, 104, 208
    a_full, b_full = bf16_round(rng.standard_normal((M, lda))), bf16_round(rng.standard_normal((N, ldb)))
    r = bf16_round(rng.standard_normal((M, N)))
    ref = orc64.linear_fwd(a_full[:, :K], b_full[:, :K])
    A, B, R = dev_bf16(a_full), dev_bf16(b_full), dev_bf16(r)
    C = torch.zeros((M, ldc), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, R.data_ptr(), N, M, N, K, 0, 0, None))
    got = host(C)
    assert rel_l2(got[:, :N], ref + r) < BF16_TOL
    assert_rows_close(got[:, :N], ref + r, ROW1, what="gemm + residual")
    assert np.all(got[:, N:] == 0)              # nothing written outside the N columns
    # fp32 output, then accumulate a second product on top
    C32 = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C32.data_ptr(), N, None, 0, M, N, K, 1, 0, None))
    assert rel_l2(host(C32), ref) < 2e-6
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C32.data_ptr(), N, None, 0, M, N, K, 1, 1, None))
    assert rel_l2(host(C32), 2 * ref) < 2e-6


@pytest.mark.parametrize("M,N,K", [(4100, 3080, 192), (3840, 3328, 64), (256 * 14, 256 * 14, 320)])
def test_gemm_large_grid_kernel_all_epilogues(orc64, M, N, K):
    """Problems with >= 192 tiles of 256 x 256 and K % 64 == 0 take the 4-wave pipelined kernel: ragged
    and exact edges, odd and even step counts, bf16 with residual and strides, fp32 with accumulate."""
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    lda, ldb, ldc, ldr = K + 8, K + 16, N + 8, N + 24
    a_full, b_full = bf16_round(rng.standard_normal((M, lda))), bf16_round(rng.standard_normal((N, ldb)))
    r_full = bf16_round(rng.standard_normal((M, ldr)))
    ref = orc64.linear_fwd(a_full[:, :K], b_full[:, :K])
    A, B, R = dev_bf16(a_full), dev_bf16(b_full), dev_bf16(r_full)
    C = torch.zeros((M, ldc), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, R.data_ptr(), ldr, M, N, K, 0, 0, None))
    got = host(C)
    assert rel_l2(got[:, :N], ref + r_full[:, :N]) < BF16_TOL
    assert_rows_close(got[:, :N], ref + r_full[:, :N], ROW1, what="large-grid gemm + residual")
    assert np.all(got[:, N:] == 0)
    C32 = torch.full((M, N), 3.0, dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C32.data_ptr(), N, None, 0, M, N, K, 1, 0, None))
    assert rel_l2(host(C32), ref) < 2e-6
    assert_rows_close(host(C32), ref, 1e-5, what="large-grid gemm fp32")
    ok(L.mt_k_gemm_nt(A.data_ptr(), lda, B.data_ptr(), ldb, C32.data_ptr(), N, None, 0, M, N, K, 1, 1, None))
    assert rel_l2(host(C32), 2 * ref) < 2e-6
    assert_rows_close(host(C32), 2 * ref, 1e-5, what="large-grid gemm fp32 accumulate")


@pytest.mark.parametrize("M,N,K", [(300, 200, 136), (4100, 3080, 128)])
def test_gemm_bias_epilogue_and_bias_gradient(orc64, M, N, K):
    """C = A B^T + bias in both GEMM kernels (small grid / large grid), and db = column sums."""
    rng = np.random.default_rng(M + N)
    a, b = bf16_round(rng.standard_normal((M, K))), bf16_round(rng.standard_normal((N, K)))
    bias = bf16_round(rng.standard_normal(N))
    ref = orc64.linear_fwd(a, b) + bias[None, :]
    A, B, BI = dev_bf16(a), dev_bf16(b), dev_bf16(bias)
    C = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_bias(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, BI.data_ptr(), M, N, K, None))
    assert rel_l2(host(C), ref) < BF16_TOL
    assert_rows_close(host(C), ref, ROW1, what="gemm + bias")
    ws = torch.empty(L.mt_k_bias_grad_ws_bytes(N) // 4, dtype=torch.float32, device="cuda")
    DB = torch.full((N,), 5.0, dtype=torch.float32, device="cuda")
    ok(L.mt_k_bias_grad(DB.data_ptr(), C.data_ptr(), N, M, N, ws.data_ptr(), None))
    want = host(C).astype(np.float64).sum(axis=0)
    assert np.max(np.abs(host(DB) - want)) <= 1e-5 * np.sqrt(M) * np.max(np.abs(host(C)))


@pytest.mark.parametrize("n,out,inn", [(2048, 136, 264), (576, 520, 1376), (64, 8, 8), (4096, 2056, 4104)])
def test_gemm_token_major_weight_gradient(orc64, n, out, inn):
    """dW[out,in] = sum_t dy[t,out] x[t,in] straight from the token-major operands (no transposes): ragged
    and tiny edges, strides, accumulate; unsupported reduction lengths are refused."""
    rng = np.random.default_rng(n + out + inn)
    ldy, ldx = out + 8, inn + 16
    dy, x = bf16_round(rng.standard_normal((n, ldy))), bf16_round(rng.standard_normal((n, ldx)))
    ref = orc64.linear_bwd_w(np.ascontiguousarray(dy[:, :out]), np.ascontiguousarray(x[:, :inn]))
    DY, X = dev_bf16(dy), dev_bf16(x)
    DW = torch.full((out, inn), 7.0, dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_tn(DY.data_ptr(), ldy, X.data_ptr(), ldx, DW.data_ptr(), inn, out, inn, n, 0, None))
    assert rel_l2(host(DW), ref) < 5e-6
    assert_rows_close(host(DW), ref, 2e-5, what="token-major weight gradient")
    ok(L.mt_k_gemm_tn(DY.data_ptr(), ldy, X.data_ptr(), ldx, DW.data_ptr(), inn, out, inn, n, 1, None))
    assert rel_l2(host(DW), 2 * ref) < 5e-6
    assert_rows_close(host(DW), 2 * ref, 2e-5, what="token-major weight gradient, accumulate")
    assert L.mt_k_gemm_tn(DY.data_ptr(), ldy, X.data_ptr(), ldx, DW.data_ptr(), inn, out, inn, n - 8, 0, None) == -2


@pytest.mark.parametrize("n,out,inn,split", [(2048, 520, 1032, 2), (4096, 264, 256, 5), (1024, 1280, 776, 3)])
def test_gemm_weight_gradient_with_split_reduction(orc64, n, out, inn, split):
    """The weight-gradient product with its reduction over the tokens cut into chunks that run as separate
    workgroups: equal to the oracle, with and without accumulation, bit-identical from run to run; ragged tiles."""
    rng = np.random.default_rng(n + out + inn)
    dy, x = bf16_round(rng.standard_normal((n, out))), bf16_round(rng.standard_normal((n, inn)))
    ref = orc64.linear_bwd_w(dy, x)
    DY, X = dev_bf16(dy), dev_bf16(x)
    WS = torch.full(((split - 1) * out * inn,), 9.0, dtype=torch.float32, device="cuda")
    DW = torch.full((out, inn), 7.0, dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_tn_split(DY.data_ptr(), out, X.data_ptr(), inn, DW.data_ptr(), inn, out, inn, n, 0, split, WS.data_ptr(), None))
    first = DW.clone()
    assert rel_l2(host(DW), ref) < 5e-6
    assert_rows_close(host(DW), ref, 2e-5, what="split weight gradient")
    ok(L.mt_k_gemm_tn_split(DY.data_ptr(), out, X.data_ptr(), inn, DW.data_ptr(), inn, out, inn, n, 1, split, WS.data_ptr(), None))
    assert rel_l2(host(DW), 2 * ref) < 5e-6
    DW2 = torch.zeros((out, inn), dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_tn_split(DY.data_ptr(), out, X.data_ptr(), inn, DW2.data_ptr(), inn, out, inn, n, 0, split, WS.data_ptr(), None))
    assert torch.equal(first, DW2)
    # more chunks than 64-deep steps, or no workspace: argument errors
    assert L.mt_k_gemm_tn_split(DY.data_ptr(), out, X.data_ptr(), inn, DW.data_ptr(), inn, out, inn, n, 0, n // 64 + 1,
                                WS.data_ptr(), None) != 0
    assert L.mt_k_gemm_tn_split(DY.data_ptr(), out, X.data_ptr(), inn, DW.data_ptr(), inn, out, inn, n, 0, 2, None, None) != 0


def test_split_choice_for_the_benchmark_shapes():
    """The split the step picks: none where the tiles fill whole rounds of 256 workgroups (7B q|k|v and output
    projections), one where the last round would be mostly empty (14B shapes)."""
    pick = L.mt_k_gemm_tn_pick_split
    assert pick(12288, 4096, 65536, 256) == 1 and pick(4096, 4096, 65536, 256) == 1
    assert pick(22016, 4096, 65536, 256) == 2
    assert pick(7168, 5120, 65536, 256) > 1 and pick(5120, 13824, 65536, 256) > 1
    assert pick(4096, 4096, 1024, 256) == 1       # short reductions are never split


def test_gemm_weight_gradient_form_long_reduction(orc64):
    """dW[out,in] = sum_t dy[t,out] x[t,in]: both operands transposed first, fp32 result."""
    rng = np.random.default_rng(2)
    n, out, inn = 2056, 136, 264
    dy, x = bf16_round(rng.standard_normal((n, out))), bf16_round(rng.standard_normal((n, inn)))
    ref = orc64.linear_bwd_w(dy, x)
    DY, X = dev_bf16(dy), dev_bf16(x)
    DYT = torch.empty((out, n), dtype=torch.bfloat16, device="cuda")
    XT = torch.empty((inn, n), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_transpose(DY.data_ptr(), DYT.data_ptr(), n, out, out, n, 1, 1, 0, 0, 0, 0, None))
    ok(L.mt_k_transpose(X.data_ptr(), XT.data_ptr(), n, inn, inn, n, 1, 1, 0, 0, 0, 0, None))
    assert np.array_equal(host(DYT), dy.T) and np.array_equal(host(XT), x.T)
    DW = torch.empty((out, inn), dtype=torch.float32, device="cuda")
    ok(L.mt_k_gemm_nt(DYT.data_ptr(), n, XT.data_ptr(), n, DW.data_ptr(), inn, None, 0, out, inn, n, 1, 0, None))
    assert rel_l2(host(DW), ref) < 5e-6


def test_gemm_rejects_bad_arguments():
    A = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    C = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    assert L.mt_k_gemm_nt(A.data_ptr(), 64, A.data_ptr(), 64, C.data_ptr(), 64, None, 0, 64, 64, 60, 0, 0, None) == -1
    assert L.mt_k_gemm_nt(A.data_ptr(), 60, A.data_ptr(), 64, C.data_ptr(), 64, None, 0, 64, 64, 56, 0, 0, None) == -1
    assert L.mt_k_gemm_nt(A.data_ptr() + 2, 64, A.data_ptr(), 64, C.data_ptr(), 64, None, 0, 32, 32, 32, 0, 0, None) == -1
    assert L.mt_k_gemm_nt(None, 64, A.data_ptr(), 64, C.data_ptr(), 64, None, 0, 64, 64, 64, 0, 0, None) == -1
    assert L.mt_k_gemm_nt(A.data_ptr(), 64, A.data_ptr(), 64, C.data_ptr(), 64, None, 0, 0, 64, 64, 0, 0, None) == -1


def test_batched_head_transpose():
    rng = np.random.default_rng(3)
    B, T, H, hd, ld = 2, 72, 3, 64, 3 * 64 + 128
    x = bf16_round(rng.standard_normal((B * T, ld)))
    X = dev_bf16(x)
    out = torch.zeros((B, H, hd, T), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_transpose(X.data_ptr() + 2 * 128, out.data_ptr(), T, hd, ld, T, B, H, T * ld, hd, H * hd * T, hd * T, None))
    ref = x[:, 128:128 + H * hd].reshape(B, T, H, hd).transpose(0, 2, 3, 1)
    assert np.array_equal(host(out), ref)


# ----------------------------------------------------------------------------- RMSNorm
@pytest.mark.parametrize("n,d", [(37, 256), (130, 2048), (64, 4096), (19, 5120)])
def test_rmsnorm_forward_backward(orc64, n, d):
    rng = np.random.default_rng(n + d)
    x, g = bf16_round(rng.standard_normal((n, d)) * 1.7), bf16_round(1 + 0.3 * rng.standard_normal(d))
    dy, dres = bf16_round(rng.standard_normal((n, d))), bf16_round(rng.standard_normal((n, d)))
    X, G, DY, DR = dev_bf16(x), dev_bf16(g), dev_bf16(dy), dev_bf16(dres)
    Y = torch.empty_like(X)
    ok(L.mt_k_rmsnorm_fwd(Y.data_ptr(), X.data_ptr(), G.data_ptr(), n, d, 1e-5, None))
    assert rel_l2(host(Y), orc64.rmsnorm_fwd(x, g, 1e-5)) < BF16_TOL
    assert_rows_close(host(Y), orc64.rmsnorm_fwd(x, g, 1e-5), ROW1, what="rmsnorm forward")
    dx_ref, dg_ref = orc64.rmsnorm_bwd(dy, x, g, 1e-5)
    ws = torch.empty(L.mt_k_rmsnorm_bwd_ws_bytes(d) // 4, dtype=torch.float32, device="cuda")
    DX = torch.empty_like(X)
    DG = torch.empty(d, dtype=torch.float32, device="cuda")
    ok(L.mt_k_rmsnorm_bwd(DX.data_ptr(), DG.data_ptr(), DY.data_ptr(), X.data_ptr(), G.data_ptr(), DR.data_ptr(),
                          ws.data_ptr(), n, d, 1e-5, None))
    assert rel_l2(host(DX), dx_ref + dres) < BF16_TOL
    assert_rows_close(host(DX), dx_ref + dres, ROW1, what="rmsnorm backward + residual")
    assert rel_l2(host(DG), dg_ref) < 1e-5
    assert_rows_close(host(DG), dg_ref, 1e-5, what="rmsnorm gain gradient")
    ok(L.mt_k_rmsnorm_bwd(DX.data_ptr(), DG.data_ptr(), DY.data_ptr(), X.data_ptr(), G.data_ptr(), None,
                          ws.data_ptr(), n, d, 1e-5, None))
    assert rel_l2(host(DX), dx_ref) < BF16_TOL
    assert_rows_close(host(DX), dx_ref, ROW1, what="rmsnorm backward")


def test_rmsnorm_backward_many_rows_gain_reduction(orc64):
    rng = np.random.default_rng(5)
    n, d = 5000, 256      # more rows than waves in the grid: exercises the strided row loop
    x, g, dy = bf16_round(rng.standard_normal((n, d))), bf16_round(np.ones(d)), bf16_round(rng.standard_normal((n, d)))
    dx_ref, dg_ref = orc64.rmsnorm_bwd(dy, x, g, 1e-5)
    X, G, DY = dev_bf16(x), dev_bf16(g), dev_bf16(dy)
    ws = torch.empty(L.mt_k_rmsnorm_bwd_ws_bytes(d) // 4, dtype=torch.float32, device="cuda")
    DX, DG = torch.empty_like(X), torch.empty(d, dtype=torch.float32, device="cuda")
    ok(L.mt_k_rmsnorm_bwd(DX.data_ptr(), DG.data_ptr(), DY.data_ptr(), X.data_ptr(), G.data_ptr(), None,
                          ws.data_ptr(), n, d, 1e-5, None))
    assert rel_l2(host(DG), dg_ref) < 1e-5 and rel_l2(host(DX), dx_ref) < BF16_TOL
    assert_rows_close(host(DX), dx_ref, ROW1, what="rmsnorm backward, 5000 rows")
    assert_rows_close(host(DG), dg_ref, 2e-5, what="rmsnorm gain gradient, 5000 rows")


# ----------------------------------------------------------------------------- RoPE
@pytest.mark.parametrize("hd,base", [(64, 10000.0), (128, 1.0e6)])
def test_rope_forward_and_inverse(orc64, hd, base):
    rng = np.random.default_rng(hd)
    B, T, H, extra = 2, 40, 3, 2 * hd
    ld = H * hd + extra
    x = bf16_round(rng.standard_normal((B * T, ld)))
    cs, sn = np.empty((T, hd // 2), np.float32), np.empty((T, hd // 2), np.float32)
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, hd, base) == 0
    X, CS, SN = dev_bf16(x), dev_f32(cs), dev_f32(sn)
    ok(L.mt_k_rope(X.data_ptr(), ld, B * T, T, H, hd, CS.data_ptr(), SN.data_ptr(), +1, None))
    got = host(X)
    ref = orc64.rope(x[:, :H * hd], B, T, H, hd, base, +1)
    assert rel_l2(got[:, :H * hd], ref) < BF16_TOL
    assert_rows_close(got[:, :H * hd], ref, ROW1, width=hd, what="rope")
    assert np.array_equal(got[:, H * hd:], x[:, H * hd:])       # columns after the heads untouched
    ok(L.mt_k_rope(X.data_ptr(), ld, B * T, T, H, hd, CS.data_ptr(), SN.data_ptr(), -1, None))
    assert rel_l2(host(X)[:, :H * hd], x[:, :H * hd]) < 2 * BF16_TOL


@pytest.mark.parametrize("M,N,K,T,rope_cols,with_bias", [(3200, 4096, 128, 640, 3072, False),
                                                            (4100, 3072, 64, 4100, 2560, True)])
def test_gemm_with_rotary_embedding_in_the_store(orc64, M, N, K, T, rope_cols, with_bias):
    """q|k|v projection with RoPE applied by the GEMM's store (heads of 128): equals the oracle's
    linear -> (bias) -> rope on the first rope_cols columns; the remaining heads are stored unrotated.
    Ragged last row tile, positions wrapping at T, small problems refused."""
    rng = np.random.default_rng(M + N + K)
    hd, base = 128, 10000.0
    a, b = bf16_round(rng.standard_normal((M, K))), bf16_round(rng.standard_normal((N, K)))
    bias = bf16_round(rng.standard_normal(N)) if with_bias else None
    lin = orc64.linear_fwd(a, b) + (bias[None, :] if with_bias else 0.0)
    pad = (-M) % T                     # the oracle rotates whole sequences: pad the rows up to a multiple of T
    linp = np.concatenate([lin, np.zeros((pad, N))]) if pad else lin
    ref = linp.copy()
    ref[:, :rope_cols] = orc64.rope(np.ascontiguousarray(linp[:, :rope_cols]), linp.shape[0] // T, T, rope_cols // hd, hd,
                                    base, +1)
    ref = ref[:M]
    cs, sn = np.empty((T, hd // 2), np.float32), np.empty((T, hd // 2), np.float32)
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, hd, base) == 0
    A, B, CS, SN = dev_bf16(a), dev_bf16(b), dev_f32(cs), dev_f32(sn)
    BI = dev_bf16(bias) if with_bias else None
    C = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_rope(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, BI.data_ptr() if with_bias else None,
                           CS.data_ptr(), SN.data_ptr(), T, rope_cols, M, N, K, None))
    got = host(C)
    assert rel_l2(got, ref) < BF16_TOL
    assert rel_l2(got[:, rope_cols:], lin[:, rope_cols:]) < BF16_TOL
    assert_rows_close(got, ref, ROW1, width=hd, what="gemm with rotary store")
    # a grid too small for the kernel that rotates, or heads that do not line up: refused, nothing silently skipped
    assert L.mt_k_gemm_nt_rope(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, CS.data_ptr(), SN.data_ptr(), T,
                               rope_cols, 256, N, K, None) == -2
    assert L.mt_k_gemm_nt_rope(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, CS.data_ptr(), SN.data_ptr(), T,
                               rope_cols - 64, M, N, K, None) == -2


@pytest.mark.parametrize("M,F,K,keep_gu", [(3300, 2048, 128, True), (6400, 1152, 64, False)])
def test_gemm_with_swiglu_in_the_store(orc64, M, F, K, keep_gu):
    """gate|up projection whose store computes silu(gate) * up: the activation equals the oracle's, is bit-identical
    to the two-kernel route (GEMM into gu, then the SwiGLU kernel), and gu is written only when asked for.
    Ragged last row tile; small problems and ffn sizes that are not multiples of 128 are refused."""
    rng = np.random.default_rng(M + F + K)
    a, w = bf16_round(rng.standard_normal((M, K))), bf16_round(rng.standard_normal((2 * F, K)) * 0.3)
    gu_ref = orc64.linear_fwd(a, w)
    gur = bf16_round(gu_ref)
    s_ref = orc64.swiglu_fwd(np.ascontiguousarray(gur[:, :F]), np.ascontiguousarray(gur[:, F:]))
    A, W = dev_bf16(a), dev_bf16(w)
    GU = torch.full((M, 2 * F), 3.0, dtype=torch.bfloat16, device="cuda")
    S = torch.zeros((M, F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_swiglu(A.data_ptr(), K, W.data_ptr(), K, GU.data_ptr() if keep_gu else None, 2 * F, S.data_ptr(), F,
                             M, F, K, None))
    assert rel_l2(host(S), s_ref) < 2 * BF16_TOL
    assert_rows_close(host(S), s_ref, ROW2, what="gemm with SwiGLU store")
    GU2 = torch.zeros((M, 2 * F), dtype=torch.bfloat16, device="cuda")
    S2 = torch.zeros((M, F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), K, W.data_ptr(), K, GU2.data_ptr(), 2 * F, None, 0, M, 2 * F, K, 0, 0, None))
    ok(L.mt_k_swiglu_fwd(S2.data_ptr(), GU2.data_ptr(), M, F, None))
    assert torch.equal(S, S2)
    if keep_gu:
        assert torch.equal(GU, GU2)
        assert rel_l2(host(GU), gu_ref) < BF16_TOL
        assert_rows_close(host(GU), gu_ref, ROW1, what="gate|up next to the SwiGLU store")
    assert L.mt_k_gemm_nt_swiglu(A.data_ptr(), K, W.data_ptr(), K, None, 0, S.data_ptr(), F, 256, F, K, None) == -2
    assert L.mt_k_gemm_nt_swiglu(A.data_ptr(), K, W.data_ptr(), K, None, 0, S.data_ptr(), F - 64, M, F - 64, K, None) == -2


@pytest.mark.parametrize("M,F,K", [(3300, 4096, 128), (12800, 1000, 64)])
def test_gemm_with_swiglu_backward_in_the_store(orc64, M, F, K):
    """ds = A B^T followed by the SwiGLU backward inside the GEMM's store: dgate | dup equal the oracle's and are
    bit-identical to the two-kernel route.  Ragged last row tile and a ragged last column tile (F = 1000)."""
    rng = np.random.default_rng(M + F + K)
    a, w = bf16_round(rng.standard_normal((M, K))), bf16_round(rng.standard_normal((F, K)) * 0.3)
    gu = bf16_round(rng.standard_normal((M, 2 * F)))
    ds = bf16_round(orc64.linear_fwd(a, w))
    dg_ref, du_ref = orc64.swiglu_bwd(ds, np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:]))
    A, W, GU = dev_bf16(a), dev_bf16(w), dev_bf16(gu)
    DGU = torch.full((M, 2 * F), 3.0, dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_swiglu_bwd(A.data_ptr(), K, W.data_ptr(), K, DGU.data_ptr(), 2 * F, GU.data_ptr(), 2 * F, M, F, K, None))
    got = host(DGU)
    assert rel_l2(got[:, :F], dg_ref) < 2 * BF16_TOL and rel_l2(got[:, F:], du_ref) < 2 * BF16_TOL
    assert_rows_close(got[:, :F], dg_ref, ROW2, what="SwiGLU-backward store, dgate")
    assert_rows_close(got[:, F:], du_ref, ROW2, what="SwiGLU-backward store, dup")
    DS = torch.zeros((M, F), dtype=torch.bfloat16, device="cuda")
    DGU2 = torch.zeros((M, 2 * F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt(A.data_ptr(), K, W.data_ptr(), K, DS.data_ptr(), F, None, 0, M, F, K, 0, 0, None))
    ok(L.mt_k_swiglu_bwd(DGU2.data_ptr(), DS.data_ptr(), GU.data_ptr(), M, F, None))
    assert torch.equal(DGU, DGU2)
    assert L.mt_k_gemm_nt_swiglu_bwd(A.data_ptr(), K, W.data_ptr(), K, DGU.data_ptr(), 2 * F, GU.data_ptr(), 2 * F, 256, F, K,
                                     None) == -2


# ----------------------------------------------------------------------------- SwiGLU
def test_swiglu_forward_backward(orc64):
    rng = np.random.default_rng(6)
    n, F = 77, 688
    gu, ds = bf16_round(rng.standard_normal((n, 2 * F)) * 2), bf16_round(rng.standard_normal((n, F)))
    GU, DS = dev_bf16(gu), dev_bf16(ds)
    S = torch.empty((n, F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_swiglu_fwd(S.data_ptr(), GU.data_ptr(), n, F, None))
    assert rel_l2(host(S), orc64.swiglu_fwd(gu[:, :F], gu[:, F:])) < BF16_TOL
    assert_rows_close(host(S), orc64.swiglu_fwd(gu[:, :F], gu[:, F:]), ROW1, what="swiglu forward")
    DGU = torch.empty_like(GU)
    ok(L.mt_k_swiglu_bwd(DGU.data_ptr(), DS.data_ptr(), GU.data_ptr(), n, F, None))
    dg, du = orc64.swiglu_bwd(ds, gu[:, :F], gu[:, F:])
    got = host(DGU)
    assert rel_l2(got[:, :F], dg) < BF16_TOL and rel_l2(got[:, F:], du) < BF16_TOL
    assert_rows_close(got[:, :F], dg, ROW1, what="swiglu backward, dgate")
    assert_rows_close(got[:, F:], du, ROW1, what="swiglu backward, dup")


# ----------------------------------------------------------------------------- embedding
def test_embedding_gather_and_scatter(orc64):
    rng = np.random.default_rng(7)
    V, d, n = 50, 264, 333
    table = bf16_round(rng.standard_normal((V, d)))
    tok = rng.integers(0, V - 5, n).astype(np.int32)      # the last rows get no token at all
    TB, TK = dev_bf16(table), dev_i32(tok)
    H = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_embed_gather(H.data_ptr(), TB.data_ptr(), TK.data_ptr(), n, d, None))
    assert np.array_equal(host(H), orc64.embed_fwd(table, tok))
    dh = bf16_round(rng.standard_normal((n, d)))
    order = np.argsort(tok, kind="stable").astype(np.int32)
    row_start = np.zeros(V + 1, np.int32)
    row_start[1:] = np.cumsum(np.bincount(tok, minlength=V))
    DT = torch.full((V, d), 3.0, dtype=torch.float32, device="cuda")
    DH, RS, ORD = dev_bf16(dh), dev_i32(row_start), dev_i32(order)      # keep the device buffers alive
    ok(L.mt_k_embed_scatter(DT.data_ptr(), DH.data_ptr(), RS.data_ptr(), ORD.data_ptr(), V, d, None))
    got = host(DT)
    assert rel_l2(got, orc64.embed_bwd(dh, tok, V)) < 1e-6
    assert np.all(got[V - 5:] == 0)


# ----------------------------------------------------------------------------- cross-entropy
@pytest.mark.parametrize("n,V", [(9, 1024), (5, 32000), (7, 520)])
def test_cross_entropy(orc64, n, V):
    rng = np.random.default_rng(V)
    z = (rng.standard_normal((n, V)) * 3).astype(np.float32)
    y = rng.integers(0, V, n).astype(np.int32)
    y[1] = -1                                            # an ignored position
    nv = int((y >= 0).sum())
    loss_ref, dl_ref = orc64.cross_entropy(z, y)
    Z, Y = dev_f32(z), dev_i32(y)
    LR = torch.empty(n, dtype=torch.float32, device="cuda")
    DZ = torch.empty((n, V), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_cross_entropy(LR.data_ptr(), DZ.data_ptr(), Z.data_ptr(), Y.data_ptr(), n, V, 1.0 / nv, None))
    out = torch.zeros(1, dtype=torch.float32, device="cuda")
    ok(L.mt_k_reduce_sum(out.data_ptr(), LR.data_ptr(), n, 1.0 / nv, 0, None))
    assert abs(host(out)[0] - loss_ref) < 1e-5 * abs(loss_ref)
    got = host(DZ)
    assert rel_l2(got, dl_ref) < BF16_TOL
    # every element: the fp32 value (softmax - onehot) / n rounded once to bf16
    assert (np.abs(got - dl_ref) <= 2.0 ** -8 * np.abs(dl_ref) + 1e-12).all()
    # every row's loss term
    lr = host(LR)
    for r in range(n):
        if y[r] >= 0:
            zz = z[r].astype(np.float64)
            want = np.log(np.exp(zz - zz.max()).sum()) + zz.max() - zz[y[r]]
            assert abs(lr[r] - want) <= 1e-5 * max(1.0, abs(want)), r
        else:
            assert lr[r] == 0
    assert np.all(got[1] == 0)


# ----------------------------------------------------------------------------- attention
def _attention_case(orc64, B, T, Hq, Hkv, hd, seed, out_pad=0):
    """out_pad: extra elements in the row pitch of every output (4: rows are then only 8-byte aligned and the
    kernels store straight from the accumulator layout instead of through LDS)."""
    rng = np.random.default_rng(seed)
    nq, nkv = Hq * hd, Hkv * hd
    ld = nq + 2 * nkv
    qkv = bf16_round(rng.standard_normal((B * T, ld)))
    q, k, v = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:]
    scale = 1.0 / np.sqrt(hd)
    QKV = dev_bf16(qkv)
    pq, pk, pv = QKV.data_ptr(), QKV.data_ptr() + 2 * nq, QKV.data_ptr() + 2 * (nq + nkv)
    ldo, ldd = nq + out_pad, ld + out_pad
    Op = torch.zeros((B * T, ldo), dtype=torch.bfloat16, device="cuda")
    LSE = torch.zeros((B, Hq, T), dtype=torch.float32, device="cuda")
    ok(L.mt_k_flash_fwd(Op.data_ptr(), ldo, LSE.data_ptr(), pq, ld, pk, ld, pv, ld, B, T, Hq, Hkv, hd, scale, None))
    a_ref = orc64.attention_fwd(q, k, v, B, T, Hq, Hkv, hd)
    assert rel_l2(host(Op)[:, :nq], a_ref) < BF16_TOL
    assert_rows_close(host(Op)[:, :nq], a_ref, ROW2, width=hd, what="attention forward (per token and head)")
    assert not host(Op)[:, nq:].any()
    O = Op[:, :nq].contiguous()
    # log-sum-exp of the first and last row of head 0: lse_0 = s_00, lse_last from the definition
    lse = host(LSE)
    s00 = float(q[0, :hd].astype(np.float64) @ k[0, :hd].astype(np.float64)) * scale
    assert abs(lse[0, 0, 0] - s00) < 1e-3 * max(1, abs(s00))
    # backward
    dout = bf16_round(rng.standard_normal((B * T, nq)))
    dq_ref, dk_ref, dv_ref = orc64.attention_bwd(dout, q, k, v, B, T, Hq, Hkv, hd)
    DO = dev_bf16(dout)
    DELTA = torch.empty((B, Hq, T), dtype=torch.float32, device="cuda")
    DQKV = torch.zeros((B * T, ldd), dtype=torch.bfloat16, device="cuda")
    pdq, pdk, pdv = DQKV.data_ptr(), DQKV.data_ptr() + 2 * nq, DQKV.data_ptr() + 2 * (nq + nkv)
    ok(L.mt_k_flash_bwd(pdq, ldd, pdk, ldd, pdv, ldd, DO.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq,
                        LSE.data_ptr(), DELTA.data_ptr(), B, T, Hq, Hkv, hd, scale, None))
    got = host(DQKV)
    assert not got[:, ld:].any()
    # the backward reads O and P in bf16, so its error is a few bf16 roundings deep
    assert rel_l2(got[:, :nq], dq_ref) < 2e-2 and cosine(got[:, :nq], dq_ref) > 0.9995
    assert rel_l2(got[:, nq:nq + nkv], dk_ref) < 2e-2 and cosine(got[:, nq:nq + nkv], dk_ref) > 0.9995
    assert rel_l2(got[:, nq + nkv:ld], dv_ref) < 1e-2 and cosine(got[:, nq + nkv:ld], dv_ref) > 0.9995
    assert_rows_close(got[:, :nq], dq_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dq (per token and head)")
    assert_rows_close(got[:, nq:nq + nkv], dk_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dk")
    assert_rows_close(got[:, nq + nkv:ld], dv_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dv")


@pytest.mark.parametrize("B,T,Hq,Hkv,hd", [(2, 128, 4, 4, 64), (1, 200, 4, 2, 64), (2, 72, 2, 2, 128),
                                           (1, 392, 5, 1, 128), (1, 8, 2, 1, 64), (1, 648, 4, 2, 128),
                                           (2, 520, 2, 2, 64)])
def test_flash_attention_forward_backward(orc64, B, T, Hq, Hkv, hd):
    _attention_case(orc64, B, T, Hq, Hkv, hd, seed=T + hd)


@pytest.mark.parametrize("B,T,Hq,Hkv,hd", [(1, 200, 4, 2, 64), (2, 72, 2, 2, 128)])
def test_flash_attention_outputs_with_8_byte_aligned_rows(orc64, B, T, Hq, Hkv, hd):
    _attention_case(orc64, B, T, Hq, Hkv, hd, seed=T + hd + 1, out_pad=4)


@pytest.mark.parametrize("B,T,Hq,Hkv,hd", [(2, 136, 4, 2, 64), (1, 264, 3, 1, 128)])
def test_flash_attention_backward_with_rotary_backward_in_the_store(orc64, B, T, Hq, Hkv, hd):
    """dq, dk rotated back inside the attention backward: q, k are the rotated tensors; the result is the
    oracle's attention backward followed by its inverse rotation (dv is untouched)."""
    rng = np.random.default_rng(B * T + hd)
    nq, nkv, base = Hq * hd, Hkv * hd, 10000.0
    ld = nq + 2 * nkv
    qkv = bf16_round(rng.standard_normal((B * T, ld)))
    q, k, v = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:]
    scale = 1.0 / np.sqrt(hd)
    dout = bf16_round(rng.standard_normal((B * T, nq)))
    dq_ref, dk_ref, dv_ref = orc64.attention_bwd(dout, q, k, v, B, T, Hq, Hkv, hd)
    dq_ref = orc64.rope(np.ascontiguousarray(dq_ref), B, T, Hq, hd, base, -1)
    dk_ref = orc64.rope(np.ascontiguousarray(dk_ref), B, T, Hkv, hd, base, -1)
    cs, sn = np.empty((T, hd // 2), np.float32), np.empty((T, hd // 2), np.float32)
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, hd, base) == 0
    QKV, DO, CS, SN = dev_bf16(qkv), dev_bf16(dout), dev_f32(cs), dev_f32(sn)
    pq, pk, pv = QKV.data_ptr(), QKV.data_ptr() + 2 * nq, QKV.data_ptr() + 2 * (nq + nkv)
    O = torch.zeros((B * T, nq), dtype=torch.bfloat16, device="cuda")
    LSE = torch.zeros((B, Hq, T), dtype=torch.float32, device="cuda")
    ok(L.mt_k_flash_fwd(O.data_ptr(), nq, LSE.data_ptr(), pq, ld, pk, ld, pv, ld, B, T, Hq, Hkv, hd, scale, None))
    DELTA = torch.empty((B, Hq, T), dtype=torch.float32, device="cuda")
    DQKV = torch.zeros((B * T, ld), dtype=torch.bfloat16, device="cuda")
    pdq, pdk, pdv = DQKV.data_ptr(), DQKV.data_ptr() + 2 * nq, DQKV.data_ptr() + 2 * (nq + nkv)
    ok(L.mt_k_flash_bwd_rope(pdq, ld, pdk, ld, pdv, ld, DO.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq,
                             LSE.data_ptr(), DELTA.data_ptr(), CS.data_ptr(), SN.data_ptr(), B, T, Hq, Hkv, hd, scale,
                             None))
    got = host(DQKV)
    assert rel_l2(got[:, :nq], dq_ref) < 2e-2 and cosine(got[:, :nq], dq_ref) > 0.9995
    assert rel_l2(got[:, nq:nq + nkv], dk_ref) < 2e-2 and cosine(got[:, nq:nq + nkv], dk_ref) > 0.9995
    assert rel_l2(got[:, nq + nkv:], dv_ref) < 1e-2 and cosine(got[:, nq + nkv:], dv_ref) > 0.9995
    assert_rows_close(got[:, :nq], dq_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dq with rotary backward")
    assert_rows_close(got[:, nq:nq + nkv], dk_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dk with rotary backward")
    assert_rows_close(got[:, nq + nkv:], dv_ref, ROW_ATT_BWD, ROW_FLOOR, width=hd, what="attention dv")
    # one table without the other is an argument error
    assert L.mt_k_flash_bwd_rope(pdq, ld, pdk, ld, pdv, ld, DO.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq,
                                 LSE.data_ptr(), DELTA.data_ptr(), CS.data_ptr(), None, B, T, Hq, Hkv, hd, scale,
                                 None) != 0


def test_flash_attention_rejects_bad_shapes():
    x = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(4096, dtype=torch.float32, device="cuda")
    p = x.data_ptr()
    assert L.mt_k_flash_fwd(p, 64, f.data_ptr(), p, 64, p, 64, p, 64, 1, 12, 1, 1, 64, 0.125, None) == -1   # T % 8
    assert L.mt_k_flash_fwd(p, 96, f.data_ptr(), p, 96, p, 96, p, 96, 1, 8, 1, 1, 96, 0.1, None) == -1      # head_dim
    assert L.mt_k_flash_fwd(p, 64, f.data_ptr(), p, 64, p, 64, p, 64, 1, 8, 3, 2, 64, 0.125, None) == -1    # Hq % Hkv
