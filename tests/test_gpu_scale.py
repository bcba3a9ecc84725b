"""Parity at the real layer shapes of the large workloads (1.3B, 7B, 14B-GQA), with one block and a short
sequence so that the fp64 CPU oracle finishes in seconds, and sampled rows of attention at the 128k
context length.  The full-size steps themselves are checked by invariants only."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import mt_inputs
import paper_2604_05091_amd as mt
from gpu_util import bf16_round, cosine, dev_bf16, host, ok, rel_l2
from test_gpu_step import check_against_oracle, gpu_step

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,T", [("1.3B", 128), ("7B", 96), ("14B", 72)])
def test_one_block_at_real_width_matches_oracle(orc64, name, T):
    shape, _, _ = mt_inputs.CONFIGS[name]
    shape = replace(shape, n_layers=1)
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, 1, T, seed=1)
    print(f"[scale] {name}: hidden {shape.hidden} ffn {shape.ffn} heads {shape.n_q_heads}/{shape.n_kv_heads} T {T}", flush=True)
    loss, grads, _ = gpu_step(shape, 1, T, params, tok, lab)
    check_against_oracle(orc64, shape, 1, T, params, tok, lab, loss, grads)


def test_many_tokens_with_a_ragged_last_row_tile_match_oracle(orc64):
    """13 x 1000 tokens: the large-grid kernels with a partial last row tile (guarded rows in the fused rotary,
    SwiGLU and SwiGLU-backward stores, the general store elsewhere) and a token count that the token-major
    weight-gradient kernel refuses (not a multiple of 64), so the transposed-copy route runs."""
    shape = mt_inputs.ModelShape(1, 256, 4, 2, 128, 512, 512)
    B, T = 13, 1000
    params = mt_inputs.make_params(shape, seed=7, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=8)
    loss, grads, _ = gpu_step(shape, B, T, params, tok, lab)
    check_against_oracle(orc64, shape, B, T, params, tok, lab, loss, grads)


@pytest.mark.parametrize("qkv_bias", [False, True])
def test_many_tokens_take_the_large_grid_kernels_and_match_oracle(orc64, qkv_bias):
    """A narrow model (heads of 128) on 12 x 1024 tokens: every projection then runs in the large-grid GEMM
    kernels that the benchmark workloads use, including the q|k|v projection whose store applies the rotary
    embedding, and the token-major weight-gradient kernel."""
    shape = mt_inputs.ModelShape(2, 256, 4, 2, 128, 512, 512, qkv_bias=qkv_bias)
    B, T = 12, 1024
    params = mt_inputs.make_params(shape, seed=5, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=6)
    print(f"[scale] narrow model, {B} x {T} tokens, qkv_bias={qkv_bias}", flush=True)
    loss, grads, _ = gpu_step(shape, B, T, params, tok, lab)
    check_against_oracle(orc64, shape, B, T, params, tok, lab, loss, grads)



def _check_dk_dv_of_late_keys(qkv, dout, DQKV, r0, T, nq, h, hd, scale, back):
    """dK and dV rows of keys close to the end of a sequence (T - 1 - d for d in back) from the definition: only the
    queries from the key to the end see it.  S = Q K^T scale (causal), P = softmax, dP = dO V^T,
    dS = P (dP - rowsum(dO O)), dV = P^T dO, dK = scale dS^T Q, in fp64 on the bf16 inputs."""
    q0 = T - 1 - max(back)
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    K = f64(qkv[r0:r0 + T, nq + h * hd: nq + (h + 1) * hd])
    V = f64(qkv[r0:r0 + T, 2 * nq + h * hd: 2 * nq + (h + 1) * hd])
    Q = f64(qkv[r0 + q0:r0 + T, h * hd:(h + 1) * hd])
    dO = f64(dout[r0 + q0:r0 + T, h * hd:(h + 1) * hd])
    S = Q @ K.T * scale
    S[np.arange(T)[None, :] > (q0 + np.arange(T - q0))[:, None]] = -np.inf
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    dS = P * (dO @ V.T - np.sum(dO * (P @ V), axis=1)[:, None])
    for d in back:
        k = T - 1 - d
        dv_ref, dk_ref = P[:, k] @ dO, scale * (dS[:, k] @ Q)
        dv = DQKV[r0 + k, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy()
        dk = DQKV[r0 + k, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy()
        assert rel_l2(dv, dv_ref) < 3e-2 and cosine(dv, dv_ref) > 0.999, (h, k, rel_l2(dv, dv_ref))
        assert rel_l2(dk, dk_ref) < 3e-2 and cosine(dk, dk_ref) > 0.999, (h, k, rel_l2(dk, dk_ref))


def test_attention_rows_at_128k_context(orc64):
    """Forward output and dq of sampled query rows at T = 131072 (one sequence, 7B head layout reduced to
    2 query heads sharing nothing): each row needs only its own keys, so the oracle can do it row by row; dK and dV
    of keys near the end of the sequence from the definition."""
    L = mt.lib()
    T, Hq, Hkv, hd = 131072, 2, 2, 128
    nq = Hq * hd
    ld = 3 * nq
    g = torch.Generator(device="cuda").manual_seed(5)
    qkv = (torch.randn((T, ld), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    dout = torch.randn((T, nq), device="cuda", generator=g).to(torch.bfloat16)
    pq, pk, pv = qkv.data_ptr(), qkv.data_ptr() + 2 * nq, qkv.data_ptr() + 4 * nq
    O = torch.zeros((T, nq), dtype=torch.bfloat16, device="cuda")
    LSE = torch.zeros((1, Hq, T), dtype=torch.float32, device="cuda")
    scale = 1.0 / np.sqrt(hd)
    ok(L.mt_k_flash_fwd(O.data_ptr(), nq, LSE.data_ptr(), pq, ld, pk, ld, pv, ld, 1, T, Hq, Hkv, hd, scale, None))
    DELTA = torch.empty((1, Hq, T), dtype=torch.float32, device="cuda")
    DQKV = torch.zeros((T, ld), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_flash_bwd(DQKV.data_ptr(), ld, DQKV.data_ptr() + 2 * nq, ld, DQKV.data_ptr() + 4 * nq, ld,
                        dout.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq, LSE.data_ptr(),
                        DELTA.data_ptr(), 1, T, Hq, Hkv, hd, scale, None))
    for h in (0, 1):
        kh = qkv[:, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        vh = qkv[:, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        for t in (0, 63, 64, 4095, 65535, 131071):
            qt = qkv[t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
            dat = dout[t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
            a_ref, dq_ref = orc64.attention_row(qt, dat, kh[: t + 1], vh[: t + 1])
            a = O[t, h * hd:(h + 1) * hd].float().cpu().numpy()
            dq = DQKV[t, h * hd:(h + 1) * hd].float().cpu().numpy()
            assert rel_l2(a, a_ref) < 1e-2, (h, t, rel_l2(a, a_ref))
            if t == 0:      # a single visible key: softmax is constant, so dq vanishes (up to rounding of p - 1)
                assert np.max(np.abs(dq)) < 1e-5 and np.all(dq_ref == 0)
            else:
                assert rel_l2(dq, dq_ref) < 3e-2 and cosine(dq, dq_ref) > 0.999, (h, t, rel_l2(dq, dq_ref))
    # dK, dV of keys in the last key block (owned by different waves of the dK/dV workgroup)
    _check_dk_dv_of_late_keys(qkv, dout, DQKV, 0, T, nq, 1, hd, scale, (0, 37, 140, 255))


# ----------------------------------------------------------------------------- full-size launches, sampled outputs
@pytest.mark.parametrize("name,M,N,K,fp32", [("7B qkv", 65536, 12288, 4096, False), ("7B down", 65536, 4096, 11008, False),
                                             ("7B wgrad gate/up", 22016, 4096, 65536, True),
                                             ("14B qkv", 65536, 7168, 5120, False)])
def test_gemm_at_benchmark_shapes_sampled_outputs(orc64, name, M, N, K, fp32):
    """The GEMM launches of the benchmark step at their real sizes (same grid, tile order and kernel as in
    bench.py); 48 output elements, sampled over first/last tiles and at random, against the oracle's dot
    products of the same bf16 inputs."""
    L = mt.lib()
    g = torch.Generator(device="cuda").manual_seed(M % 1000 + N)
    A = (torch.randn((M, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    B = (torch.randn((N, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    C = torch.zeros((M, N), dtype=torch.float32 if fp32 else torch.bfloat16, device="cuda")
    print(f"[scale] gemm {name}: {M} x {N} x {K}", flush=True)
    ok(L.mt_k_gemm_nt(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, 0, M, N, K, int(fp32), 0, None))
    rng = np.random.default_rng(7)
    rows = np.concatenate([[0, 255, 256, M - 1, M - 256], rng.integers(0, M, 11)])
    cols = np.concatenate([[0, 255, N - 1], rng.integers(0, N, 0)])
    picks = [(int(r), int(c)) for r in rows[:8] for c in cols] + [(int(r), int(rng.integers(0, N))) for r in rows for _ in range(2)]
    for r, c in picks[:48]:
        a = A[r].float().cpu().numpy().astype(np.float64)[None, :]
        b = B[c].float().cpu().numpy().astype(np.float64)[None, :]
        ref = float(orc64.linear_fwd(a, b)[0, 0])
        got = float(C[r, c].float().cpu())
        tol = (1e-5 if fp32 else 2.0 ** -8) * max(abs(ref), 1.0) + 1e-6 * np.sqrt(K)
        assert abs(got - ref) <= tol, (name, r, c, got, ref)


def test_attention_at_benchmark_shape_sampled_rows(orc64):
    """Forward output and dq at the 7B benchmark shape (16 sequences x 4096 tokens, 32 heads of 128): rows of
    several sequences and heads against the single-row oracle."""
    L = mt.lib()
    Bn, T, Hq, Hkv, hd = 16, 4096, 32, 32, 128
    nq = Hq * hd
    ld = 3 * nq
    g = torch.Generator(device="cuda").manual_seed(9)
    qkv = (torch.randn((Bn * T, ld), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    dout = torch.randn((Bn * T, nq), device="cuda", generator=g).to(torch.bfloat16)
    pq, pk, pv = qkv.data_ptr(), qkv.data_ptr() + 2 * nq, qkv.data_ptr() + 4 * nq
    O = torch.zeros((Bn * T, nq), dtype=torch.bfloat16, device="cuda")
    LSE = torch.zeros((Bn, Hq, T), dtype=torch.float32, device="cuda")
    DELTA = torch.empty((Bn, Hq, T), dtype=torch.float32, device="cuda")
    DQKV = torch.zeros((Bn * T, ld), dtype=torch.bfloat16, device="cuda")
    scale = 1.0 / np.sqrt(hd)
    ok(L.mt_k_flash_fwd(O.data_ptr(), nq, LSE.data_ptr(), pq, ld, pk, ld, pv, ld, Bn, T, Hq, Hkv, hd, scale, None))
    ok(L.mt_k_flash_bwd(DQKV.data_ptr(), ld, DQKV.data_ptr() + 2 * nq, ld, DQKV.data_ptr() + 4 * nq, ld,
                        dout.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq, LSE.data_ptr(),
                        DELTA.data_ptr(), Bn, T, Hq, Hkv, hd, scale, None))
    for b, h, t in ((0, 0, 1), (0, 31, 4095), (7, 13, 2047), (15, 5, 255), (15, 31, 256), (3, 17, 3000)):
        r0 = b * T
        kh = qkv[r0:r0 + t + 1, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        vh = qkv[r0:r0 + t + 1, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        qt = qkv[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
        dat = dout[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
        a_ref, dq_ref = orc64.attention_row(qt, dat, kh, vh)
        a = O[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy()
        dq = DQKV[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy()
        assert rel_l2(a, a_ref) < 1e-2, (b, h, t)
        assert cosine(dq, dq_ref) > 0.999 and rel_l2(dq, dq_ref) < 3e-2, (b, h, t, rel_l2(dq, dq_ref))
    # dK, dV of the last key of a sequence depend on the last query alone: a closed form from the row oracle's pieces
    b, h, t = 9, 20, T - 1
    r0 = b * T
    kh = qkv[r0:r0 + T, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
    vh = qkv[r0:r0 + T, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
    qt = qkv[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
    dat = dout[r0 + t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
    s = kh @ qt * scale
    p = np.exp(s - s.max())
    p /= p.sum()
    a_row = p @ vh
    dv_ref = p[-1] * dat
    dk_ref = p[-1] * (vh[-1] @ dat - a_row @ dat) * scale * qt
    dv = DQKV[r0 + t, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy()
    dk = DQKV[r0 + t, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy()
    assert rel_l2(dv, dv_ref) < 3e-2 and rel_l2(dk, dk_ref) < 3e-2, (rel_l2(dv, dv_ref), rel_l2(dk, dk_ref))
    # and keys further back, which several queries see, from the definition
    _check_dk_dv_of_late_keys(qkv, dout, DQKV, 4 * T, T, nq, 11, hd, scale, (0, 33, 100, 250, 300))
