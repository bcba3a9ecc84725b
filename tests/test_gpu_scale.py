"""Parity at the shapes the benchmark workloads run (1.3B, 7B, 14B-GQA, 128k context).

Three kinds of test: (1) whole steps of one block at the exact layer widths, on a short sequence against the fp64
oracle and on one full-length sequence (1 x 4096 tokens, so that every launch takes the large-grid kernels of the
benchmark) against its fp32 build; (2) single launches at their full benchmark sizes (GEMMs with each fused store,
the token-major weight-gradient kernel with the reduction split the step picks, attention at 16 x 4096 and at
131 072 tokens) with sampled outputs that the oracle computes one by one; (3) properties of the full 1.3B step that
hold at any size (pipelined == serial == repeated, bit for bit; finite, smooth gradient norms; the initial loss in
closed form)."""
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



def _check_dk_dv_of_late_keys(orc64, qkv, dout, DQKV, r0, T, nq, h, hd, back):
    """dK and dV rows of sampled keys (T - 1 - d for d in back; the cost on the CPU grows with the number of queries
    that see the key, so long sequences sample keys near their end) against the oracle's single
    key row (orc_attention_key_row: only the queries from the key to the end see it), on the same bf16 inputs."""
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    K = f64(qkv[r0:r0 + T, nq + h * hd: nq + (h + 1) * hd])
    V = f64(qkv[r0:r0 + T, 2 * nq + h * hd: 2 * nq + (h + 1) * hd])
    Q = f64(qkv[r0:r0 + T, h * hd:(h + 1) * hd])
    dO = f64(dout[r0:r0 + T, h * hd:(h + 1) * hd])
    for d in back:
        k = T - 1 - d
        dk_ref, dv_ref = orc64.attention_key_row(Q, dO, K, V, k)
        dv = DQKV[r0 + k, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy()
        dk = DQKV[r0 + k, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy()
        assert rel_l2(dv, dv_ref) < 3e-2 and cosine(dv, dv_ref) > 0.999, (h, k, rel_l2(dv, dv_ref))
        assert rel_l2(dk, dk_ref) < 3e-2 and cosine(dk, dk_ref) > 0.999, (h, k, rel_l2(dk, dk_ref))
        # per element, at the row's scale: bf16 result; P, dS and O (inside delta, which dS subtracts from a
        # number of its own size) each rounded to bf16 once on the way
        assert np.max(np.abs(dv - dv_ref)) <= 2.0 ** -5 * np.max(np.abs(dv_ref)), (h, k)
        assert np.max(np.abs(dk - dk_ref)) <= 2.0 ** -5 * np.max(np.abs(dk_ref)), (h, k)


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
    _check_dk_dv_of_late_keys(orc64, qkv, dout, DQKV, 0, T, nq, 1, hd, (0, 37, 140, 255, 4096, 8191))


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
    _check_dk_dv_of_late_keys(orc64, qkv, dout, DQKV, 4 * T, T, nq, 11, hd, (0, 33, 100, 250, 300))
    # at T = 4096 the oracle can also afford the earliest keys, which every query of the sequence sees: keys 0, 1,
    # 63 | 64 (a tile seam), 255 | 256 (a key-block seam), 2047
    _check_dk_dv_of_late_keys(orc64, qkv, dout, DQKV, 9 * T, T, nq, 30, hd,
                              (T - 1, T - 2, T - 64, T - 65, T - 256, T - 257, T - 2048))


# ----------------------------------------------------------------------------- weight gradients at the benchmark shapes
def _rows_and_cols(rng, M, N):
    """8 output rows x 6 output columns = 48 sampled outputs: corners of the first and the last 256 x 256 tile, the
    seam between the first two tiles, and random ones."""
    rows = np.unique(np.concatenate([[0, 255, 256, M - 256, M - 1], rng.integers(0, M, 8)]))[:8]
    cols = np.unique(np.concatenate([[0, 255, 256, N - 1], rng.integers(0, N, 6)]))[:6]
    rows = np.unique(np.concatenate([rows, [M - 1]]))
    cols = np.unique(np.concatenate([cols, [N - 1]]))
    return rows, cols


@pytest.mark.parametrize("name,M,N,K,extra_split", [
    ("7B q|k|v", 12288, 4096, 65536, 2), ("7B o", 4096, 4096, 65536, 3), ("7B gate|up", 22016, 4096, 65536, 2),
    ("7B down", 4096, 11008, 65536, 5), ("14B q|k|v", 7168, 5120, 65536, 4)])
def test_weight_gradient_kernel_at_benchmark_shapes_sampled_outputs(orc64, name, M, N, K, extra_split):
    """dW [M, N] = dY^T X over the K = 65 536 tokens of a 7B / 14B step, through the token-major kernel the step uses
    (mt_k_gemm_tn), unsplit, with the reduction split the step would pick on 256 compute units, and with one more
    split so that every shape also crosses chunk seams; >= 48 sampled outputs each against the oracle's weight
    gradient (orc_linear_bwd_w) of the same bf16 columns."""
    L = mt.lib()
    g = torch.Generator(device="cuda").manual_seed(M % 997 + N)
    dY = (torch.randn((K, M), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    X = (torch.randn((K, N), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    rng = np.random.default_rng(M + N)
    rows, cols = _rows_and_cols(rng, M, N)
    dy_cols = dY[:, torch.as_tensor(rows, device="cuda")].float().cpu().numpy().astype(np.float64)
    x_cols = X[:, torch.as_tensor(cols, device="cuda")].float().cpu().numpy().astype(np.float64)
    ref = orc64.linear_bwd_w(dy_cols, x_cols)                       # [len(rows), len(cols)]
    assert ref.shape == (len(rows), len(cols)) and ref.size >= 48
    tol = 1e-5 * np.maximum(np.abs(ref), 1.0) + 1e-6 * np.sqrt(K)
    picked = L.mt_k_gemm_tn_pick_split(M, N, K, 256)
    splits = sorted({1, picked, extra_split})
    print(f"[scale] wgrad {name}: {M} x {N} x {K}, picked split {picked}, testing {splits}", flush=True)
    ws = torch.empty((max(splits) - 1) * M * N, dtype=torch.float32, device="cuda")
    ri, ci = torch.as_tensor(rows, device="cuda"), torch.as_tensor(cols, device="cuda")
    first = None
    for sp in splits:
        C = torch.full((M, N), 3.0, dtype=torch.float32, device="cuda")
        if sp == 1:
            ok(L.mt_k_gemm_tn(dY.data_ptr(), M, X.data_ptr(), N, C.data_ptr(), N, M, N, K, 0, None))
        else:
            ok(L.mt_k_gemm_tn_split(dY.data_ptr(), M, X.data_ptr(), N, C.data_ptr(), N, M, N, K, 0, sp, ws.data_ptr(),
                                    None))
        got = C[ri][:, ci].cpu().numpy().astype(np.float64)
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (name, sp, rows[np.where(bad)[0]], cols[np.where(bad)[1]], got[bad], ref[bad])
        # nothing left unwritten, and splitting only reorders fp32 sums
        assert bool(torch.isfinite(C).all())
        if first is None:
            first = C
        else:
            d = (C - first).abs().max().item()
            assert d <= 5e-3, (name, sp, d)
    # accumulate != 0 adds to what is there (the LM head's gradient over token chunks)
    if picked > 1:
        C2 = first.clone()
        ok(L.mt_k_gemm_tn_split(dY.data_ptr(), M, X.data_ptr(), N, C2.data_ptr(), N, M, N, K, 1, picked, ws.data_ptr(), None))
        got = C2[ri][:, ci].cpu().numpy().astype(np.float64)
        assert (np.abs(got - 2 * ref) <= 2 * tol).all(), name


# ----------------------------------------------------------------------------- fused stores at the 7B shapes
SAMPLE_ROWS_7B = (0, 255, 256, 4095, 4096, 30001, 65280, 65535)   # tile corners, sequence seams, last tile


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def test_rope_store_at_7b_shape_sampled_rows(orc64):
    """The q|k|v projection of a 7B block (65 536 x 12 288 x 4096) with the rotary embedding applied in the store:
    whole sampled rows against the oracle's linear map followed by its rotary embedding at the row's position."""
    L = mt.lib()
    M, N, K, T, hd, base = 65536, 12288, 4096, 4096, 128, 10000.0
    rope_cols = 8192                       # q and k heads rotate, v does not
    g = torch.Generator(device="cuda").manual_seed(31)
    A = (torch.randn((M, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    W = (torch.randn((N, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)
    C = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    cs, sn = np.empty((T, hd // 2), np.float32), np.empty((T, hd // 2), np.float32)
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, hd, base) == 0
    CS, SN = torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda()
    ok(L.mt_k_gemm_nt_rope(A.data_ptr(), K, W.data_ptr(), K, C.data_ptr(), N, None, CS.data_ptr(), SN.data_ptr(), T,
                           rope_cols, M, N, K, None))
    w = _f64(W)
    rows = (0, 255, 256, 4094, 4097, 30001, 65280, 65535)     # distinct positions inside their sequences
    lin = orc64.linear_fwd(_f64(A[list(rows)]), w)                      # [8, N] unrotated
    # rotate: the oracle's rope works on [B*T, H*hd] with positions 0..T-1; place each sampled row at its position
    pos = [r % T for r in rows]
    assert len(set(pos)) == len(pos)
    buf = np.zeros((T, rope_cols))
    for i, p in enumerate(pos):
        buf[p] = lin[i, :rope_cols]
    rot = orc64.rope(buf, 1, T, rope_cols // hd, hd, base, +1)
    for i, (r, p) in enumerate(zip(rows, pos)):
        ref = np.concatenate([rot[p], lin[i, rope_cols:]])
        got = _f64(C[r])
        # a rotated element mixes both members of its pair: the rounding is relative to the pair's size
        pair = np.abs(lin[i, :rope_cols]).reshape(-1, 2, hd // 2)
        scale = np.concatenate([np.repeat(np.hypot(pair[:, 0], pair[:, 1])[:, None, :], 2, axis=1).reshape(-1),
                                np.abs(lin[i, rope_cols:])])
        tol = 2.0 ** -8 * scale + 1e-6 * np.sqrt(K)
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (r, np.where(bad)[0][:8], got[bad][:4], ref[bad][:4])
    assert rel_l2(_f64(C[list(rows)]), np.concatenate([rot[pos], lin[:, rope_cols:]], axis=1)) < 6e-3


def test_swiglu_store_at_7b_shape_sampled_rows(orc64):
    """The gate|up projection of a 7B block (65 536 x 22 016 x 4096) with the activation in the store: gate|up rows
    against the oracle's linear map, s rows against its SwiGLU."""
    L = mt.lib()
    M, F, K = 65536, 11008, 4096
    g = torch.Generator(device="cuda").manual_seed(32)
    A = (torch.randn((M, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    W = (torch.randn((2 * F, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)
    GU = torch.zeros((M, 2 * F), dtype=torch.bfloat16, device="cuda")
    S = torch.zeros((M, F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_swiglu(A.data_ptr(), K, W.data_ptr(), K, GU.data_ptr(), 2 * F, S.data_ptr(), F, M, F, K, None))
    rows = list(SAMPLE_ROWS_7B)
    lin = orc64.linear_fwd(_f64(A[rows]), _f64(W))                      # [8, 2F]
    gu = _f64(GU[rows])
    assert (np.abs(gu - lin) <= 2.0 ** -8 * np.abs(lin) + 1e-6 * np.sqrt(K)).all()
    gate, up = lin[:, :F], lin[:, F:]
    ref = orc64.swiglu_fwd(gate, up)
    got = _f64(S[rows])
    # the kernel applies the activation to the bf16-rounded gate and up: d s = u silu'(g) dg + silu(g) du with
    # |silu'| <= 1.1, |silu(g)| <= |g|, |dg| <= 2^-8 |g|, |du| <= 2^-8 |u|, plus the rounding of s itself
    tol = 2.0 ** -8 * (2.1 * np.abs(gate * up) + np.abs(ref)) + 1e-5
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (np.where(bad), got[bad][:4], ref[bad][:4])
    assert rel_l2(got, ref) < 6e-3
    # without the gate|up output (the streaming forward keeps only s): the same s, bit for bit
    S2 = torch.zeros_like(S)
    ok(L.mt_k_gemm_nt_swiglu(A.data_ptr(), K, W.data_ptr(), K, None, 0, S2.data_ptr(), F, M, F, K, None))
    assert torch.equal(S.view(torch.int16), S2.view(torch.int16))


def test_swiglu_backward_store_at_7b_shape_sampled_rows(orc64):
    """The input gradient of the 7B down projection (65 536 x 11 008 x 4096) with the SwiGLU backward in the store:
    dgate|dup rows against the oracle's linear map followed by its SwiGLU backward on the same gate and up."""
    L = mt.lib()
    M, F, K = 65536, 11008, 4096
    g = torch.Generator(device="cuda").manual_seed(33)
    DY = (torch.randn((M, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    WT = (torch.randn((F, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)      # W_down^T: [F, d]
    GU = (torch.randn((M, 2 * F), device="cuda", generator=g) * 1.5).to(torch.bfloat16)
    DGU = torch.zeros((M, 2 * F), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_gemm_nt_swiglu_bwd(DY.data_ptr(), K, WT.data_ptr(), K, DGU.data_ptr(), 2 * F, GU.data_ptr(), 2 * F, M, F, K,
                                 None))
    rows = list(SAMPLE_ROWS_7B)
    ds = orc64.linear_fwd(_f64(DY[rows]), _f64(WT))                     # [8, F]
    gu = _f64(GU[rows])
    dg_ref, du_ref = orc64.swiglu_bwd(ds, gu[:, :F], gu[:, F:])
    ref = np.concatenate([dg_ref, du_ref], axis=1)
    got = _f64(DGU[rows])
    # linear in ds, which the kernel rounds to bf16 once (2^-9) before the result is rounded again (2^-9)
    tol = 2.0 ** -7 * np.abs(ref) + 1e-6 * np.sqrt(K)
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (np.where(bad), got[bad][:4], ref[bad][:4])
    assert rel_l2(got, ref) < 6e-3


@pytest.mark.parametrize("name,N,K", [("7B o + residual", 4096, 4096), ("7B down + residual", 4096, 11008)])
def test_residual_store_at_7b_shape_sampled_rows(orc64, name, N, K):
    """The two projections of a 7B block whose store adds the residual stream (65 536 rows): whole sampled rows
    against the oracle's linear map plus the residual."""
    L = mt.lib()
    M = 65536
    g = torch.Generator(device="cuda").manual_seed(34 + K)
    A = (torch.randn((M, K), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    W = (torch.randn((N, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)
    R = torch.randn((M, N), device="cuda", generator=g).to(torch.bfloat16)
    C = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    print(f"[scale] {name}: {M} x {N} x {K}", flush=True)
    ok(L.mt_k_gemm_nt(A.data_ptr(), K, W.data_ptr(), K, C.data_ptr(), N, R.data_ptr(), N, M, N, K, 0, 0, None))
    rows = list(SAMPLE_ROWS_7B)
    lin = orc64.linear_fwd(_f64(A[rows]), _f64(W))
    ref = lin + _f64(R[rows])
    got = _f64(C[rows])
    tol = 2.0 ** -8 * np.abs(ref) + 1e-6 * np.sqrt(K) * 4
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (name, np.where(bad), got[bad][:4], ref[bad][:4])


# ----------------------------------------------------------------------------- one block, exact width, T = 4096
@pytest.mark.parametrize("name", ["7B", "14B"])
def test_one_block_at_benchmark_width_and_sequence_length_matches_oracle(orc32, name):
    """One block at the exact 7B / 14B layer widths on one full-length sequence (1 x 4096 tokens, vocabulary 32 000):
    every projection then has at least 192 tiles of 256 x 256, so the engine runs the same large-grid GEMM kernels
    (with their fused rotary / SwiGLU / SwiGLU-backward / residual stores), the token-major weight-gradient kernel
    and the attention kernels that the benchmark step runs; loss and every gradient tensor at the step tolerances.
    The reference is the oracle's fp32 build (about 1e13 FLOP: its fp64 build takes several minutes here); the fp32
    build is pinned to the fp64 one within 1e-4, far inside these tolerances."""
    shape, _, T = mt_inputs.CONFIGS[name]
    shape = replace(shape, n_layers=1)
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, 1, T, seed=1)
    print(f"[scale] {name} one block, 1 x {T} tokens: GPU step", flush=True)
    loss, grads, _ = gpu_step(shape, 1, T, params, tok, lab)
    print(f"[scale] {name} one block: loss {loss:.5f}; oracle (fp32 build) ...", flush=True)
    ref_loss, ref_grads = orc32.train_step(shape, params, tok, lab, mode=1)
    print(f"[scale] {name} one block: oracle loss {ref_loss:.5f}", flush=True)
    assert abs(loss - ref_loss) <= 1e-2 * abs(ref_loss), (loss, ref_loss)
    for (tname, _, _), gq, r in zip(mt_inputs.tensor_table(shape), grads, ref_grads):
        c, e = cosine(gq, r), rel_l2(gq, r)
        assert c >= 0.999 and e <= 3e-2, (tname, c, e)
        # no row of a gradient matrix may be off on its own (a wrong tile would hide inside the tensor norm)
        if r.ndim == 2:
            g64, r64 = gq.astype(np.float64), r.astype(np.float64)
            row_err = np.linalg.norm(g64 - r64, axis=1)
            row_ref = np.linalg.norm(r64, axis=1)
            floor = 1e-3 * row_ref.max()
            worst = np.max(row_err / np.maximum(row_ref, floor))
            assert worst <= 0.25, (tname, worst)


# ----------------------------------------------------------------------------- invariants at the exact 1.3B workload
def test_full_1p3b_step_invariants():
    """The whole 1.3B workload (24 layers, 8 x 2048 tokens): pipelined and serial schedules give the same loss and
    gradients bit for bit, a repeated step reproduces them, every gradient tensor is finite with a per-layer norm
    profile without jumps, and the loss of the freshly initialised model is ln V + sigma^2 / 2 (logits of a random
    head are N(0, sigma^2) with sigma^2 = 0.02^2 * hidden, and E log-sum-exp of such logits is ln V + sigma^2 / 2)."""
    shape, B, T = mt_inputs.CONFIGS["1.3B"]
    print("[scale] 1.3B: parameters", flush=True)
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=1)
    from test_gpu_step import make_cfg
    print("[scale] 1.3B: pipelined steps", flush=True)
    with mt.TrainHandle(make_cfg(shape, B, T), params) as h:
        l1 = h.train_step(tok, lab)
        g1 = [g.copy() for g in h.grads()]
        l2 = h.train_step(tok, lab)
        assert l1 == l2
        for a, b in zip(g1, h.grads()):
            assert np.array_equal(a, b)
    print("[scale] 1.3B: serial step", flush=True)
    with mt.TrainHandle(make_cfg(shape, B, T, flags=mt.FLAG_SERIAL), params) as h:
        l3 = h.train_step(tok, lab)
        assert l1 == l3
        for a, b in zip(g1, h.grads()):
            assert np.array_equal(a, b)
    expect = np.log(shape.vocab) + 0.5 * 0.02 ** 2 * shape.hidden
    assert abs(l1 - expect) <= 1e-2 * expect, (l1, expect)
    names = [t[0] for t in mt_inputs.tensor_table(shape)]
    norms = {}
    for n, g in zip(names, g1):
        assert np.isfinite(g).all(), n
        norms[n] = float(np.linalg.norm(g.astype(np.float64)))
        assert norms[n] > 0, n
    for kind in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "mlp_norm"):
        # from the second layer on (the first one sees the raw embedding rows and stands apart, e.g. its q/k weight
        # gradients are an order of magnitude larger) the profile has no jumps
        prof = np.array([norms[f"l{l}.{kind}"] for l in range(1, shape.n_layers)])
        ratio = prof[1:] / prof[:-1]
        assert (ratio > 0.4).all() and (ratio < 2.5).all(), (kind, prof)
