"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numeric example (no loss, gradient or update value), so
the oracle is pinned by: central finite differences in double, PyTorch CPU autograd
assembled from library routines, closed forms, and structural invariants
(Algorithm 1: recompute changes where and when, not what; Section 4.2: no drift).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import mt_inputs
from dataclasses import replace

from mt_inputs import ModelShape

SMALL_MHA = ModelShape(n_layers=2, hidden=16, n_q_heads=4, n_kv_heads=4, head_dim=8, ffn=24, vocab=32)
SMALL_GQA = ModelShape(n_layers=2, hidden=24, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=40, vocab=29,
                       rope_base=500.0, rms_eps=1e-6)


def small_problem(shape, B=2, T=8, seed=3, std=0.3):
    rng = np.random.default_rng(seed)
    params = []
    for name, r, c in mt_inputs.tensor_table(shape):
        if name.endswith("norm"):
            params.append(1.0 + 0.2 * rng.standard_normal(r))
        elif c == 1:
            params.append(std * rng.standard_normal(r))      # bias vectors
        else:
            params.append(std * rng.standard_normal((r, c)))
    tokens = rng.integers(0, shape.vocab, (B, T)).astype(np.int32)
    labels = rng.integers(0, shape.vocab, (B, T)).astype(np.int32)
    return params, tokens, labels


# ----------------------------------------------------------------------------- finite differences
SMALL_GQA_BIAS = replace(SMALL_GQA, qkv_bias=True)
SMALL_TIED = replace(SMALL_GQA, qkv_bias=True, tie_embeddings=True)


@pytest.mark.parametrize("shape", [SMALL_MHA, SMALL_GQA, SMALL_GQA_BIAS, SMALL_TIED],
                         ids=["mha", "gqa", "gqa-bias", "tied"])
def test_backward_matches_central_differences(orc64, shape):
    params, tokens, labels = small_problem(shape)
    loss, grads = orc64.train_step(shape, params, tokens, labels, mode=1)
    rng = np.random.default_rng(0)
    h = 1e-5
    worst = 0.0
    for ti, (p, g) in enumerate(zip(params, grads)):
        flat = p.reshape(-1)
        picks = rng.choice(flat.size, size=min(6, flat.size), replace=False)
        for i in picks:
            keep = flat[i]
            flat[i] = keep + h
            lp = orc64.forward_loss(shape, params, tokens, labels)
            flat[i] = keep - h
            lm = orc64.forward_loss(shape, params, tokens, labels)
            flat[i] = keep
            fd = (lp - lm) / (2 * h)
            an = g.reshape(-1)[i]
            err = abs(fd - an) / max(abs(fd), abs(an), 1e-3)
            worst = max(worst, err)
            assert err < 1e-6, (ti, i, fd, an)
    assert worst < 1e-6


# ----------------------------------------------------------------------------- library routines (torch CPU autograd)
def torch_model_loss(shape, tparams, tokens, labels):
    """The same decoder-only LM assembled from torch library ops; backward is autograd's."""
    L, d, Hq, Hkv, hd = shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    B, T = tokens.shape
    tok = torch.from_numpy(tokens.astype(np.int64))
    lab = torch.from_numpy(labels.astype(np.int64))
    pos = torch.arange(T, dtype=torch.float64)
    inv = shape.rope_base ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]

    def rope(x):  # x [B,T,H,hd]; rotate_half convention
        x1, x2 = x[..., : hd // 2], x[..., hd // 2:]
        return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)

    h = F.embedding(tok, tparams[0])
    pl = 12 if shape.qkv_bias else 9
    for l in range(L):
        g1, wq, wk, wv, wo, g2, wg, wu, wd = tparams[1 + pl * l: 10 + pl * l]
        bq, bk, bv = tparams[10 + pl * l: 13 + pl * l] if shape.qkv_bias else (None, None, None)
        xn = F.rms_norm(h, (d,), g1, shape.rms_eps)
        q = rope(F.linear(xn, wq, bq).view(B, T, Hq, hd)).transpose(1, 2)
        k = rope(F.linear(xn, wk, bk).view(B, T, Hkv, hd)).transpose(1, 2)
        v = F.linear(xn, wv, bv).view(B, T, Hkv, hd).transpose(1, 2)
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B, T, Hq * hd)
        h = h + F.linear(a, wo)
        yn = F.rms_norm(h, (d,), g2, shape.rms_eps)
        h = h + F.linear(F.silu(F.linear(yn, wg)) * F.linear(yn, wu), wd)
    gf, wlm = (tparams[-1], tparams[0]) if shape.tie_embeddings else (tparams[-2], tparams[-1])
    z = F.linear(F.rms_norm(h, (d,), gf, shape.rms_eps), wlm)
    return F.cross_entropy(z.view(B * T, -1), lab.view(-1), ignore_index=-100)


@pytest.mark.parametrize("shape", [SMALL_MHA, SMALL_GQA, SMALL_GQA_BIAS, SMALL_TIED],
                         ids=["mha", "gqa", "gqa-bias", "tied"])
def test_step_matches_torch_autograd(orc64, shape):
    params, tokens, labels = small_problem(shape, B=3, T=11, seed=5)
    loss, grads = orc64.train_step(shape, params, tokens, labels, mode=1)
    tparams = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    tl = torch_model_loss(shape, tparams, tokens, labels)
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12 * max(1, abs(loss))
    for (name, _, _), g, tp in zip(mt_inputs.tensor_table(shape), grads, tparams):
        ref = tp.grad.numpy()
        err = np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30)
        assert err < 1e-10, (name, err)


def test_ignored_labels_match_torch(orc64):
    shape = SMALL_MHA
    params, tokens, labels = small_problem(shape, B=2, T=6, seed=9)
    labels = labels.copy()
    labels[0, :3] = -100
    loss, grads = orc64.train_step(shape, params, tokens, labels, mode=0)
    tparams = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    tl = torch_model_loss(shape, tparams, tokens, labels)
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    assert np.allclose(grads[-1], tparams[-1].grad.numpy(), rtol=1e-9, atol=1e-14)


# ----------------------------------------------------------------------------- recompute invariant
@pytest.mark.parametrize("L", [1, 2, 5])
def test_streamed_recompute_equals_monolithic_bitwise(orc64, L):
    shape = ModelShape(L, 16, 4, 2, 8, 24, 32)
    params, tokens, labels = small_problem(shape, seed=L)
    l0, g0 = orc64.train_step(shape, params, tokens, labels, mode=0)
    l1, g1 = orc64.train_step(shape, params, tokens, labels, mode=1)
    assert l0 == l1
    for a, b in zip(g0, g1):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("L,K", [(5, 2), (5, 3), (6, 3), (4, 4), (3, 7)])
def test_checkpoint_interval_k_equals_monolithic_bitwise(orc64, L, K):
    """Algorithm 1 with checkpoint interval K (blocks of K layers, partial last block, K >= L): the
    boundaries that are not checkpoints are destroyed after the forward, so a NaN-free, bit-identical
    result proves the block recomputation restores exactly what the backward needs."""
    shape = ModelShape(L, 16, 4, 2, 8, 24, 32)
    params, tokens, labels = small_problem(shape, seed=10 * L + K)
    l0, g0 = orc64.train_step(shape, params, tokens, labels, mode=0)
    lk, gk = orc64.train_step(shape, params, tokens, labels, mode=K)
    assert l0 == lk
    for a, b in zip(g0, gk):
        assert np.all(np.isfinite(b)) and np.array_equal(a, b)


# ----------------------------------------------------------------------------- loss closed forms
@pytest.mark.parametrize("V", [1024, 32000])
def test_zero_head_gives_log_vocab(orc64, V):
    rng = np.random.default_rng(0)
    loss, dl = orc64.cross_entropy(np.zeros((5, V)), rng.integers(0, V, 5))
    assert abs(loss - math.log(V)) < 1e-12
    assert abs(math.log(1024) - 6.931472) < 1e-6 and abs(math.log(32000) - 10.373491) < 1e-6
    assert np.allclose(dl.sum(axis=1), 0, atol=1e-15)
    # every wrong class gets 1/(V n), the right one (1/V - 1)/n
    assert np.allclose(np.sort(dl, axis=1)[:, -1], 1.0 / (V * 5))


def test_cross_entropy_matches_torch(orc64):
    rng = np.random.default_rng(1)
    z = rng.standard_normal((7, 50)) * 3
    y = rng.integers(0, 50, 7)
    loss, dl = orc64.cross_entropy(z, y)
    zt = torch.tensor(z, requires_grad=True)
    lt = F.cross_entropy(zt, torch.tensor(y))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-13
    assert np.allclose(dl, zt.grad.numpy(), rtol=1e-11, atol=1e-15)


def test_seeded_init_loss_close_to_log_vocab(orc64):
    s, B, T = mt_inputs.CONFIGS["tiny"]
    params = mt_inputs.make_params(s)
    tok, lab = mt_inputs.make_batch(s.vocab, B, T)
    loss = orc64.forward_loss(s, params, tok, lab)
    assert abs(loss / math.log(s.vocab) - 1) < 0.02


# ----------------------------------------------------------------------------- attention
def test_attention_special_cases(orc64):
    rng = np.random.default_rng(2)
    B, T, Hq, Hkv, hd = 2, 9, 4, 2, 8
    q = rng.standard_normal((B * T, Hq * hd))
    k = rng.standard_normal((B * T, Hkv * hd))
    v = rng.standard_normal((B * T, Hkv * hd))
    # T = 1: a = v (of the head's KV group)
    a1 = orc64.attention_fwd(q[:B], k[:B], v[:B], B, 1, Hq, Hkv, hd).reshape(B, Hq, hd)
    assert np.allclose(a1, np.repeat(v[:B].reshape(B, Hkv, hd), Hq // Hkv, axis=1), atol=1e-15)
    # q = 0: uniform weights -> running mean of v
    a0 = orc64.attention_fwd(np.zeros_like(q), k, v, B, T, Hq, Hkv, hd).reshape(B, T, Hq, hd)
    vm = np.cumsum(v.reshape(B, T, Hkv, hd), axis=1) / np.arange(1, T + 1)[None, :, None, None]
    assert np.allclose(a0, np.repeat(vm, Hq // Hkv, axis=2), atol=1e-14)
    # causality: changing rows after t leaves outputs up to t unchanged
    a = orc64.attention_fwd(q, k, v, B, T, Hq, Hkv, hd).reshape(B, T, -1)
    k2, v2 = k.reshape(B, T, -1).copy(), v.reshape(B, T, -1).copy()
    k2[:, 5:] += 1.0
    v2[:, 5:] -= 2.0
    ab = orc64.attention_fwd(q, k2.reshape(B * T, -1), v2.reshape(B * T, -1), B, T, Hq, Hkv, hd).reshape(B, T, -1)
    assert np.array_equal(a[:, :5], ab[:, :5]) and not np.allclose(a[:, 5:], ab[:, 5:])


def test_attention_matches_torch_sdpa_and_its_autograd(orc64):
    rng = np.random.default_rng(3)
    B, T, Hq, Hkv, hd = 2, 13, 6, 2, 16
    q = rng.standard_normal((B * T, Hq * hd))
    k = rng.standard_normal((B * T, Hkv * hd))
    v = rng.standard_normal((B * T, Hkv * hd))
    da = rng.standard_normal((B * T, Hq * hd))
    a = orc64.attention_fwd(q, k, v, B, T, Hq, Hkv, hd)
    dq, dk, dv = orc64.attention_bwd(da, q, k, v, B, T, Hq, Hkv, hd)
    tq = torch.tensor(q.reshape(B, T, Hq, hd), requires_grad=True)
    tk = torch.tensor(k.reshape(B, T, Hkv, hd), requires_grad=True)
    tv = torch.tensor(v.reshape(B, T, Hkv, hd), requires_grad=True)
    G = Hq // Hkv
    ta = F.scaled_dot_product_attention(tq.transpose(1, 2), tk.transpose(1, 2).repeat_interleave(G, 1),
                                        tv.transpose(1, 2).repeat_interleave(G, 1), is_causal=True)
    ta = ta.transpose(1, 2).reshape(B * T, Hq * hd)
    ta.backward(torch.tensor(da))
    assert np.allclose(a, ta.detach().numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(dq, tq.grad.reshape(B * T, -1).numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dk, tk.grad.reshape(B * T, -1).numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dv, tv.grad.reshape(B * T, -1).numpy(), rtol=1e-10, atol=1e-13)


def test_single_row_attention_matches_torch_sdpa_and_autograd(orc64):
    rng = np.random.default_rng(21)
    T, hd = 37, 16
    q, k, v, da = (rng.standard_normal((T, hd)) for _ in range(4))
    tq = torch.tensor(q[None, None], requires_grad=True)
    ta = F.scaled_dot_product_attention(tq, torch.tensor(k[None, None]), torch.tensor(v[None, None]), is_causal=True)
    ta.backward(torch.tensor(da[None, None]))
    for t in (0, 1, 17, T - 1):
        a, dq = orc64.attention_row(q[t], da[t], k[: t + 1], v[: t + 1])
        assert np.allclose(a, ta[0, 0, t].detach().numpy(), rtol=1e-11, atol=1e-13)
        assert np.allclose(dq, tq.grad[0, 0, t].numpy(), rtol=1e-10, atol=1e-13)


def test_single_key_row_matches_full_backward_and_torch_autograd(orc64):
    """orc_attention_key_row (dK, dV of one key from the queries that see it) against the full backward routine
    and against torch autograd through scaled_dot_product_attention; first, middle and last keys."""
    rng = np.random.default_rng(23)
    T, hd = 41, 16
    q, k, v, da = (rng.standard_normal((T, hd)) for _ in range(4))
    _, dk_full, dv_full = orc64.attention_bwd(da, q, k, v, 1, T, 1, 1, hd)
    tk = torch.tensor(k[None, None], requires_grad=True)
    tv = torch.tensor(v[None, None], requires_grad=True)
    ta = F.scaled_dot_product_attention(torch.tensor(q[None, None]), tk, tv, is_causal=True)
    ta.backward(torch.tensor(da[None, None]))
    for u in (0, 1, 19, T - 2, T - 1):
        dk, dv = orc64.attention_key_row(q, da, k, v, u)
        assert np.allclose(dk, dk_full[u], rtol=1e-10, atol=1e-13) and np.allclose(dv, dv_full[u], rtol=1e-10, atol=1e-13)
        assert np.allclose(dk, tk.grad[0, 0, u].numpy(), rtol=1e-10, atol=1e-13)
        assert np.allclose(dv, tv.grad[0, 0, u].numpy(), rtol=1e-10, atol=1e-13)
    # the last key is seen by the last query alone: dv = p da, with p from the single-row routine's softmax
    a_last, _ = orc64.attention_row(q[T - 1], da[T - 1], k, v)
    s = k @ q[T - 1] / np.sqrt(hd)
    p_last = np.exp(s[-1] - s.max()) / np.exp(s - s.max()).sum()
    dk, dv = orc64.attention_key_row(q, da, k, v, T - 1)
    assert np.allclose(dv, p_last * da[T - 1], rtol=1e-12)
    assert np.allclose(dk, p_last * (da[T - 1] @ v[-1] - da[T - 1] @ a_last) / np.sqrt(hd) * q[T - 1], rtol=1e-10)
    # rows of q and da before the key are not read
    q2, da2 = q.copy(), da.copy()
    q2[:19], da2[:19] = np.nan, np.nan
    dk2, dv2 = orc64.attention_key_row(q2, da2, k, v, 19)
    assert np.array_equal(dk2, orc64.attention_key_row(q, da, k, v, 19)[0]) and np.isfinite(dv2).all()


def test_gqa_equals_mha_with_replicated_kv_weights(orc64):
    gqa = ModelShape(1, 16, 4, 2, 8, 24, 20)
    mha = ModelShape(1, 16, 4, 4, 8, 24, 20)
    params, tokens, labels = small_problem(gqa, seed=11)
    lg, gg = orc64.train_step(gqa, params, tokens, labels)
    pm = list(params)
    rep = lambda w: np.repeat(w.reshape(2, 8, 16), 2, axis=0).reshape(32, 16)
    pm[3], pm[4] = rep(params[3]), rep(params[4])
    lm, gm = orc64.train_step(mha, pm, tokens, labels)
    assert abs(lg - lm) < 1e-14
    fold = lambda g: g.reshape(2, 2, 8, 16).sum(axis=1).reshape(16, 16)
    assert np.allclose(gg[3], fold(gm[3]), rtol=1e-11, atol=1e-16)
    assert np.allclose(gg[4], fold(gm[4]), rtol=1e-11, atol=1e-16)
    assert np.allclose(gg[2], gm[2], rtol=1e-11, atol=1e-16)


# ----------------------------------------------------------------------------- RoPE
def test_rope_properties(orc64):
    rng = np.random.default_rng(4)
    B, T, H, hd = 2, 12, 3, 16
    x = rng.standard_normal((B * T, H * hd))
    y = orc64.rope(x, B, T, H, hd, 10000.0, +1)
    X, Y = x.reshape(B, T, H, hd), y.reshape(B, T, H, hd)
    assert np.array_equal(X[:, 0], Y[:, 0])                                  # position 0 is the identity
    assert np.allclose(np.linalg.norm(X, axis=-1), np.linalg.norm(Y, axis=-1), rtol=1e-13)   # rotation
    assert np.allclose(orc64.rope(y, B, T, H, hd, 10000.0, -1), x, atol=1e-14)               # backward = inverse
    # relative phase: <R_m q, R_n k> depends only on m - n
    qv, kv = rng.standard_normal(hd), rng.standard_normal(hd)
    qs = orc64.rope(np.tile(qv, (T, 1)), 1, T, 1, hd, 10000.0, +1)
    ks = orc64.rope(np.tile(kv, (T, 1)), 1, T, 1, hd, 10000.0, +1)
    dots = qs @ ks.T
    for off in (0, 1, 4):
        diag = np.array([dots[m, m - off] for m in range(off, T)])
        assert np.allclose(diag, diag[0], rtol=1e-12, atol=1e-13)
    # explicit value: pair (j, j+hd/2), frequency base^(-2j/hd), at t = 3, j = 2
    t, j, base = 3, 2, 10000.0
    ang = t * base ** (-2 * j / hd)
    a, b = X[0, t, 1, j], X[0, t, 1, j + hd // 2]
    assert abs(Y[0, t, 1, j] - (a * math.cos(ang) - b * math.sin(ang))) < 1e-14
    assert abs(Y[0, t, 1, j + hd // 2] - (b * math.cos(ang) + a * math.sin(ang))) < 1e-14


# ----------------------------------------------------------------------------- RMSNorm / SwiGLU
def test_rmsnorm_constant_input_and_torch(orc64):
    c, d, eps = 1.7, 12, 1e-5
    y = orc64.rmsnorm_fwd(np.full((3, d), c), np.ones(d), eps)
    assert np.allclose(y, c / math.sqrt(c * c + eps), rtol=1e-14)
    rng = np.random.default_rng(5)
    x, g, dy = rng.standard_normal((6, d)), rng.standard_normal(d), rng.standard_normal((6, d))
    tx, tg = torch.tensor(x, requires_grad=True), torch.tensor(g, requires_grad=True)
    ty = F.rms_norm(tx, (d,), tg, eps)
    ty.backward(torch.tensor(dy))
    dx, dg = orc64.rmsnorm_bwd(dy, x, g, eps)
    assert np.allclose(orc64.rmsnorm_fwd(x, g, eps), ty.detach().numpy(), rtol=1e-13)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-14)
    assert np.allclose(dg, tg.grad.numpy(), rtol=1e-11, atol=1e-14)


def test_swiglu_closed_forms(orc64):
    up = np.array([2.0, -3.0, 0.5])
    assert np.array_equal(orc64.swiglu_fwd(np.zeros(3), up), np.zeros(3))          # silu(0) = 0
    dg, du = orc64.swiglu_bwd(np.ones(3), np.zeros(3), up)
    assert np.allclose(dg, 0.5 * up, rtol=1e-15) and np.array_equal(du, np.zeros(3))  # silu'(0) = 1/2
    g = np.array([30.0, -30.0, 1.0])
    s = orc64.swiglu_fwd(g, up)
    assert abs(s[0] - 60.0) < 1e-10 and abs(s[1]) < 1e-10                           # silu(x) -> x, 0
    assert abs(s[2] - 0.5 / (1 + math.exp(-1.0))) < 1e-15


# ----------------------------------------------------------------------------- linear maps against numpy
def test_linear_maps_match_numpy(orc64):
    rng = np.random.default_rng(6)
    x, w, dy = rng.standard_normal((7, 5)), rng.standard_normal((3, 5)), rng.standard_normal((7, 3))
    assert np.allclose(orc64.linear_fwd(x, w), x @ w.T, rtol=1e-13)
    assert np.allclose(orc64.linear_bwd_x(dy, w), dy @ w, rtol=1e-13)
    assert np.allclose(orc64.linear_bwd_w(dy, x), dy.T @ x, rtol=1e-13)


def test_embedding_scatter_add_brute_force(orc64):
    rng = np.random.default_rng(7)
    V, d, n = 6, 4, 15
    tok = rng.integers(0, V, n)
    dh = rng.standard_normal((n, d))
    ref = np.zeros((V, d))
    for t in range(n):
        ref[tok[t]] += dh[t]
    assert np.allclose(orc64.embed_bwd(dh, tok, V), ref, rtol=1e-14)
    table = rng.standard_normal((V, d))
    assert np.array_equal(orc64.embed_fwd(table, tok), table[tok])


# ----------------------------------------------------------------------------- batch structure
def test_batch_is_mean_of_independent_sequences(orc64):
    shape = SMALL_GQA
    params, tokens, labels = small_problem(shape, B=3, T=7, seed=13)
    loss, grads = orc64.train_step(shape, params, tokens, labels)
    acc_l, acc_g = 0.0, [np.zeros_like(g) for g in grads]
    for b in range(3):
        l, g = orc64.train_step(shape, params, tokens[b:b + 1], labels[b:b + 1])
        acc_l += l / 3
        for a, gi in zip(acc_g, g):
            a += gi / 3
    assert abs(loss - acc_l) < 1e-13
    for a, g in zip(acc_g, grads):
        assert np.allclose(a, g, rtol=1e-10, atol=1e-15)


# ----------------------------------------------------------------------------- Adam
def test_adam_closed_forms(orc64):
    rng = np.random.default_rng(8)
    n, lr, b1, b2, eps, wd = 50, 1e-2, 0.9, 0.999, 1e-8, 0.1
    p0, g = rng.standard_normal(n), rng.standard_normal(n)
    # first step from m = v = 0
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    orc64.adam(p, g, m, v, lr, b1, b2, eps, wd, 1)
    assert np.allclose(p, p0 * (1 - lr * wd) - lr * g / (np.abs(g) + eps), rtol=1e-12)
    assert np.allclose(m, (1 - b1) * g) and np.allclose(v, (1 - b2) * g * g)
    # constant gradient, no decay: p_t = p0 - t lr g/(|g|+eps)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        orc64.adam(p, g, m, v, lr, b1, b2, eps, 0.0, t)
    assert np.allclose(p, p0 - 5 * lr * g / (np.abs(g) + eps), rtol=1e-9)
    # zero gradient: only the decay acts
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    orc64.adam(p, np.zeros(n), m, v, lr, b1, b2, eps, wd, 1)
    assert np.allclose(p, p0 * (1 - lr * wd), rtol=1e-15)


def test_adam_matches_torch_adamw(orc64):
    rng = np.random.default_rng(9)
    n, lr, b1, b2, eps, wd = 64, 3e-3, 0.8, 0.95, 1e-6, 0.05
    p0 = rng.standard_normal(n)
    tp = torch.tensor(p0.copy(), requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 5):
        g = rng.standard_normal(n)
        tp.grad = torch.tensor(g)
        opt.step()
        orc64.adam(p, g, m, v, lr, b1, b2, eps, wd, t)
    assert np.allclose(p, tp.detach().numpy(), rtol=1e-11, atol=1e-14)


# ----------------------------------------------------------------------------- fp32 build against the fp64 build
def test_float_oracle_tracks_double_oracle(orc64, orc32):
    s, B, T = mt_inputs.CONFIGS["tiny"]
    params = mt_inputs.make_params(s)
    tok, lab = mt_inputs.make_batch(s.vocab, B, T)
    l64, g64 = orc64.train_step(s, params, tok, lab)
    l32, g32 = orc32.train_step(s, params, tok, lab)
    assert abs(l32 - l64) / l64 < 1e-5
    for a, b in zip(g64, g32):
        assert np.linalg.norm(a - b) <= 1e-4 * np.linalg.norm(a)


def test_out_of_range_token_is_rejected(orc64):
    params, tokens, labels = small_problem(SMALL_MHA)
    tokens = tokens.copy()
    tokens[0, 0] = SMALL_MHA.vocab
    with pytest.raises(ValueError):
        orc64.train_step(SMALL_MHA, params, tokens, labels)
