"""GPU parity of the whole streamed training step (Algorithm 1) and the host Adam update against
the CPU oracle, through mt_create / mt_train_step / mt_adam_step.

Tolerances are the ones this build is held to: loss relative error <= 1e-2; per-tensor gradient
cosine >= 0.999 and relative L2 error <= 3e-2; parameters after Adam within relative L2 1e-3.
The oracle sees the unrounded fp32 parameters (in fp64); the GPU path streams their bf16 copy and
keeps activations in bf16, so these tolerances absorb that quantisation."""
import ctypes

import numpy as np
import pytest
import torch

import mt_inputs
import paper_2604_05091_amd as mt
from gpu_util import cosine, rel_l2
from mt_inputs import ModelShape
from paper_2604_05091_amd.binding import KIND_ADAM_M, KIND_ADAM_V, ModelCfg

pytestmark = pytest.mark.gpu

LOSS_RTOL, GRAD_COS, GRAD_L2, PARAM_L2 = 1e-2, 0.999, 3e-2, 1e-3


def make_cfg(shape, B, T, flags=0, **kw):
    return ModelCfg.make(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                         shape.vocab, B, T, rope_base=shape.rope_base, rms_eps=shape.rms_eps, flags=flags,
                         qkv_bias=shape.qkv_bias, tie_embeddings=shape.tie_embeddings, **kw)


def gpu_step(shape, B, T, params, tok, lab, flags=0):
    ps = [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, B, T, flags), ps) as h:
        loss = h.train_step(tok, lab)
        grads = [g.copy() for g in h.grads()]
        stats = h.stats()
    return loss, grads, stats


def check_against_oracle(orc64, shape, B, T, params, tok, lab, loss, grads):
    ref_loss, ref_grads = orc64.train_step(shape, params, tok, lab, mode=1)
    assert abs(loss - ref_loss) <= LOSS_RTOL * abs(ref_loss), (loss, ref_loss)
    for (name, _, _), g, r in zip(mt_inputs.tensor_table(shape), grads, ref_grads):
        c, e = cosine(g, r), rel_l2(g, r)
        assert c >= GRAD_COS and e <= GRAD_L2, (name, c, e)
    return ref_loss, ref_grads


def test_tiny_config_step_and_adam_match_oracle(orc64):
    shape, B, T = mt_inputs.CONFIGS["tiny"]
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=1)
    ps = [p.copy() for p in params]
    lr, b1, b2, eps = 1e-4, 0.9, 0.999, 1e-8
    with mt.TrainHandle(make_cfg(shape, B, T), ps) as h:
        loss = h.train_step(tok, lab)
        grads = [g.copy() for g in h.grads()]
        ref_loss, ref_grads = check_against_oracle(orc64, shape, B, T, params, tok, lab, loss, grads)
        h.adam_step(lr, b1, b2, eps, wd=0.0, step=1)
        # second step after the update: the refreshed bf16 copy must be what gets streamed
        loss2 = h.train_step(tok, lab)
        f = lambda x: float(np.float32(x))
        for i, (p0, g_ref) in enumerate(zip(params, ref_grads)):
            pr = p0.astype(np.float64)
            m, v = np.zeros_like(pr), np.zeros_like(pr)
            orc64.adam(pr, g_ref, m, v, f(lr), f(b1), f(b2), f(eps), 0.0, 1)
            assert rel_l2(ps[i], pr) <= PARAM_L2
            # the update itself (lr * g/(|g|+eps) at step 1): direction must agree, not only p
            assert cosine(ps[i].astype(np.float64) - p0, pr - p0) > 0.97, i
            assert rel_l2(h.tensor(i, KIND_ADAM_M), m) <= GRAD_L2
        ref_loss2 = orc64.forward_loss(shape, ps, tok, lab)
        assert abs(loss2 - ref_loss2) <= LOSS_RTOL * ref_loss2
        assert loss2 < loss            # one Adam step on the same batch lowers its loss


@pytest.mark.parametrize("shape,B,T", [
    (ModelShape(3, 128, 4, 2, 64, 344, 520), 3, 72),                      # GQA 2:1, ragged everything
    (ModelShape(2, 256, 4, 1, 128, 264, 1000, rope_base=1.0e6), 2, 136),  # head_dim 128, one KV head
], ids=["gqa-hd64", "mqa-hd128"])
def test_small_variants_match_oracle(orc64, shape, B, T):
    params = mt_inputs.make_params(shape, seed=4, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=5)
    lab = lab.copy()
    lab[0, :5] = -1                                       # ignored positions
    loss, grads, _ = gpu_step(shape, B, T, params, tok, lab)
    check_against_oracle(orc64, shape, B, T, params, tok, lab, loss, grads)


def test_pipelined_equals_serial_and_is_reproducible(orc64):
    shape, B, T = mt_inputs.CONFIGS["tiny"]
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, B, T, seed=1)
    l1, g1, s1 = gpu_step(shape, B, T, params, tok, lab)
    l2, g2, _ = gpu_step(shape, B, T, params, tok, lab)
    l3, g3, _ = gpu_step(shape, B, T, params, tok, lab, flags=mt.FLAG_SERIAL)
    assert l1 == l2 == l3
    for a, b, c in zip(g1, g2, g3):
        assert np.array_equal(a, b) and np.array_equal(a, c)
    n = mt_inputs.n_params(shape)
    per_layer = (n - 2 * shape.vocab * shape.hidden - shape.hidden) // shape.n_layers
    # weights cross the link twice per block (forward, backward) minus the last block's second load,
    # gradients once
    assert s1["d2h_bytes"] == 4 * n
    assert s1["h2d_bytes"] == 2 * (2 * n - 2 * shape.vocab * shape.hidden - shape.hidden - per_layer)
    assert s1["n_params"] == n


def test_overlapped_adam_equals_separate_calls_bitwise():
    """mt_train_step_adam (update of each unit as its gradients land) == mt_train_step + mt_adam_step."""
    shape = ModelShape(3, 128, 4, 2, 64, 344, 520)
    params = mt_inputs.make_params(shape, seed=11, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 64, seed=12)
    pa, pb = [p.copy() for p in params], [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 64), pa) as ha, mt.TrainHandle(make_cfg(shape, 2, 64), pb) as hb:
        for step in (1, 2, 3):
            la = ha.train_step(tok, lab)
            ha.adam_step(3e-4, wd=0.01, step=step)
            lb = hb.train_step_adam(tok, lab, 3e-4, wd=0.01, step=step)
            assert la == lb
            for i, (a, b) in enumerate(zip(pa, pb)):
                assert np.array_equal(a, b), (step, i)
                assert np.array_equal(ha.tensor(i, KIND_ADAM_V), hb.tensor(i, KIND_ADAM_V))
                assert np.array_equal(ha.tensor(i), hb.tensor(i))
        assert hb.stats()["adam_ms"] > 0
    assert not np.array_equal(pa[1], params[1])


def test_gradient_pieces_in_sub_ranges_give_the_same_update(monkeypatch):
    """Large gradient pieces leave in sub-ranges with a copy-done event each, and the optimizer updates each
    sub-range as it lands.  With the sub-range forced down to 1000 elements every piece of this small model is cut,
    mid-tensor and off every vector boundary; parameters and Adam moments must equal the separate-call route bitwise."""
    shape = ModelShape(3, 128, 4, 2, 64, 344, 520)
    params = mt_inputs.make_params(shape, seed=31, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 64, seed=32)
    pa, pb = [p.copy() for p in params], [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 64), pa) as ha, mt.TrainHandle(make_cfg(shape, 2, 64), pb) as hb:
        for step in (1, 2):
            monkeypatch.delenv("MT_SUBPIECE_ELEMS", raising=False)
            la = ha.train_step(tok, lab)
            ha.adam_step(3e-4, wd=0.01, step=step)
            monkeypatch.setenv("MT_SUBPIECE_ELEMS", "1000")
            lb = hb.train_step_adam(tok, lab, 3e-4, wd=0.01, step=step)
            assert la == lb
            for i, (a, b) in enumerate(zip(pa, pb)):
                assert np.array_equal(a, b), (step, i)
                assert np.array_equal(ha.tensor(i, KIND_ADAM_V), hb.tensor(i, KIND_ADAM_V)), (step, i)
                assert np.array_equal(ha.tensor(i), hb.tensor(i)), (step, i)
            ga, gb = ha.grads(), hb.grads()
            for i, (a, b) in enumerate(zip(ga, gb)):
                assert np.array_equal(a, b), (step, i)
    monkeypatch.delenv("MT_SUBPIECE_ELEMS", raising=False)


def test_gradient_slab_pool_equals_fully_pinned_gradients():
    """Gradient blocks in pageable memory behind 4 recycled pinned slabs (the paper's slab pool) must give
    the same bytes as the fully pinned layout, with and without the overlapped optimizer."""
    shape = ModelShape(6, 128, 2, 2, 64, 264, 520)          # 8 gradient blocks > 4 slabs: slabs are recycled
    params = mt_inputs.make_params(shape, seed=21, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 64, seed=22)
    la, ga, _ = gpu_step(shape, 2, 64, params, tok, lab)
    lb, gb, sb = gpu_step(shape, 2, 64, params, tok, lab, flags=mt.FLAG_GRAD_SLABS)
    assert la == lb
    for a, b in zip(ga, gb):
        assert np.array_equal(a, b)
    pa, pb = [p.copy() for p in params], [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 64), pa) as ha, \
            mt.TrainHandle(make_cfg(shape, 2, 64, flags=mt.FLAG_GRAD_SLABS), pb) as hb:
        assert hb.stats()["host_pinned_bytes"] < ha.stats()["host_pinned_bytes"]
        for step in (1, 2):
            assert ha.train_step_adam(tok, lab, 1e-3, step=step) == hb.train_step_adam(tok, lab, 1e-3, step=step)
        for i, (a, b) in enumerate(zip(pa, pb)):
            assert np.array_equal(a, b), i
            assert np.array_equal(ha.tensor(i), hb.tensor(i))


@pytest.mark.parametrize("flags", [0, mt.FLAG_GRAD_SLABS])
def test_micro_batch_accumulation_adds_gradients(orc64, flags):
    """mt_train_step then mt_train_step_accumulate on a second (differently shaped) micro-batch: every
    gradient tensor is the fp32 sum of the two separately computed gradients, bit for bit, and matches
    the sum of the oracle's two gradients; Adam afterwards uses the accumulated gradient."""
    shape = ModelShape(5, 128, 2, 2, 64, 264, 520)           # 7 gradient blocks > 4 slabs
    params = mt_inputs.make_params(shape, seed=31, std=0.05)
    t1, l1 = mt_inputs.make_batch(shape.vocab, 2, 64, seed=32)
    t2, l2 = mt_inputs.make_batch(shape.vocab, 1, 48, seed=33)
    _, g1, _ = gpu_step(shape, 2, 64, params, t1, l1)
    loss2, g2, _ = gpu_step(shape, 2, 64, params, t2, l2)
    ps = [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 64, flags=flags), ps) as h:
        with pytest.raises(mt.MtError) as e:
            h.train_step_accumulate(t2, l2)
        assert e.value.status == -8
        h.train_step(t1, l1)
        assert h.train_step_accumulate(t2, l2) == loss2
        acc = [g.copy() for g in h.grads()]
        for i, (a, x, y) in enumerate(zip(acc, g1, g2)):
            assert np.array_equal(a, x + y), i
        ref1 = orc64.train_step(shape, params, t1, l1, mode=1)[1]
        ref2 = orc64.train_step(shape, params, t2, l2, mode=1)[1]
        for i, (a, x, y) in enumerate(zip(acc, ref1, ref2)):
            r = (x + y).ravel()
            g = a.astype(np.float64).ravel()
            assert np.dot(g, r) / (np.linalg.norm(g) * np.linalg.norm(r)) > 0.999, i
            assert np.linalg.norm(g - r) / np.linalg.norm(r) < 3e-2, i
        # a fresh mt_train_step starts a new window (overwrites)
        h.train_step(t1, l1)
        for a, x in zip(h.grads(), g1):
            assert np.array_equal(a, x)
        # the optimizer consumes the accumulated gradient
        h.train_step_accumulate(t2, l2)
        h.adam_step(1e-3, step=1)
        for i, (p, p0, g) in enumerate(zip(ps, params, acc)):
            m = 0.1 * g.astype(np.float64)
            v = 0.001 * g.astype(np.float64) ** 2
            want = p0 - 1e-3 * (m / 0.1) / (np.sqrt(v / 0.001) + 1e-8)
            assert np.max(np.abs(p - want)) < 1e-6, i


@pytest.mark.parametrize("K,flags", [(1, 0), (2, mt.FLAG_STAGED_WEIGHTS)])
def test_qkv_bias_layers_match_oracle(orc64, K, flags):
    """Layers with q, k, v biases (12 tensors per layer): loss, every gradient including the bias gradients,
    and one Adam step against the oracle."""
    shape = ModelShape(3, 128, 4, 2, 64, 264, 520, qkv_bias=True)
    names = [t[0] for t in mt_inputs.tensor_table(shape)]
    assert len(names) == 12 * 3 + 3 and names[10:13] == ["l0.bq", "l0.bk", "l0.bv"]
    params = mt_inputs.make_params(shape, seed=61, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 72, seed=62)
    ps = [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 72, flags=flags, ckpt_interval=K), ps) as h:
        loss = h.train_step(tok, lab)
        grads = [g.copy() for g in h.grads()]
        check_against_oracle(orc64, shape, 2, 72, params, tok, lab, loss, grads)
        assert all(np.linalg.norm(grads[i]) > 0 for i in (10, 11, 12))
        h.adam_step(1e-3, step=1)
        for i in (10, 11, 12):      # first Adam step: p - lr * sign-like update of the bias
            want = params[i] - 1e-3 * grads[i] / (np.abs(grads[i]) + 1e-8)
            assert np.max(np.abs(ps[i] - want)) < 1e-6
        loss2 = h.train_step(tok, lab)          # the updated biases are streamed in the next step
        ref2, _ = orc64.train_step(shape, ps, tok, lab, mode=1)
        assert abs(loss2 - ref2) <= LOSS_RTOL * abs(ref2)


@pytest.mark.parametrize("K,flags", [(1, 0), (2, mt.FLAG_STAGED_WEIGHTS), (1, mt.FLAG_GRAD_SLABS), (3, mt.FLAG_SERIAL)])
def test_tied_embeddings_match_oracle(orc64, K, flags):
    """Output projection tied to the embedding table: one tensor fewer, the table streamed a second time for the
    loss, its gradient = head weight gradient + scatter-add (summed on the host).  Loss, gradients, separate and
    overlapped Adam, and micro-batch accumulation."""
    shape = ModelShape(3, 128, 4, 2, 64, 264, 520, qkv_bias=True, tie_embeddings=True)
    table = mt_inputs.tensor_table(shape)
    assert len(table) == 12 * 3 + 2 and table[-1][0] == "final_norm"
    params = mt_inputs.make_params(shape, seed=71, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 72, seed=72)
    pa, pb = [p.copy() for p in params], [p.copy() for p in params]
    with mt.TrainHandle(make_cfg(shape, 2, 72, flags=flags, ckpt_interval=K), pa) as ha, \
            mt.TrainHandle(make_cfg(shape, 2, 72, flags=flags, ckpt_interval=K), pb) as hb:
        loss = ha.train_step(tok, lab)
        grads = [g.copy() for g in ha.grads()]
        ref_loss, ref_grads = check_against_oracle(orc64, shape, 2, 72, params, tok, lab, loss, grads)
        # the table gradient really has both parts: it differs from the scatter-add alone (rows of unseen tokens)
        unseen = np.setdiff1d(np.arange(shape.vocab), tok.ravel())
        assert np.linalg.norm(grads[0][unseen]) > 0
        ha.adam_step(1e-3, step=1)
        assert hb.train_step_adam(tok, lab, 1e-3, step=1) == loss
        for i, (a, b) in enumerate(zip(pa, pb)):
            assert np.array_equal(a, b), i
        # second step sees the updated table in both of its roles
        l2 = ha.train_step(tok, lab)
        ref2, _ = orc64.train_step(shape, pa, tok, lab, mode=1)
        assert abs(l2 - ref2) <= LOSS_RTOL * abs(ref2)
        g2 = [g.copy() for g in ha.grads()]
        ha.train_step_accumulate(tok, lab)
        for i, (a, g) in enumerate(zip(ha.grads(), g2)):
            if i == 0:      # ((head + scatter) + head) + scatter: same sum, another order of fp32 additions
                assert np.allclose(a, g + g, rtol=1e-5, atol=1e-9)
            else:
                assert np.array_equal(a, g + g)


def test_chunked_mlp_matches_unchunked_and_oracle(orc64):
    """cfg.mlp_chunk: the MLP runs (and is recomputed in the backward) in token chunks, ragged last chunk.  The
    forward is row-wise identical, so the loss is bit-identical; weight gradients are sums over chunks in a
    different order; the device arena shrinks."""
    shape = ModelShape(3, 128, 2, 2, 64, 264, 520)
    params = mt_inputs.make_params(shape, seed=81, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 72, seed=82)     # 144 tokens: chunks 64 + 64 + 16

    def run(chunk, K=1, flags=0):
        ps = [p.copy() for p in params]
        with mt.TrainHandle(make_cfg(shape, 2, 72, flags=flags, ckpt_interval=K, mlp_chunk=chunk), ps) as h:
            loss = h.train_step(tok, lab)
            return loss, [g.copy() for g in h.grads()], h.stats()

    l0, g0, s0 = run(0)
    for chunk, K in ((64, 1), (64, 2), (8, 3), (144, 1), (1024, 1)):
        lc, gc, sc = run(chunk, K)
        assert lc == l0, (chunk, K)
        for i, (a, b) in enumerate(zip(g0, gc)):
            assert rel_l2(b, a) < 1e-5, (chunk, K, i)
            if chunk >= 144:        # a single chunk is the unchunked path
                assert np.array_equal(a, b), (chunk, i)
        if chunk < 144 and K == 1:
            assert sc["device_arena_bytes"] < s0["device_arena_bytes"]
    lc, gc, _ = run(64, 2, mt.FLAG_SERIAL | mt.FLAG_STAGED_WEIGHTS)
    check_against_oracle(orc64, shape, 2, 72, params, tok, lab, lc, gc)


def test_staged_weights_equal_pinned_bf16_copy():
    """MT_FLAG_STAGED_WEIGHTS: weights converted just in time into three recycled pinned slabs instead of
    being read from a persistent pinned bf16 copy.  Same bytes reach the GPU, so losses, gradients and the
    parameters after overlapped Adam steps are bit-identical; the pinned footprint is smaller."""
    shape = ModelShape(6, 128, 2, 2, 64, 264, 520)
    params = mt_inputs.make_params(shape, seed=51, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 64, seed=52)
    for K, extra in ((1, 0), (3, 0), (1, mt.FLAG_SERIAL), (2, mt.FLAG_GRAD_SLABS)):
        pa, pb = [p.copy() for p in params], [p.copy() for p in params]
        with mt.TrainHandle(make_cfg(shape, 2, 64, flags=extra, ckpt_interval=K), pa) as ha, \
                mt.TrainHandle(make_cfg(shape, 2, 64, flags=extra | mt.FLAG_STAGED_WEIGHTS, ckpt_interval=K), pb) as hb:
            assert hb.stats()["host_pinned_bytes"] < ha.stats()["host_pinned_bytes"]
            assert ha.train_step(tok, lab) == hb.train_step(tok, lab)
            for a, b in zip(ha.grads(), hb.grads()):
                assert np.array_equal(a, b)
            for step in (1, 2, 3):      # the master copy changes every step: the packer must pick it up
                assert ha.train_step_adam(tok, lab, 1e-3, step=step) == hb.train_step_adam(tok, lab, 1e-3, step=step)
            ha.adam_step(1e-3, step=4)
            hb.adam_step(1e-3, step=4)
            assert ha.train_step(tok, lab) == hb.train_step(tok, lab)
            for i, (a, b) in enumerate(zip(pa, pb)):
                assert np.array_equal(a, b), (K, i)


def test_checkpoint_interval_k_blocks(orc64):
    """Algorithm 1 with K layers per recomputation block: same kernels on the same inputs, so the loss and
    every gradient are bit-identical to K = 1; fewer checkpoints are held, more weight bytes are streamed;
    the result matches the oracle run with the same interval."""
    shape = ModelShape(5, 128, 2, 2, 64, 264, 520)
    params = mt_inputs.make_params(shape, seed=41, std=0.05)
    tok, lab = mt_inputs.make_batch(shape.vocab, 2, 72, seed=42)

    def run(K, flags=0):
        ps = [p.copy() for p in params]
        cfg = make_cfg(shape, 2, 72, flags=flags, ckpt_interval=K)
        with mt.TrainHandle(cfg, ps) as h:
            loss = h.train_step(tok, lab)
            return loss, [g.copy() for g in h.grads()], h.stats()

    l1, g1, s1 = run(1)
    for K in (2, 3, 5, 9):
        lk, gk, sk = run(K)
        assert lk == l1, K
        for i, (a, b) in enumerate(zip(g1, gk)):
            assert np.array_equal(a, b), (K, i)
        assert sk["d2h_bytes"] == s1["d2h_bytes"]
        assert sk["h2d_bytes"] >= s1["h2d_bytes"]
    l3, g3, _ = run(3, flags=mt.FLAG_SERIAL)
    assert l3 == l1 and all(np.array_equal(a, b) for a, b in zip(g1, g3))
    ref_loss, ref_grads = orc64.train_step(shape, params, tok, lab, mode=3)
    assert abs(l1 - ref_loss) <= LOSS_RTOL * abs(ref_loss)
    for g, r in zip(g3, ref_grads):
        assert cosine(g, r) >= GRAD_COS and rel_l2(g, r) <= GRAD_L2


def test_smaller_batch_than_capacity_and_error_paths(orc64):
    shape = ModelShape(2, 128, 2, 2, 64, 264, 520)
    params = mt_inputs.make_params(shape, seed=7, std=0.05)
    ps = [p.copy() for p in params]
    L = mt.lib()
    with mt.TrainHandle(make_cfg(shape, 4, 64), ps) as h:
        with pytest.raises(mt.MtError) as e:
            h.adam_step(1e-3)
        assert e.value.status == -8
        tok, lab = mt_inputs.make_batch(shape.vocab, 4, 64, seed=8)
        h.train_step(tok, lab)
        tok2, lab2 = mt_inputs.make_batch(shape.vocab, 1, 40, seed=9)     # smaller than the arena was sized for
        loss = h.train_step(tok2, lab2)
        grads = [g.copy() for g in h.grads()]
        check_against_oracle(orc64, shape, 1, 40, params, tok2, lab2, loss, grads)
        bad = tok2.copy()
        bad[0, 3] = shape.vocab
        with pytest.raises(mt.MtError) as e:
            h.train_step(bad, lab2)
        assert e.value.status == -7
        with pytest.raises(mt.MtError) as e:
            h.train_step(*mt_inputs.make_batch(shape.vocab, 5, 64))
        assert e.value.status == -6
        with pytest.raises(mt.MtError) as e:
            h.train_step(*mt_inputs.make_batch(shape.vocab, 1, 36))
        assert e.value.status == -6
        # the handle is still usable after rejected calls
        assert abs(h.train_step(tok2, lab2) - loss) == 0.0


def test_device_arena_does_not_grow_with_depth_beyond_the_checkpoints():
    """Section 4.4 (depth scaling): device memory is independent of depth apart from the h_i checkpoints."""
    sizes = {}
    for L_ in (2, 6):
        shape = ModelShape(L_, 256, 4, 4, 64, 688, 1024)
        ps = mt_inputs.make_params(shape)
        with mt.TrainHandle(make_cfg(shape, 2, 128), ps) as h:
            sizes[L_] = h.stats()["device_arena_bytes"]
    anchors = 4 * 2 * 128 * 256 * 2
    assert abs((sizes[6] - sizes[2]) - anchors) <= 4 * 256


def test_link_probe_reports_plausible_bandwidth():
    r = mt.link_probe(64 << 20, 3)
    assert 5 < r["h2d_gbs"] < 200 and 5 < r["d2h_gbs"] < 200 and r["bidir_gbs"] > max(r["h2d_gbs"], r["d2h_gbs"]) * 0.8
