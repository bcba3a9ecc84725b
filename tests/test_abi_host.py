"""CPU-side checks of the product library: it loads, exports every declared symbol, rejects bad
arguments before touching a GPU, and its host arithmetic (Adam, bf16 rounding, rotary tables)
matches the oracle.  No GPU compute is launched here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2604_05091_amd as mt
from paper_2604_05091_amd.binding import ModelCfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for hdr in ("megatrain.h", "megatrain_kernels.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(mt_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(mt.lib_path())
    syms = declared_symbols()
    assert len(syms) >= 30
    for s in syms:
        assert hasattr(L, s), f"{s} is declared in include/ but not exported"


def test_tensor_table_matches_the_input_module():
    import mt_inputs
    L = mt.lib()
    for name in ("tiny", "14B"):
        shape, B, T = mt_inputs.CONFIGS[name]
        cfg = ModelCfg.make(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                            shape.vocab, B, T)
        n = ctypes.c_int32()
        assert L.mt_tensor_count(ctypes.byref(cfg), ctypes.byref(n)) == 0
        table = mt_inputs.tensor_table(shape)
        assert n.value == len(table) == 9 * shape.n_layers + 3
        for i, (nm, r, c) in enumerate(table):
            rr, cc, p = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_char_p()
            assert L.mt_tensor_info(ctypes.byref(cfg), i, ctypes.byref(rr), ctypes.byref(cc), ctypes.byref(p)) == 0
            assert (p.value.decode(), rr.value, cc.value) == (nm, r, c)
        assert L.mt_tensor_info(ctypes.byref(cfg), n.value, ctypes.byref(rr), ctypes.byref(cc), None) == -1


def test_create_rejects_bad_configurations_without_a_gpu():
    L = mt.lib()
    h = ctypes.c_void_p()
    good = dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688, vocab=1024, max_batch=2,
                max_seq=128)
    dummy = (ctypes.c_void_p * 21)(*([1] * 21))

    def create(**kw):
        cfg = ModelCfg.make(**{**good, **kw})
        return L.mt_create(ctypes.byref(cfg), dummy, ctypes.byref(h))

    assert L.mt_create(None, dummy, ctypes.byref(h)) == -1
    assert create(n_layers=0) == -1
    assert create(n_q_heads=4, n_kv_heads=3) == -1
    assert create(head_dim=96) == -2
    assert create(ffn=690) == -2
    assert create(ckpt_interval=0) == -1
    assert create(max_seq=100) == -2
    assert create(rms_eps=0.0) == -1
    cfg = ModelCfg.make(**good)
    cfg.struct_size = 8
    assert L.mt_create(ctypes.byref(cfg), dummy, ctypes.byref(h)) == -1
    cfg = ModelCfg.make(**good)
    assert L.mt_create(ctypes.byref(cfg), None, ctypes.byref(h)) == -1
    assert b"host_param_ptrs" in L.mt_last_error()
    # the arena plan is checked against the cap before any device call
    assert create(max_device_bytes=1 << 20) == -4
    assert b"device arena" in L.mt_last_error()
    assert L.mt_destroy(None) == 0
    assert L.mt_adam_step(None, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1) == -1
    assert L.mt_train_step(None, None, None, 1, 8, None) == -1


def test_host_adam_matches_oracle(orc64):
    L = mt.lib()
    rng = np.random.default_rng(0)
    n = 200_003                                  # several thread chunks and a ragged tail
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    pr, mr, vr = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    shadow = np.zeros(n, np.uint16)
    for t, wd in ((1, 0.0), (2, 0.01), (3, 0.01)):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        assert L.mt_k_host_adam(p.ctypes.data, g.ctypes.data, m.ctypes.data, v.ctypes.data, shadow.ctypes.data, n,
                                1e-4, 0.9, 0.999, 1e-8, wd, t) == 0
        # the C ABI takes float arguments: give the oracle the same (float-rounded) hyper-parameters
        f = lambda x: float(np.float32(x))
        orc64.adam(pr, g.astype(np.float64), mr, vr, f(1e-4), f(0.9), f(0.999), f(1e-8), f(wd), t)
    assert np.linalg.norm(p - pr) / np.linalg.norm(pr) < 1e-6
    upd, upd_ref = p.astype(np.float64) - p0, pr - p0
    assert np.linalg.norm(upd - upd_ref) / np.linalg.norm(upd_ref) < 1e-4     # the update itself, not just p
    assert np.linalg.norm(m - mr) / np.linalg.norm(mr) < 1e-6 and np.linalg.norm(v - vr) / np.linalg.norm(vr) < 1e-6
    # the bf16 copy is the updated parameter rounded to nearest even
    import torch
    ref_bits = torch.from_numpy(p).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(shadow, ref_bits)
    assert L.mt_k_host_adam(p.ctypes.data, g.ctypes.data, m.ctypes.data, v.ctypes.data, None, n, 1e-4, 0.9, 0.999,
                            1e-8, 0.0, 0) == -1


def test_host_adam_from_two_threads_at_once_equals_one_at_a_time():
    """The host pool runs one job at a time; a caller that finds it busy (the optimizer thread next to the weight
    packing thread) spawns threads of its own.  Both take chunks from a shared counter.  Two updates issued at the
    same moment must give, bit for bit, what the same updates give one after the other."""
    import threading
    L = mt.lib()
    rng = np.random.default_rng(5)
    n = 3_000_017                                # ~46 chunks of 65536 with a ragged tail
    def fresh(seed):
        r = np.random.default_rng(seed)
        return [(r.standard_normal(n) * 0.02).astype(np.float32), (r.standard_normal(n) * 1e-3).astype(np.float32),
                np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)]
    def run(a, reps):
        for t in range(1, reps + 1):
            assert L.mt_k_host_adam(a[0].ctypes.data, a[1].ctypes.data, a[2].ctypes.data, a[3].ctypes.data,
                                    a[4].ctypes.data, n, 1e-3, 0.9, 0.999, 1e-8, 0.01, t) == 0
    ref = [fresh(1), fresh(2)]
    for a in ref:
        run(a, 3)
    got = [fresh(1), fresh(2)]
    th = [threading.Thread(target=run, args=(a, 3)) for a in got]
    for t in th:
        t.start()
    for t in th:
        t.join()
    for a, b in zip(ref, got):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    assert not np.array_equal(got[0][0], fresh(1)[0])


def test_host_bf16_rounding_is_nearest_even():
    import torch
    L = mt.lib()
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(100_000).astype(np.float32) * 10,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.4e38, 1e-40, np.inf, -np.inf], np.float32)])
    out = np.zeros(x.size, np.uint16)
    assert L.mt_k_host_f32_to_bf16(out.ctypes.data, x.ctypes.data, x.size) == 0
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(out, ref)


@pytest.mark.parametrize("hd,base", [(64, 10000.0), (128, 1.0e6)])
def test_rope_table_matches_oracle_rotation(orc64, hd, base):
    """cos/sin at (t, j) must be what the oracle's rotation does to the unit vector of pair j."""
    L = mt.lib()
    T = 4096
    cs, sn = np.empty((T, hd // 2), np.float32), np.empty((T, hd // 2), np.float32)
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, hd, base) == 0
    x = np.zeros((T, hd))
    x[:, : hd // 2] = 1.0
    y = orc64.rope(x, 1, T, 1, hd, base, +1)
    assert np.max(np.abs(y[:, : hd // 2] - cs)) < 6e-8 and np.max(np.abs(y[:, hd // 2:] - sn)) < 6e-8
    assert L.mt_k_rope_table(cs.ctypes.data, sn.ctypes.data, T, 63, base) == -1


def test_model_flops_formula_reproduces_the_paper_rows():
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "paper_table7_flops.txt"))
            if l.strip() and not l.startswith("#")]
    for ctx, bs, secs, tflops in rows:
        f = mt.model_flops(n_params=7.62e9, n_layers=28, hidden=3584, batch=int(bs), seq=int(ctx))
        assert abs(f / float(secs) / 1e12 / float(tflops) - 1) < 0.015, (ctx, f / float(secs) / 1e12, tflops)
