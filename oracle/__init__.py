"""ctypes front end of the CPU oracle (oracle/mt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the GPU library or its Python binding
imports this package.

Two builds of the same C source: REAL=double (`F64`, the reference every parity
test compares against and the judge of the finite-difference pins) and
REAL=float (`F32`, the plain fp32 CPU step that the benchmark times).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mt_oracle.c")


class OrcCfg(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("hidden", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("qkv_bias", ctypes.c_int32), ("tie_embeddings", ctypes.c_int32),
                ("rope_base", ctypes.c_double),
                ("rms_eps", ctypes.c_double)]


def lib_path(real: str) -> str:
    return os.path.join(_HERE, f"libmtoracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile both precisions with gcc (-O3, OpenMP; no fast-math, no BLAS)."""
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", f"-DREAL={ctype}",
                                   "-o", out, _SRC, "-lm"])


def _cfg(shape) -> OrcCfg:
    g = shape if isinstance(shape, dict) else shape.__dict__
    return OrcCfg(g["n_layers"], g["hidden"], g["n_q_heads"], g["n_kv_heads"], g["head_dim"], g["ffn"],
                  g["vocab"], int(bool(g.get("qkv_bias", False))), int(bool(g.get("tie_embeddings", False))),
                  float(g.get("rope_base", 10000.0)),
                  float(g.get("rms_eps", 1e-5)))


class Oracle:
    """One precision of the oracle.  All arrays are numpy, C-contiguous, of self.dtype."""

    def __init__(self, real: str = "f64"):
        assert real in ("f64", "f32")
        if not os.path.exists(lib_path(real)):
            build()
        self.lib = ctypes.CDLL(lib_path(real))
        self.dtype = np.float64 if real == "f64" else np.float32
        assert self.lib.orc_real_bytes() == np.dtype(self.dtype).itemsize
        self.real = real
        L = self.lib
        vp, i64, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double
        L.orc_linear_fwd.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_linear_bwd_x.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_linear_bwd_w.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_rmsnorm_fwd.argtypes = [vp, vp, vp, i64, i64, dbl]
        L.orc_rmsnorm_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, dbl]
        L.orc_rope.argtypes = [vp, i64, i64, i64, i64, dbl, ctypes.c_int]
        L.orc_attention_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64]
        L.orc_attention_bwd.argtypes = [vp] * 7 + [i64] * 5
        L.orc_attention_row.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64]
        L.orc_attention_row.restype = None
        L.orc_attention_key_row.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64]
        L.orc_attention_key_row.restype = None
        L.orc_swiglu_fwd.argtypes = [vp, vp, vp, i64]
        L.orc_swiglu_bwd.argtypes = [vp, vp, vp, vp, vp, i64]
        L.orc_cross_entropy.argtypes = [vp, vp, vp, vp, i64, i64]
        L.orc_embed_fwd.argtypes = [vp, vp, vp, i64, i64]
        L.orc_embed_bwd.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_adam.argtypes = [vp, vp, vp, vp, i64, dbl, dbl, dbl, dbl, dbl, i64]
        L.orc_train_step.argtypes = [ctypes.POINTER(OrcCfg), vp, vp, vp, i64, i64, vp, vp, ctypes.c_int]
        L.orc_train_step.restype = ctypes.c_int
        L.orc_forward_loss.argtypes = [ctypes.POINTER(OrcCfg), vp, vp, vp, i64, i64, vp, vp, vp]
        L.orc_forward_loss.restype = ctypes.c_int
        for name in ("orc_linear_fwd", "orc_linear_bwd_x", "orc_linear_bwd_w", "orc_rmsnorm_fwd", "orc_rmsnorm_bwd",
                     "orc_rope", "orc_attention_fwd", "orc_attention_bwd", "orc_swiglu_fwd", "orc_swiglu_bwd",
                     "orc_cross_entropy", "orc_embed_fwd", "orc_embed_bwd", "orc_adam"):
            getattr(L, name).restype = None

    # -- helpers
    def arr(self, a) -> np.ndarray:
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _ptrs(self, arrays):
        return (ctypes.c_void_p * len(arrays))(*[a.ctypes.data for a in arrays])

    # -- primitive ops (each returns fresh arrays)
    def linear_fwd(self, x, w):
        x, w = self.arr(x), self.arr(w)
        y = np.empty((x.shape[0], w.shape[0]), self.dtype)
        self.lib.orc_linear_fwd(y.ctypes.data, x.ctypes.data, w.ctypes.data, x.shape[0], x.shape[1], w.shape[0])
        return y

    def linear_bwd_x(self, dy, w):
        dy, w = self.arr(dy), self.arr(w)
        dx = np.empty((dy.shape[0], w.shape[1]), self.dtype)
        self.lib.orc_linear_bwd_x(dx.ctypes.data, dy.ctypes.data, w.ctypes.data, dy.shape[0], w.shape[1], w.shape[0])
        return dx

    def linear_bwd_w(self, dy, x):
        dy, x = self.arr(dy), self.arr(x)
        dw = np.empty((dy.shape[1], x.shape[1]), self.dtype)
        self.lib.orc_linear_bwd_w(dw.ctypes.data, dy.ctypes.data, x.ctypes.data, x.shape[0], x.shape[1], dy.shape[1])
        return dw

    def rmsnorm_fwd(self, x, g, eps=1e-5):
        x, g = self.arr(x), self.arr(g)
        y = np.empty_like(x)
        self.lib.orc_rmsnorm_fwd(y.ctypes.data, x.ctypes.data, g.ctypes.data, x.shape[0], x.shape[1], eps)
        return y

    def rmsnorm_bwd(self, dy, x, g, eps=1e-5):
        dy, x, g = self.arr(dy), self.arr(x), self.arr(g)
        dx, dg = np.empty_like(x), np.empty_like(g)
        self.lib.orc_rmsnorm_bwd(dx.ctypes.data, dg.ctypes.data, dy.ctypes.data, x.ctypes.data, g.ctypes.data,
                                 x.shape[0], x.shape[1], eps)
        return dx, dg

    def rope(self, x, B, T, H, hd, base=10000.0, sign=1):
        """x: [B*T, H*hd]; returns the rotated copy."""
        y = self.arr(x).copy()
        assert y.size == B * T * H * hd
        self.lib.orc_rope(y.ctypes.data, B, T, H, hd, base, sign)
        return y

    def attention_fwd(self, q, k, v, B, T, Hq, Hkv, hd):
        q, k, v = self.arr(q), self.arr(k), self.arr(v)
        a = np.empty_like(q)
        self.lib.orc_attention_fwd(a.ctypes.data, q.ctypes.data, k.ctypes.data, v.ctypes.data, B, T, Hq, Hkv, hd)
        return a

    def attention_bwd(self, da, q, k, v, B, T, Hq, Hkv, hd):
        da, q, k, v = self.arr(da), self.arr(q), self.arr(k), self.arr(v)
        dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
        self.lib.orc_attention_bwd(dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, da.ctypes.data, q.ctypes.data,
                                   k.ctypes.data, v.ctypes.data, B, T, Hq, Hkv, hd)
        return dq, dk, dv

    def attention_row(self, q, da, k, v):
        """One query row: q, da [hd]; k, v [n_keys, hd] (the keys visible to it).  Returns (a, dq)."""
        q, da, k, v = self.arr(q), self.arr(da), self.arr(k), self.arr(v)
        a, dq = np.empty_like(q), np.empty_like(q)
        self.lib.orc_attention_row(a.ctypes.data, dq.ctypes.data, q.ctypes.data, da.ctypes.data, k.ctypes.data,
                                   v.ctypes.data, k.shape[0], k.shape[1])
        return a, dq

    def attention_key_row(self, q, da, k, v, u):
        """One key row of one head of one sequence: q, da, k, v [T, hd]; returns (dk_u, dv_u), the gradients key u
        and its value receive from the queries u .. T-1."""
        q, da, k, v = self.arr(q), self.arr(da), self.arr(k), self.arr(v)
        assert q.shape == da.shape == k.shape == v.shape and 0 <= u < q.shape[0]
        dk, dv = np.empty(q.shape[1], self.dtype), np.empty(q.shape[1], self.dtype)
        self.lib.orc_attention_key_row(dk.ctypes.data, dv.ctypes.data, q.ctypes.data, da.ctypes.data, k.ctypes.data,
                                       v.ctypes.data, q.shape[0], q.shape[1], u)
        return dk, dv

    def swiglu_fwd(self, gate, up):
        gate, up = self.arr(gate), self.arr(up)
        s = np.empty_like(gate)
        self.lib.orc_swiglu_fwd(s.ctypes.data, gate.ctypes.data, up.ctypes.data, gate.size)
        return s

    def swiglu_bwd(self, ds, gate, up):
        ds, gate, up = self.arr(ds), self.arr(gate), self.arr(up)
        dg, du = np.empty_like(gate), np.empty_like(up)
        self.lib.orc_swiglu_bwd(dg.ctypes.data, du.ctypes.data, ds.ctypes.data, gate.ctypes.data, up.ctypes.data,
                                gate.size)
        return dg, du

    def cross_entropy(self, logits, labels):
        logits = self.arr(logits)
        labels = np.ascontiguousarray(labels, dtype=np.int32).reshape(-1)
        loss = np.zeros(1, self.dtype)
        dl = np.empty_like(logits)
        self.lib.orc_cross_entropy(loss.ctypes.data, dl.ctypes.data, logits.ctypes.data, labels.ctypes.data,
                                   logits.shape[0], logits.shape[1])
        return float(loss[0]), dl

    def embed_fwd(self, table, tokens):
        table = self.arr(table)
        tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(-1)
        h = np.empty((tokens.size, table.shape[1]), self.dtype)
        self.lib.orc_embed_fwd(h.ctypes.data, table.ctypes.data, tokens.ctypes.data, tokens.size, table.shape[1])
        return h

    def embed_bwd(self, dh, tokens, V):
        dh = self.arr(dh)
        tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(-1)
        dt = np.empty((V, dh.shape[1]), self.dtype)
        self.lib.orc_embed_bwd(dt.ctypes.data, dh.ctypes.data, tokens.ctypes.data, tokens.size, V, dh.shape[1])
        return dt

    def adam(self, p, g, m, v, lr, b1, b2, eps, wd, t):
        """In place on p, m, v (arrays of self.dtype)."""
        for a in (p, g, m, v):
            assert a.dtype == self.dtype and a.flags["C_CONTIGUOUS"]
        self.lib.orc_adam(p.ctypes.data, g.ctypes.data, m.ctypes.data, v.ctypes.data, p.size, lr, b1, b2, eps, wd, t)

    # -- the step
    def train_step(self, shape, params, tokens, labels, mode: int = 1):
        """Returns (loss, grads) with grads in canonical tensor order; mode 0 monolithic, 1 streamed."""
        cfg = _cfg(shape)
        ps = [self.arr(p) for p in params]
        assert len(ps) == (12 if cfg.qkv_bias else 9) * cfg.n_layers + (2 if cfg.tie_embeddings else 3)
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        B, T = tokens.shape
        grads = [np.empty_like(p) for p in ps]
        loss = np.zeros(1, self.dtype)
        rc = self.lib.orc_train_step(ctypes.byref(cfg), self._ptrs(ps), tokens.ctypes.data, labels.ctypes.data, B, T,
                                     self._ptrs(grads), loss.ctypes.data, mode)
        if rc != 0:
            raise ValueError("token or label outside the vocabulary")
        return float(loss[0]), grads

    def forward_loss(self, shape, params, tokens, labels, want_logits=False):
        cfg = _cfg(shape)
        ps = [self.arr(p) for p in params]
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        B, T = tokens.shape
        loss = np.zeros(1, self.dtype)
        logits = np.empty((B * T, cfg.vocab), self.dtype) if want_logits else None
        rc = self.lib.orc_forward_loss(ctypes.byref(cfg), self._ptrs(ps), tokens.ctypes.data, labels.ctypes.data, B, T,
                                       loss.ctypes.data, logits.ctypes.data if want_logits else None, None)
        if rc != 0:
            raise ValueError("token or label outside the vocabulary")
        return (float(loss[0]), logits) if want_logits else float(loss[0])
