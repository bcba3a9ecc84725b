"""Seeded synthetic inputs (weights, tokens) shared by the tests, the benchmark and the oracle checks.

This package holds none of the training method's arithmetic: it produces
reproducible random arrays and the table of tensor shapes of a decoder-only
model, nothing else.  Both the CPU oracle and the GPU library are fed from here
so that they see identical bytes while sharing no code of their own.

Recipe (the synthetic stand-in for the fine-tuning batches of the paper's
evaluation, Section 4.1): matrices and embeddings are i.i.d. N(0, 0.02) in fp32,
RMSNorm gains are 1.0, tokens are i.i.d. uniform over the vocabulary with T+1
draws per row so that labels are the inputs shifted by one position.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, asdict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmtinputs.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.c into libmtinputs.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.mti_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_uint64,
                                        ctypes.c_float, ctypes.c_float]
        lib.mti_fill_normal.restype = None
        lib.mti_fill_const.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float]
        lib.mti_fill_const.restype = None
        lib.mti_fill_tokens.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_uint64,
                                        ctypes.c_int32]
        lib.mti_fill_tokens.restype = None
        _lib = lib
    return _lib


@dataclass(frozen=True)
class ModelShape:
    """Architecture of a decoder-only LM (pre-norm, RMSNorm, RoPE, SwiGLU).  qkv_bias adds a bias vector to the
    q, k and v projections (three more tensors per layer, after w_down); tie_embeddings makes the output
    projection reuse the embedding table (the lm_head tensor disappears from the table)."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    qkv_bias: bool = False
    tie_embeddings: bool = False

    def dict(self):
        return asdict(self)


# The five workloads (model shape, batch, seq) of this build.
CONFIGS = {
    "tiny": (ModelShape(2, 256, 4, 4, 64, 688, 1024), 2, 128),
    "1.3B": (ModelShape(24, 2048, 16, 16, 128, 5504, 32000), 8, 2048),
    "7B": (ModelShape(32, 4096, 32, 32, 128, 11008, 32000), 16, 4096),
    "14B": (ModelShape(48, 5120, 40, 8, 128, 13824, 32000, rope_base=1.0e6), 16, 4096),
    "7B-128k": (ModelShape(32, 4096, 32, 32, 128, 11008, 32000), 1, 131072),
}
# Longer contexts of the paper's long-context table (Section 4.6), beyond the five workloads above.
LONG_CONTEXT = {
    "7B-256k": (ModelShape(32, 4096, 32, 32, 128, 11008, 32000), 1, 262144),
    "7B-512k": (ModelShape(32, 4096, 32, 32, 128, 11008, 32000), 1, 524288),
}


def tensor_table(s: ModelShape):
    """Canonical tensor order: (name, rows, cols) for the 9L+3 (12L+3 with qkv_bias; one fewer with tie_embeddings)
    parameter tensors.

    Matrices are row-major [out_features, in_features]; a vector of n elements is reported as (rows=n, cols=1).
    """
    nq, nkv = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    t = [("embed", s.vocab, s.hidden)]
    for l in range(s.n_layers):
        t += [(f"l{l}.attn_norm", s.hidden, 1), (f"l{l}.wq", nq, s.hidden), (f"l{l}.wk", nkv, s.hidden),
              (f"l{l}.wv", nkv, s.hidden), (f"l{l}.wo", s.hidden, nq), (f"l{l}.mlp_norm", s.hidden, 1),
              (f"l{l}.w_gate", s.ffn, s.hidden), (f"l{l}.w_up", s.ffn, s.hidden),
              (f"l{l}.w_down", s.hidden, s.ffn)]
        if s.qkv_bias:
            t += [(f"l{l}.bq", nq, 1), (f"l{l}.bk", nkv, 1), (f"l{l}.bv", nkv, 1)]
    t += [("final_norm", s.hidden, 1)]
    if not s.tie_embeddings:
        t += [("lm_head", s.vocab, s.hidden)]
    return t


def n_params(s: ModelShape) -> int:
    return sum(r * c for _, r, c in tensor_table(s))


def fill_normal(out: np.ndarray, seed: int, stream_id: int, mean: float = 0.0, std: float = 1.0) -> None:
    assert out.dtype == np.float32 and out.flags["C_CONTIGUOUS"]
    _load().mti_fill_normal(out.ctypes.data, out.size, seed, stream_id, mean, std)


def normal(shape, seed: int, stream_id: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    fill_normal(out, seed, stream_id, mean, std)
    return out


def fill_param(out: np.ndarray, name: str, idx: int, seed: int = 0, std: float = 0.02) -> None:
    """Fill tensor number idx of the canonical order: gains 1.0, everything else N(0, std)."""
    assert out.dtype == np.float32 and out.flags["C_CONTIGUOUS"]
    if name.endswith("norm"):
        _load().mti_fill_const(out.ctypes.data, out.size, 1.0)
    else:
        _load().mti_fill_normal(out.ctypes.data, out.size, seed, idx, 0.0, std)


def make_params(s: ModelShape, seed: int = 0, std: float = 0.02, alloc=None):
    """List of fp32 arrays in canonical order.  alloc(nbytes-shaped request) may supply the storage:
    alloc(shape) -> np.ndarray(float32)."""
    out = []
    for idx, (name, r, c) in enumerate(tensor_table(s)):
        shape = (r,) if c == 1 else (r, c)
        a = np.empty(shape, dtype=np.float32) if alloc is None else alloc(shape)
        fill_param(a, name, idx, seed, std)
        out.append(a)
    return out


def make_batch(vocab: int, batch: int, seq: int, seed: int = 1, stream_id: int = 0):
    """tokens, labels int32 [batch, seq]; labels are the next token (T+1 draws per row)."""
    raw = np.empty((batch, seq + 1), dtype=np.int32)
    _load().mti_fill_tokens(raw.ctypes.data, raw.size, seed, stream_id, vocab)
    return np.ascontiguousarray(raw[:, :-1]), np.ascontiguousarray(raw[:, 1:])
