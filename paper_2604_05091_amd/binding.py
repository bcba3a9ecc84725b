"""ctypes binding of include/megatrain.h and include/megatrain_kernels.h.

Argument marshalling only: every step of the training path runs inside the library.
Functions keep the C names (`lib().mt_train_step`, `lib().mt_k_gemm_nt`, ...); `TrainHandle`
is a convenience wrapper that owns an mt_handle and numpy views of its host tensors.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t, c_uint16, c_uint32, c_uint64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

STATUS_NAMES = {0: "MT_OK", -1: "MT_ERR_INVALID_ARG", -2: "MT_ERR_UNSUPPORTED", -3: "MT_ERR_HOST_OOM",
                -4: "MT_ERR_DEVICE_OOM", -5: "MT_ERR_HIP", -6: "MT_ERR_SHAPE", -7: "MT_ERR_TOKEN_RANGE",
                -8: "MT_ERR_STATE"}
FLAG_SERIAL, FLAG_COMPUTE_ONLY, FLAG_COPY_ONLY, FLAG_KERNEL_TIMING, FLAG_GRAD_SLABS = 1, 2, 4, 8, 16
FLAG_STAGED_WEIGHTS = 32
KIND_GRAD, KIND_ADAM_M, KIND_ADAM_V = 0, 1, 2
ABI_VERSION = 2


class MtError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class ModelCfg(ctypes.Structure):
    _fields_ = [("struct_size", c_uint32), ("abi_version", c_uint32),
                ("n_layers", c_int32), ("hidden", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32),
                ("head_dim", c_int32), ("ffn", c_int32), ("vocab", c_int32),
                ("max_batch", c_int32), ("max_seq", c_int32),
                ("rope_base", c_float), ("rms_eps", c_float),
                ("ckpt_interval", c_int32), ("device_id", c_int32), ("flags", c_uint32), ("qkv_bias", c_uint32),
                ("max_device_bytes", c_uint64), ("tie_embeddings", c_uint32), ("mlp_chunk", c_uint32)]

    @classmethod
    def make(cls, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, max_batch, max_seq,
             rope_base=10000.0, rms_eps=1e-5, ckpt_interval=1, device_id=0, flags=0, max_device_bytes=0, qkv_bias=False,
             tie_embeddings=False, mlp_chunk=0):
        return cls(ctypes.sizeof(cls), ABI_VERSION, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                   max_batch, max_seq, rope_base, rms_eps, ckpt_interval, device_id, flags, int(bool(qkv_bias)),
                   max_device_bytes, int(bool(tie_embeddings)), int(mlp_chunk))


class Stats(ctypes.Structure):
    _fields_ = [("step_ms", c_double), ("adam_ms", c_double),
                ("compute_busy_ms", c_double), ("h2d_busy_ms", c_double), ("d2h_busy_ms", c_double),
                ("h2d_hidden_ms", c_double), ("d2h_hidden_ms", c_double),
                ("h2d_bytes", c_uint64), ("d2h_bytes", c_uint64),
                ("device_arena_bytes", c_uint64), ("host_pinned_bytes", c_uint64), ("host_pageable_bytes", c_uint64),
                ("n_params", c_uint64), ("steps_done", c_uint64),
                ("class_ms", c_double * 3), ("class_flops", c_double * 3), ("class_launches", c_uint64 * 3), ("class_bytes", c_double * 3)]

    def dict(self):
        out = {}
        for k, _ in self._fields_:
            v = getattr(self, k)
            out[k] = list(v) if hasattr(v, "__len__") else v
        return out


def lib_path() -> str:
    return os.path.join(_HERE, "libmegatrain_mi355.so")


def lib():
    """Load the built library.  Raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2604_05091_amd.build`")
    L = ctypes.CDLL(path)
    p16, pf, pi = c_void_p, c_void_p, c_void_p  # device or host pointers travel as integers
    sig = {
        "mt_tensor_count": ([POINTER(ModelCfg), POINTER(c_int32)], c_int32),
        "mt_tensor_info": ([POINTER(ModelCfg), c_int32, POINTER(c_int64), POINTER(c_int64), POINTER(c_char_p)], c_int32),
        "mt_create": ([POINTER(ModelCfg), POINTER(c_void_p), POINTER(c_void_p)], c_int32),
        "mt_train_step": ([c_void_p, c_void_p, c_void_p, c_int32, c_int32, POINTER(c_float)], c_int32),
        "mt_adam_step": ([c_void_p, c_float, c_float, c_float, c_float, c_float, c_int64], c_int32),
        "mt_train_step_adam": ([c_void_p, c_void_p, c_void_p, c_int32, c_int32, POINTER(c_float), c_float, c_float,
                                c_float, c_float, c_float, c_int64], c_int32),
        "mt_train_step_accumulate": ([c_void_p, c_void_p, c_void_p, c_int32, c_int32, POINTER(c_float)], c_int32),
        "mt_refresh_shadow": ([c_void_p], c_int32),
        "mt_get_tensor": ([c_void_p, c_int32, c_int32, POINTER(c_void_p), POINTER(c_size_t)], c_int32),
        "mt_get_stats": ([c_void_p, POINTER(Stats)], c_int32),
        "mt_destroy": ([c_void_p], c_int32),
        "mt_host_alloc": ([c_size_t], c_void_p),
        "mt_host_free": ([c_void_p], None),
        "mt_last_error": ([], c_char_p),
        "mt_device_count": ([], c_int32),
        "mt_device_synchronize": ([c_int32], c_int32),
        "mt_link_probe": ([c_int32, c_size_t, c_int32, POINTER(c_double), POINTER(c_double), POINTER(c_double)], c_int32),
        # kernels
        "mt_k_gemm_nt": ([p16, c_int64, p16, c_int64, c_void_p, c_int64, p16, c_int64, c_int32, c_int32, c_int32,
                          c_int32, c_int32, c_void_p], c_int32),
        "mt_k_transpose": ([p16, p16, c_int32, c_int32, c_int64, c_int64, c_int32, c_int32, c_int64, c_int64, c_int64,
                            c_int64, c_void_p], c_int32),
        "mt_k_rmsnorm_fwd": ([p16, p16, p16, c_int64, c_int32, c_float, c_void_p], c_int32),
        "mt_k_rmsnorm_bwd_ws_bytes": ([c_int32], c_size_t),
        "mt_k_rmsnorm_bwd": ([p16, pf, p16, p16, p16, p16, c_void_p, c_int64, c_int32, c_float, c_void_p], c_int32),
        "mt_k_rmsnorm_bwd_noalloc": ([p16, pf, p16, p16, p16, p16, c_int64, c_int32, c_float, c_void_p], c_int32),
        "mt_k_rope_table": ([pf, pf, c_int32, c_int32, c_double], c_int32),
        "mt_k_rope": ([p16, c_int64, c_int64, c_int32, c_int32, c_int32, pf, pf, c_int32, c_void_p], c_int32),
        "mt_k_swiglu_fwd": ([p16, p16, c_int64, c_int32, c_void_p], c_int32),
        "mt_k_swiglu_bwd": ([p16, p16, p16, c_int64, c_int32, c_void_p], c_int32),
        "mt_k_embed_gather": ([p16, p16, pi, c_int64, c_int32, c_void_p], c_int32),
        "mt_k_embed_scatter": ([pf, p16, pi, pi, c_int32, c_int32, c_void_p], c_int32),
        "mt_k_cross_entropy": ([pf, p16, pf, pi, c_int64, c_int32, c_float, c_void_p], c_int32),
        "mt_k_reduce_sum": ([pf, pf, c_int64, c_float, c_int32, c_void_p], c_int32),
        "mt_k_gemm_nt_bias": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int32, c_int32, c_int32, c_void_p], c_int32),
        "mt_k_gemm_nt_rope": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, pf, pf, c_int32, c_int32, c_int32, c_int32,
                               c_int32, c_void_p], c_int32),
        "mt_k_flash_bwd_rope": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16,
                                 c_int64, p16, c_int64, pf, pf, pf, pf, c_int32, c_int32, c_int32, c_int32, c_int32,
                                 c_float, c_void_p], c_int32),
        "mt_k_gemm_nt_swiglu": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, c_int32, c_int32, c_int32, c_void_p],
                                c_int32),
        "mt_k_gemm_nt_swiglu_bwd": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, c_int32, c_int32, c_int32,
                                     c_void_p], c_int32),
        "mt_k_gemm_tn": ([p16, c_int64, p16, c_int64, pf, c_int64, c_int32, c_int32, c_int32, c_int32, c_void_p], c_int32),
        "mt_k_gemm_tn_split": ([p16, c_int64, p16, c_int64, pf, c_int64, c_int32, c_int32, c_int32, c_int32, c_int32, pf,
                                c_void_p], c_int32),
        "mt_k_gemm_tn_pick_split": ([c_int64, c_int64, c_int64, c_int32], c_int32),
        "mt_k_bias_grad_ws_bytes": ([c_int32], c_size_t),
        "mt_k_bias_grad": ([pf, p16, c_int64, c_int64, c_int32, c_void_p, c_void_p], c_int32),
        "mt_k_flash_fwd": ([p16, c_int64, pf, p16, c_int64, p16, c_int64, p16, c_int64, c_int32, c_int32, c_int32,
                            c_int32, c_int32, c_float, c_void_p], c_int32),
        "mt_k_flash_bwd": ([p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16, c_int64, p16,
                            c_int64, p16, c_int64, pf, pf, c_int32, c_int32, c_int32, c_int32, c_int32, c_float,
                            c_void_p], c_int32),
        "mt_k_host_adam": ([pf, pf, pf, pf, p16, c_size_t, c_float, c_float, c_float, c_float, c_float, c_int64], c_int32),
        "mt_k_host_f32_to_bf16": ([p16, pf, c_size_t], c_int32),
    }
    for name, (args, res) in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = res
    _LIB = L
    return L


def check(status: int) -> None:
    if status != 0:
        raise MtError(status, (lib().mt_last_error() or b"").decode())


def model_flops(n_params: int, n_layers: int, hidden: int, batch: int, seq: int) -> float:
    """Model FLOPs of one step by the paper's accounting (caption of its long-context table):
    6 N D + 12 L H T^2 per sequence, with N all parameters, D = batch*seq tokens; full (non-causal)
    attention is counted and recomputation is not."""
    return 6.0 * n_params * batch * seq + 12.0 * n_layers * hidden * float(seq) ** 2 * batch


def device_count() -> int:
    return lib().mt_device_count()


def device_synchronize(device_id: int = 0) -> None:
    check(lib().mt_device_synchronize(device_id))


def link_probe(nbytes: int = 256 << 20, reps: int = 4, device_id: int = 0):
    a, b, c = c_double(), c_double(), c_double()
    check(lib().mt_link_probe(device_id, nbytes, reps, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return {"h2d_gbs": a.value, "d2h_gbs": b.value, "bidir_gbs": c.value}


class TrainHandle:
    """Owns an mt_handle.  `params` is the list of caller-owned fp32 numpy arrays in canonical order
    (they are updated in place by adam_step and must stay alive as long as the handle)."""

    def __init__(self, cfg: ModelCfg, params):
        self.cfg = cfg
        self.params = [p for p in params]
        for p in self.params:
            assert p.dtype == np.float32 and p.flags["C_CONTIGUOUS"]
        n = c_int32()
        check(lib().mt_tensor_count(ctypes.byref(cfg), ctypes.byref(n)))
        assert n.value == len(self.params), (n.value, len(self.params))
        ptrs = (c_void_p * len(self.params))(*[p.ctypes.data for p in self.params])
        h = c_void_p()
        check(lib().mt_create(ctypes.byref(cfg), ptrs, ctypes.byref(h)))
        self._h = h

    def train_step(self, tokens: np.ndarray, labels: np.ndarray) -> float:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        assert tokens.shape == labels.shape and tokens.ndim == 2
        loss = c_float()
        check(lib().mt_train_step(self._h, tokens.ctypes.data, labels.ctypes.data, tokens.shape[0], tokens.shape[1],
                                  ctypes.byref(loss)))
        return loss.value

    def train_step_accumulate(self, tokens: np.ndarray, labels: np.ndarray) -> float:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        assert tokens.shape == labels.shape and tokens.ndim == 2
        loss = c_float()
        check(lib().mt_train_step_accumulate(self._h, tokens.ctypes.data, labels.ctypes.data, tokens.shape[0],
                                             tokens.shape[1], ctypes.byref(loss)))
        return loss.value

    def train_step_adam(self, tokens: np.ndarray, labels: np.ndarray, lr, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0,
                        step=1) -> float:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        assert tokens.shape == labels.shape and tokens.ndim == 2
        loss = c_float()
        check(lib().mt_train_step_adam(self._h, tokens.ctypes.data, labels.ctypes.data, tokens.shape[0],
                                       tokens.shape[1], ctypes.byref(loss), lr, beta1, beta2, eps, wd, step))
        return loss.value

    def adam_step(self, lr, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, step=1) -> None:
        check(lib().mt_adam_step(self._h, lr, beta1, beta2, eps, wd, step))

    def refresh_shadow(self) -> None:
        check(lib().mt_refresh_shadow(self._h))

    def tensor(self, idx: int, kind: int = KIND_GRAD) -> np.ndarray:
        """Borrowed numpy view of a library-owned host array (valid until close())."""
        p, n = c_void_p(), c_size_t()
        check(lib().mt_get_tensor(self._h, idx, kind, ctypes.byref(p), ctypes.byref(n)))
        buf = (c_float * n.value).from_address(p.value)
        return np.frombuffer(buf, dtype=np.float32).reshape(self.params[idx].shape)

    def grads(self):
        return [self.tensor(i, KIND_GRAD) for i in range(len(self.params))]

    def stats(self) -> dict:
        s = Stats()
        check(lib().mt_get_stats(self._h, ctypes.byref(s)))
        return s.dict()

    def close(self) -> None:
        if self._h is not None and self._h.value:
            lib().mt_destroy(self._h)
        self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
