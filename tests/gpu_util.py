"""Helpers for the GPU parity tests: torch is used only to hold device memory."""
import numpy as np
import torch

import paper_2604_05091_amd as mt


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 array rounded to the nearest bf16 (returned as float32)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def dev_bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda().contiguous()


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().contiguous()


def dev_i32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda().contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.float().cpu().numpy().astype(np.float64)


def ok(status: int) -> None:
    mt.binding.check(status)
    torch.cuda.synchronize()


def rel_l2(a, ref) -> float:
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


def cosine(a, ref) -> float:
    a, ref = np.asarray(a, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    return float(a @ ref / max(np.linalg.norm(a) * np.linalg.norm(ref), 1e-300))


def rows_close(got, ref, frac, afrac=0.0, width=None):
    """Per-row bound: every element of a row is within frac * (largest |ref| of that row) + afrac * (largest |ref|
    of the tensor).  A tensor norm hides one wrong row among thousands; this does not.  width: split the rows into
    segments of that many columns first (e.g. one attention head).  Returns the worst error / bound ratio."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if width is not None:
        got, ref = got.reshape(-1, width), ref.reshape(-1, width)
    elif got.ndim == 1:
        got, ref = got[None, :], ref[None, :]
    bound = frac * np.abs(ref).max(axis=1) + afrac * np.abs(ref).max()
    err = np.abs(got - ref).max(axis=1)
    return float(np.max(err / np.maximum(bound, 1e-300)))


def assert_rows_close(got, ref, frac, afrac=0.0, width=None, what=""):
    worst = rows_close(got, ref, frac, afrac, width)
    assert worst <= 1.0, f"{what}: worst row is {worst:.2f} x its bound (frac {frac}, afrac {afrac})"
