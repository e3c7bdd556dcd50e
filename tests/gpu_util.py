"""Helpers for the GPU parity tests: move seeded NumPy data to device memory and back.
fp16 device tensors are made from NumPy float16 bit patterns (not through the library under test)."""
import numpy as np
import torch

from oracle import MIXED
from oracle.numerics import half_bits


def h16(x) -> torch.Tensor:
    """fp32/fp64 NumPy values -> device fp16 tensor holding RNE16(x) (rounded by NumPy)."""
    with np.errstate(over="ignore"):
        return torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.float32).astype(np.float16))).cuda()


def f32(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.float32))).cuda()


def i32(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.int32))).cuda()


def empty16(*shape) -> torch.Tensor:
    return torch.empty(shape, dtype=torch.float16, device="cuda")


def empty32(*shape) -> torch.Tensor:
    return torch.empty(shape, dtype=torch.float32, device="cuda")


def ws_bytes(n: int) -> torch.Tensor:
    return torch.empty(max(int(n), 16) // 4 + 64, dtype=torch.float32, device="cuda")


def np32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().astype(np.float32)


def bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def rel_fro(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def assert_close16(got: torch.Tensor, ref: np.ndarray, tol=1e-3, max_ulp=None, what=""):
    """Relative Frobenius error bound, plus finiteness pattern equality (inf/NaN positions must agree)."""
    g = np32(got)
    r = np.asarray(ref, np.float32)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    fin_g, fin_r = np.isfinite(g), np.isfinite(r)
    assert np.array_equal(fin_g, fin_r), f"{what}: non-finite pattern differs"
    e = rel_fro(np.where(fin_r, g, 0), np.where(fin_r, r, 0))
    assert e <= tol, f"{what}: rel Frobenius error {e:.3e} > {tol}"
    if max_ulp is not None:
        # element by element: within max_ulp fp16 units in the last place of the reference, plus an
        # absolute floor for entries that are small only through cancellation in the fp32 accumulation
        # (their error scales with the magnitude of the summed terms, not of the result).
        rr = np.where(fin_r, np.abs(r), 0).astype(np.float64)
        ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(rr, 2.0 ** -14))) - 10), 2.0 ** -24)
        bound = max_ulp * ulp + 8e-6 * rr.max(initial=0)
        diff = np.abs(np.where(fin_r, g, 0).astype(np.float64) - np.where(fin_r, r, 0))
        worst = (diff - bound).max(initial=-1)
        assert worst <= 0, f"{what}: an element is {diff.max():.3e} from the reference (bound exceeded by {worst:.3e})"
    return e
