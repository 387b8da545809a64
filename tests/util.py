"""Helpers shared by the tests: bf16 <-> bit patterns and error metrics (no method arithmetic)."""
import numpy as np
import torch


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """torch bf16 tensor (any device) -> uint16 numpy array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    return float(num / den) if den > 0 else float(num)


def first_overflow_code(r: int) -> int:
    """Smallest 8-bit code whose r-bit slice rounds up to 2^r (errata section: q / 2^(8-r) + 1/2 >= 2^r),
    i.e. 256 - 2^(8-r)/2.  Used only to plant test inputs; the expected values come from the oracle."""
    return 256 - (1 << (8 - r)) // 2
