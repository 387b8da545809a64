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


def assert_close(got, want, c_rms=2.0 ** -7, tol=1e-2, what="", extra=None):
    """The two bars of a floating-point output against the fp64 oracle: rel-L2 <= tol over the tensor AND, for
    every element, |got - want| <= 2^-7 |want| + c_rms * rms(want) (+ extra).

    The first term of the element bar is one bf16 step of the value (the output is rounded once to bf16 and a
    tiny difference before the rounding may pick the neighbouring bf16 number); the second covers what is
    absolute rather than relative: the cancellation of the zero-point term and, in the backward, the bf16
    rounding of the scaled gradient operands (independent relative errors of at most 2^-9 per term, i.e. about
    2^-9.5 * rms per output: c_rms = 2^-6 is five standard deviations).  `extra` (a scalar or an array like
    `want`) is a further absolute allowance that the caller derives from the arithmetic of the case, e.g.
    accumulation_allowance() below for long contractions.  A wrong element (a dropped term, a tile that was
    skipped or written twice) is off by about rms(want) and fails the bar by far.
    """
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return 0.0
    err = rel_l2(got, want)
    assert err <= tol, (what, "rel-L2", err)
    rms = float(np.sqrt(np.mean(want * want)))
    diff = np.abs(got - want)
    bar = 2.0 ** -7 * np.abs(want) + c_rms * rms
    if extra is not None:
        bar = bar + extra
    bad = diff > bar
    if bad.any():
        at = np.unravel_index(int(np.argmax(diff - bar)), want.shape)
        raise AssertionError((what, "elements beyond the bar", int(bad.sum()), "of", want.size, "worst at", at,
                              float(got[at]), float(want[at]), "rms", rms, "bar", float(np.broadcast_to(bar, want.shape)[at])))
    return err


def accumulation_allowance(L: int, operand_rms, code_scale):
    """Absolute error that fp32 accumulation on the matrix core may add to an output of the quantized layer,
    as a function of the contraction length L.

    The kernels contract the activations (or scaled gradients) with 128 + code, a bf16 number that holds the
    code exactly, and remove the 128 in the epilogue; r = 8 contracts with the code itself, which is centred
    on z = about 128 just the same.  The running sum therefore has the magnitude of 136 * |sum of the operand so
    far| <= about 136 * 3 sqrt(L) * operand_rms, and each of the L / 16 sequential additions into it may be off by
    one fp32 step of that magnitude (2^-24 relative).  In output units (code_scale = alpha_n 2^s, times lambda for
    gradients) that is

        (L / 16) * 2^-24 * 136 * 3 sqrt(L) * operand_rms * code_scale

    with all roundings taken in the same direction: 0.006 code steps at L = 256, 0.33 at L = 3584, 2.6 at L = 14336, 11 at L = 36864
    (where the useful sum itself is about sigma_code * 192 code steps)."""
    return (L / 16.0) * 2.0 ** -24 * 136.0 * 3.0 * np.sqrt(float(L)) * operand_rms * np.asarray(code_scale, np.float64)
