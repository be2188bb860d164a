"""Shared test helpers: bf16 decoding and error norms."""
import numpy as np


def bf16_to_f64(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def rel_max_err(got, ref):
    """max|got-ref| / max|ref| over the whole tensor (the spec norm); NaN/Inf count as failure."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if not np.all(np.isfinite(got)):
        return float("inf")
    den = np.max(np.abs(ref)) if ref.size else 0.0
    num = np.max(np.abs(got - ref)) if ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


from oracle.subproblem import expert_subproblem, token_subproblem  # noqa: E402,F401  (re-exported for the tests)
