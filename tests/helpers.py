"""Shared test helpers: bf16 decoding, error norms, sub-problem extraction (pure indexing)."""
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


def token_subproblem(sel_tokens, x, w, idx, W1, W3, W2, dY=None):
    """Restrict a problem to some tokens and relabel the experts they touch to 0..E'-1.

    Tokens are independent in y and dX, and the layer is invariant under relabelling experts, so the
    oracle's y / dX on the returned problem are the full problem's rows ``sel_tokens``.
    Weight tensors may be numpy arrays or anything indexable by an integer list along axis 0 whose
    result converts with np.asarray (so a caller can hand in lazily fetched slices).
    """
    sel_tokens = np.asarray(sel_tokens, dtype=np.int64)
    sub_idx = idx[sel_tokens]
    used = np.unique(sub_idx)
    remap = -np.ones(int(idx.max()) + 1 if idx.size else 1, dtype=np.int64)
    remap[used] = np.arange(used.size)
    out = dict(x=x[sel_tokens], w=w[sel_tokens], idx=remap[sub_idx].astype(np.int32), W1=W1[used], W3=W3[used],
               W2=W2[used], experts=used)
    if dY is not None:
        out["dY"] = dY[sel_tokens]
    return out


def expert_subproblem(e, x, w, idx, W1, W3, W2, dY):
    """All (token, slot) pairs routed to expert e as a top-1, single-expert problem.

    dW of expert e depends only on those pairs, so the oracle's dW on the returned problem is the full
    problem's dW[e].  Rows keep ascending slot order.
    """
    k = idx.shape[1]
    flat = np.flatnonzero(idx.reshape(-1) == e)
    tok = flat // k
    return dict(x=x[tok], w=w.reshape(-1)[flat].reshape(-1, 1), idx=np.zeros((flat.size, 1), dtype=np.int32),
                W1=W1[e:e + 1], W3=W3[e:e + 1], W2=W2[e:e + 1], dY=dY[tok], slots=flat)
