"""Sub-problem extraction for checking full-size runs against the oracle - TEST INFRASTRUCTURE ONLY.

Pure indexing, no arithmetic.  Tokens are independent in y and dX, the layer is invariant under
relabelling experts, and dW of one expert depends only on the (token, slot) pairs routed to it; so the
oracle evaluated on these reduced problems returns exactly the corresponding pieces of the full problem.
"""
import numpy as np


def token_subproblem(sel_tokens, x, w, idx, W1, W3, W2, dY=None):
    """Restrict a problem to some tokens and relabel the experts they touch to 0..E'-1.

    Weight tensors may be numpy arrays or anything indexable by an integer array along axis 0 whose
    result is a numpy array (so a caller can hand in lazily fetched expert slabs).
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
    """All (token, slot) pairs routed to expert e as a top-1, single-expert problem (rows in ascending slot order)."""
    k = idx.shape[1]
    flat = np.flatnonzero(idx.reshape(-1) == e)
    tok = flat // k
    return dict(x=x[tok], w=w.reshape(-1)[flat].reshape(-1, 1), idx=np.zeros((flat.size, 1), dtype=np.int32),
                W1=W1[e:e + 1], W3=W3[e:e + 1], W2=W2[e:e + 1], dY=dY[tok], slots=flat)
